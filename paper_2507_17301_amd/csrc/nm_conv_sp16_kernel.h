// bf16 convolution without a gather: the activations stay dense in LDS and the
// N:M selection happens inside the matrix core.
//
// gfx950 has sparse matrix instructions (v_smfmac_f32_16x16x64_bf16): operand A
// holds, for every aligned group of 4 positions along K, two values and their
// 2-bit positions; operand B is dense.  A column-wise pruned tile (section 3.1:
// all rows of a tile keep the same columns) is a special case of that format
// whenever no aligned group of 4 columns keeps more than two of them, which
// holds for every N:M with N <= 2 and M a multiple of 4 -- 2:4 in particular.
// Groups that keep fewer than two columns are padded with a zero weight.
// The contraction then reads the im2col strip exactly as it was staged
// ([pixel][channel], 16 consecutive channels per lane, two 16-byte LDS reads
// per 16-pixel block) and never forms the compacted data matrix of Alg. 1 at
// all: the index array of the compressed format becomes the instruction's
// index operand.
//
// SPARSE = false is the same kernel on the zero-filled dense weights with the
// dense v_mfma_f32_16x16x32_bf16 (two per 64 channels): it serves N = M layers
// and the patterns the sparse operand cannot express (e.g. 4:8).
//
// Lane layouts (measured on the device, one-hot operands):
//   B (both instructions): lane n + 16 qb holds, for pixel n, 16 channels of the
//     64-channel k-step; this kernel gives lane group qb the channels
//     16 qb .. 16 qb + 15, elements 0-7 first.
//   sparse A: lane i + 16 qa (row i) element ea pairs with B lane group
//     2 (qa % 2) + ea / 4, elements 8 (qa / 2) + 4 ((ea % 4) / 2) + position,
//     where position is the 2-bit field number ea of the lane's own index
//     operand (bits 2 ea + 1 .. 2 ea of its low half, ABID = 0).
//   dense A: lane i + 16 q element e pairs with B lane group q element e.
//   D: lane n + 16 q register r is row 4 q + r, column n.
//
// F8 = true is the same staging, ring and barriers for E4M3 tensors (one byte per element,
// bf16 output): a k-step is again 64 channels, now 64 bytes of a pixel's row, so lane group q's
// share is one 16-byte read (channels 16 q .. 16 q + 15) that feeds two dense
// v_mfma_f32_16x16x32_fp8_fp8 -- bytes 0-7 the first, bytes 8-15 the second; operands are 8 bytes per
// lane, lane i + 16 q holding K positions 8 q .. 8 q + 7, and which channel a K position stands
// for is free as long as both operands agree -- against weights that nm_prune lays out to match.
// With chunks of 128 channels or more, two k-steps go into one v_mfma_f32_16x16x128_f8f6f4 (both
// operands 32 bytes per lane: the two k-steps' 16 bytes, same pairing of lane group and byte on
// both sides; checked on the device against a plain product): twice the rate of the 32-deep
// instruction, which is what the late layers' K loops are bound by.
// The accumulators start from zero and are scaled back by the layer's weight scale before the
// bias is added.
#pragma once

#include "nm_conv_kernel.h"

namespace nm {

typedef __bf16 bf8x __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x __attribute__((ext_vector_type(16)));

// The strip goes from global memory straight into LDS (buffer loads with the
// LDS modifier, 16 bytes per lane): lane L of a wave-wide load writes the 16-byte
// granule L of a 1 KB window, so a stage is the plain [pixel][CK channels] array
// and the lane decides which (pixel, octet) it fetches.  To keep the 16-byte
// operand reads of 16 pixels conflict-free without padding, octet g of pixel
// row r is stored at granule position g ^ swz(r) of the row.
// Out-of-image taps are fetched with an out-of-range offset, which writes zeros.
// The weights and index words of a chunk travel the same way into a per-wave
// part of the stage.  Three stages form a ring: while chunk c is contracted,
// the loads of chunks c + 1 and c + 2 are in flight; no global load returns
// into registers inside the loop.
constexpr int kSp16Stages = 3;
// one stage: the strip [BP][CK] bf16, then per wave the weights (and index words) of its row blocks
// (fp8: rows of CK bytes, one 16-byte weight operand per k-step and row block)
constexpr int sp16_stage_bytes(int BP, int CK, int NJ, bool sparse, bool areg = false, bool f8 = false)
{
    return BP * CK * (f8 ? 1 : 2) +
           (areg ? 0 : 4 * NJ * (CK / 64) * ((sparse || f8 ? 1 : 2) * 1024 + (sparse ? 256 : 0)));
}
// (8 consecutive lanes of a 16-byte LDS read are served together: their granules must differ
// modulo 128 bytes; the extra bit keeps rows r and r + 8 apart modulo 256 bytes as well.
// RB = bytes per pixel row: with 64-byte rows two rows share 128 bytes, so the row's parity
// already separates them and the other bits of the row number pick the granule.)
__device__ inline int sp16_swz(int row, int RB)
{
    return RB == 64 ? ((row >> 1) & 3) : RB == 128 ? ((row & 7) ^ ((row >> 3) & 1)) : (row & 15);
}
// two 16-byte operands side by side, as the 128-deep fp8 matrix instruction takes them
typedef int i8v __attribute__((ext_vector_type(8)));
__device__ inline i8v sp16_pair(const u4v& lo, const u4v& hi)
{
    return i8v{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}
// one 8-byte half of a 16-byte operand, as the fp8 matrix instruction takes it
__device__ inline long sp16_half(const u4v& v, int h)
{
    const unsigned long long lo = h ? v.z : v.x, hi = h ? v.w : v.y;
    return (long)(lo | (hi << 32));
}

// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt in
// bits 3:0 and 15:14, the other counters at their maxima).
#define NM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0f70)

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// s_waitcnt on the LDS counter that also tells the compiler that the BH registers of one
// strip read (R) are defined from here on (used inside the kernel, where BH is known)
#define NM_SP16_WAIT(N, R)                                                               \
    do {                                                                                 \
        if constexpr (BH == 2)                                                           \
            asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"((R)[0]), "+v"((R)[BH - 1])); \
        else                                                                             \
            asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"((R)[0]));                    \
    } while (0)

//
// SPEC = true adds four producer wavefronts to the workgroup (512 threads): they issue every
// load of the ring and nothing else, the other four contract and never touch global memory
// until the epilogue.  A wave-wide load into LDS occupies the CU's memory path for 16 clocks
// and stalls its wavefront while the path is backed up, so a wavefront that does both jobs
// alternates between them; split, the two overlap.  Both roles execute the same barriers.
//
// AREG = true (only with SPEC): the weights and index words do not pass through LDS.  Each
// contracting wavefront loads the operands of its own row blocks straight into registers,
// one chunk ahead (they are laid out in lane order by nm_prune, so these are plain
// coalesced 16-byte loads, and the compiler counts them itself: a contracting wavefront
// issues no other vector-memory load inside the loop).  A stage is then the strip alone,
// which halves the LDS traffic of tiles whose wavefronts hold four row blocks, and the
// strip reads run four deep instead of two.
template <int NBLK, int WP, int NJ, int CK, bool SPARSE, bool SPEC, bool AREG = false, bool F8 = false>
__global__ __launch_bounds__(SPEC ? 512 : 256) void nm_conv_sp16_kernel(const ConvParams p)
{
    static_assert(!AREG || SPEC, "register operands need the producer wavefronts");
    static_assert(!F8 || !SPARSE, "the fp8 form runs the dense instruction");
    constexpr int ES = F8 ? 1 : 2;               // bytes per element of x and of the weights
    constexpr int BPW = 16 * NBLK;
    constexpr int BP = BPW * WP;
    constexpr int WC = 4 / WP;
    constexpr bool F8X = F8 && CK % 128 == 0;    // fp8 with 128-channel k-steps (one 128-deep instruction each)
    constexpr int KS = F8X ? CK / 128 : CK / 64; // k-steps (64 channels; 128 for F8X) per chunk
    constexpr int AH = (SPARSE || (F8 && !F8X)) ? 1 : 2;   // 16-byte A operands per k-step and row block
    constexpr int BH = (F8 && !F8X) ? 1 : 2;     // 16-byte strip reads per k-step and pixel block
    constexpr int RB = CK * ES;                  // bytes per pixel row of a stage
    const int D = p.nchunks < kSp16Stages ? p.nchunks : kSp16Stages;   // stages in use (and allocated)
    constexpr int STAGE = sp16_stage_bytes(BP, CK, NJ, SPARSE, AREG, F8);
    static_assert(CK % 64 == 0, "a chunk is a whole number of 64-channel k-steps");

    extern __shared__ __attribute__((aligned(16))) char lds8[];   // [D][BP][RB]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);   // 0..3; 4..7 are the producers
    const bool producer = SPEC && wave_id >= 4;
    const int wave = SPEC ? (wave_id & 3) : wave_id;                // position among the four of its role
    const int q = lane >> 4;
    const int n = lane & 15;

    const int bid = blockIdx.x;
    const int logical = (bid & 7) * p.wg_per_xcd + (bid >> 3);
    if (logical >= p.n_wg) return;
    const int cblock = logical % p.n_cblocks;
    const int ptile = logical / p.n_cblocks;
    const int p0 = ptile * BP;
    const int wpx = wave % WP, wcx = wave / WP;
    const int rb0 = (cblock * WC + wcx) * NJ;
    const int wpix = wpx * BPW;

    const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.x, p.x_bytes);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wfrag, p.wfrag_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.rows, p.rows_bytes);

    // ---- staging: wave-wide loads of 64 granules; load i of the stage covers
    // granules 64 i .. 64 i + 63 and is issued by wave i % 4 -------------------
    constexpr int OPR = RB / 16;                 // 16-byte granules per pixel row
    constexpr int EPG = 16 / ES;                 // elements per granule
    constexpr int NW = BP * OPR / 64;            // wave-wide loads per stage
    constexpr int NIT = (NW + 3) / 4;            // per wave
    int hi0[NIT], wi0[NIT];
    unsigned base[NIT], voff[NIT];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int G = (wave + 4 * it) * 64 + lane;            // granule of the stage this lane fills
        const int pl = G / OPR;
        const int oct = (G % OPR) ^ sp16_swz(pl, RB);         // the granule of the row that belongs at that position
        const int pp = p0 + pl;
        const bool live = (pp < p.P) & (pl < BP);
        const int b = (int)fdiv((unsigned)pp, p.howo_mul, p.howo_shift);
        const int rem = pp - b * HoWo;
        const int ho = (int)fdiv((unsigned)rem, p.wo_mul, p.wo_shift);
        const int wo = rem - ho * p.Wo;
        const int h0 = ho * p.sh - p.ph, w0 = wo * p.sw - p.pw;
        hi0[it] = live ? h0 : -(1 << 28);   // a dead pixel has every tap outside the image
        wi0[it] = w0;
        base[it] = (unsigned)(((b * p.H + h0) * p.W + w0) * p.Cin + oct * EPG) * ES;
    }
    int f_c = 0, f_kh = 0, f_kw = 0, f_ci0 = 0;
    bool f_live = true;                          // false once the iterator has run past the last chunk
    auto retap = [&]() {
        const int dhh = f_kh * p.dh, dww = f_kw * p.dw;
        const unsigned tapoff = (unsigned)((dhh * p.W + dww) * p.Cin) * ES;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int hi = hi0[it] + dhh, wi = wi0[it] + dww;
            const bool inb = ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            voff[it] = inb ? base[it] + tapoff : kOOB;
        }
    };
    // one wave-wide load of the current fetch chunk into stage `stage`
    auto fetch_item = [&](int it, int stage) {
        if (NW % 4 != 0 && wave + 4 * it >= NW) return;       // wave-uniform
        const unsigned off = f_live ? voff[it] + (unsigned)(f_ci0 * ES) : kOOB;
        char* dst = lds8 + stage * STAGE + (wave + 4 * it) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (lds_ptr_t)dst, 16, off, 0, 0, 0);
    };
    auto fetch_advance = [&]() {
        const bool adv = f_c + 1 < p.nchunks;
        f_live = f_live & adv;
        f_c += adv ? 1 : 0;
        const int nci = f_ci0 + CK;
        const bool wrap = adv & (nci >= p.Cin);
        f_ci0 = wrap ? 0 : (adv ? nci : f_ci0);
        if (wrap) {
            const int nkw = f_kw + 1;
            const bool wrap2 = nkw == p.Kw;
            f_kw = wrap2 ? 0 : nkw;
            f_kh += wrap2 ? 1 : 0;
            retap();
        }
    };

    // ---- operand streams ------------------------------------------------------
    // weights: [row block][chunk][k-step][AH][lane] x 16 bytes (8 bf16, or 16 E4M3)
    // index operands (sparse): [column tile][chunk][lane group][k-step] x 4 bytes
    // Both take the same road as the strip: each wave loads the operands of its
    // own row blocks into a private part of the stage (lane L's 16 bytes, or 4
    // for the index word, land at position L) and reads them back when the
    // chunk's turn comes.
    constexpr unsigned WCH = KS * AH * 1024;     // weight bytes per (row block, chunk)
    constexpr unsigned ICH = KS * 16;            // index bytes per (tile, chunk)
    constexpr int AW = NJ * KS * (AH * 1024 + (SPARSE ? 256 : 0));   // operand bytes per wave and stage
    constexpr int NOPS = AREG ? 0 : NJ * KS * (AH + (SPARSE ? 1 : 0));   // operand loads (into LDS) per wave and stage
    constexpr int NL = NIT + NOPS;                                   // loads per wave and stage
    static_assert(NL <= 63, "a stage's loads must fit the memory counter");
    const unsigned wvoff = (unsigned)lane * 16;
    unsigned wsoff[NJ], isoff[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;
        wsoff[jj] = (unsigned)rb * p.nchunks * WCH;
        isoff[jj] = (unsigned)(rb / p.rbpt) * p.nchunks * ICH;
    }
    int o_c = 0;                                 // chunk whose operands the next fetch_ops brings in
    auto fetch_ops = [&](int stage) {
        char* dst = lds8 + stage * STAGE + BP * RB + wave * AW;
        const int c = o_c < p.nchunks ? o_c : p.nchunks - 1;   // past the end: any valid chunk, never used
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int h = 0; h < AH; ++h) {
                    const unsigned vo = wvoff + wsoff[jj] + (unsigned)c * WCH + (unsigned)(s * AH + h) * 1024;
                    char* d = dst + ((jj * KS + s) * AH + h) * 1024;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (lds_ptr_t)d, 16, vo, 0, 0, 0);
                }
                if constexpr (SPARSE) {
                    const unsigned vo = (unsigned)(q * KS + s) * 4 + isoff[jj] + (unsigned)c * ICH;
                    char* d = dst + NJ * KS * AH * 1024 + (jj * KS + s) * 256;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rr, (lds_ptr_t)d, 4, vo, 0, 0, 0);
                }
            }
        ++o_c;
    };

    // this lane's operand granules inside block 0 of a stage: k-step s, half h
    // (bf16: granules 2 q and 2 q + 1 of the k-step's eight; fp8: granule q of its four, and for
    // 128-channel k-steps granule q of either half)
    unsigned roff[KS][BH];
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int h = 0; h < BH; ++h)
            roff[s][h] = (unsigned)((wpix + n) * RB +
                                    (((F8X ? (2 * s + h) * 4 + q : F8 ? s * 4 + q : s * 8 + q * 2 + h) ^ sp16_swz(n, RB)) * 16));

    // The memory counter retires loads in order, so "at most one stage's loads
    // outstanding" means that the stage before it has landed.
    //   prologue:    stage(0) stage(1)
    //   iteration c: wait, barrier | issue stage(c + 2) | contract chunk c
    auto fetch_stage = [&](int stage) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) fetch_item(it, stage);
        fetch_advance();
        if constexpr (!AREG) fetch_ops(stage);
    };
    // bias of this lane's rows, requested first: the accumulators start from it
    const bool fast = (p.tile % 4 == 0) && (p.Cout % 4 == 0);
    f4 bb[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        bb[jj] = f4{0.f, 0.f, 0.f, 0.f};
        const int rb = rb0 + jj;
        const int j = rb / p.rbpt;
        const int rit = (rb - j * p.rbpt) * 16 + q * 4;
        const int co = j * p.tile + rit;
        if (fast && p.bias && rb < p.n_rowblocks && rit < p.tile && co < p.Cout)
            bb[jj] = *reinterpret_cast<const f4*>(p.bias + co);
    }
    constexpr int WGC = WC * NJ * 16;            // output channels of the workgroup
    // whole 128-byte lines through an LDS tile (two more barriers), or stores straight from the accumulators
    const bool tile_path = WGC * 2 >= 128 && fast && tile_out_ok<bf16_t>(p);
    if (!SPEC || producer) {
        retap();
        fetch_stage(0);
        if (p.nchunks > 1) fetch_stage(1);
    }
    if constexpr (SPEC) {
        if (producer) {
            // the producer's whole life: per chunk, wait until its own loads of that chunk have
            // landed, meet the consumers at the barrier, then refill the stage they have just left
            const bool short_w = (NW % 4 != 0) && (wave + 4 * (NIT - 1) >= NW);
            int wst = D - 1;
            for (int c = 0; c < p.nchunks; ++c) {
                if (c + 1 < p.nchunks) {
                    if (short_w) NM_WAIT_VMCNT(NL - 1); else NM_WAIT_VMCNT(NL);
                } else {
                    NM_WAIT_VMCNT(0);
                }
                __builtin_amdgcn_s_barrier();
                if (c + 2 < p.nchunks) fetch_stage(wst);
                wst = wst + 1 == D ? 0 : wst + 1;
            }
            if (tile_path) {   // the consumers' two epilogue barriers
                __syncthreads();
                __syncthreads();
            }
            return;
        }
    }

    // the accumulators start from the bias (zero where there is none or rows are handled one by one;
    // fp8: from zero, the bias joins after the accumulator is back at the weights' scale)
    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = F8 ? f4{0.f, 0.f, 0.f, 0.f} : bb[jj];

    constexpr int NM = KS * NBLK;                // B operands (LDS reads) per chunk for this wavefront
    static_assert((NBLK - 1) * 16 * RB < 65536, "block offsets must fit the LDS instruction's immediate");
    static_assert(AW < 65536, "operand offsets must fit the LDS instruction's immediate");
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds8;
    const unsigned aoff = (unsigned)(BP * RB + wave * AW) + wvoff;            // this lane's weights in a stage
    const unsigned ioff = (unsigned)(BP * RB + wave * AW + NJ * KS * AH * 1024) + (unsigned)lane * 4;
    // a wave whose last strip load does not exist has one load less per stage
    const bool short_wave = (NW % 4 != 0) && (wave + 4 * (NIT - 1) >= NW);
    int rstage = 0, wstage = D - 1;              // stage read by this chunk / filled for chunk c + 2

    // All LDS reads are inline assembly with hand-placed waits: the compiler,
    // which cannot tell the stages of the ring apart, would otherwise make
    // every LDS read wait for the loads just issued into the other stages.
    auto chunk = [&](int c) {
        // all of this wave's loads for chunk c have landed once at most the next
        // stage's loads (if there is a next chunk) are outstanding
        if constexpr (!SPEC) {
            if (c + 1 < p.nchunks) {
                if (short_wave) NM_WAIT_VMCNT(NL - 1); else NM_WAIT_VMCNT(NL);
            } else {
                NM_WAIT_VMCNT(0);
            }
        }
        // A bare barrier: the fences of __syncthreads() would wait for every load
        // into LDS that is in flight, i.e. for the stages being filled ahead.  What
        // must be ordered is ordered by hand: this wave's loads for chunk c have
        // landed (the wait above), and its LDS reads of chunk c - 1 have returned
        // (each was waited for before the matrix instruction that used it).
        __builtin_amdgcn_s_barrier();
        if constexpr (!SPEC) {
            if (c + 2 < p.nchunks) fetch_stage(wstage);
        }

        const unsigned sbase = lds0 + (unsigned)(rstage * STAGE);
        u4v a[NJ][KS][AH];
        unsigned idx[NJ][KS];
        {
            const unsigned aa = sbase + aoff, ia = sbase + ioff;
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
                for (int s = 0; s < KS; ++s) {
#pragma unroll
                    for (int h = 0; h < AH; ++h)
                        asm volatile("ds_read_b128 %0, %1 offset:%2"
                                     : "=v"(a[jj][s][h]) : "v"(aa), "n"(((jj * KS + s) * AH + h) * 1024) : "memory");
                    if constexpr (SPARSE)
                        asm volatile("ds_read_b32 %0, %1 offset:%2"
                                     : "=v"(idx[jj][s]) : "v"(ia), "n"((jj * KS + s) * 256) : "memory");
                }
        }
        unsigned raddr[KS][BH];
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int h = 0; h < BH; ++h) raddr[s][h] = sbase + roff[s][h];
        auto read_b = [&](int m, u4v (&dst)[BH]) {
            const int s = m / NBLK, b = m % NBLK;
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst[0]) : "v"(raddr[s][0]), "n"(b * 16 * RB) : "memory");
            if constexpr (BH == 2)
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst[BH - 1]) : "v"(raddr[s][BH - 1]), "n"(b * 16 * RB) : "memory");
        };
        u4v ring[2][BH];
        read_b(0, ring[0]);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const int s = m / NBLK, b = m % NBLK;
            if (m + 1 < NM) {   // the next read is in flight (BH instructions); this one must be back
                read_b(m + 1, ring[(m + 1) & 1]);
                if constexpr (BH == 2) NM_SP16_WAIT(2, ring[m & 1]); else NM_SP16_WAIT(1, ring[m & 1]);
            } else {
                NM_SP16_WAIT(0, ring[m & 1]);
            }
            if (m == 0) {
                // the operands were requested before the first strip read, so the wait
                // above covers them too; tell the compiler that they are defined here
#pragma unroll
                for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
                    for (int s2 = 0; s2 < KS; ++s2) {
#pragma unroll
                        for (int h = 0; h < AH; ++h) asm volatile("" : "+v"(a[jj][s2][h]));
                        if constexpr (SPARSE) asm volatile("" : "+v"(idx[jj][s2]));
                    }
            }
            const u4v(&bo)[BH] = ring[m & 1];
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj) {
                if constexpr (SPARSE) {
                    const bf16x bv = __builtin_shufflevector(__builtin_bit_cast(bf8x, bo[0]),
                                                             __builtin_bit_cast(bf8x, bo[BH - 1]), 0, 1, 2, 3, 4,
                                                             5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                    acc[jj][b] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(
                        __builtin_bit_cast(bf8x, a[jj][s][0]), bv, acc[jj][b], (int)idx[jj][s], 0, 0);
                } else if constexpr (F8X) {
                    acc[jj][b] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        sp16_pair(a[jj][s][0], a[jj][s][AH - 1]), sp16_pair(bo[0], bo[BH - 1]), acc[jj][b], 0, 0, 0, 0, 0, 0);
                } else if constexpr (F8) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(
                            sp16_half(a[jj][s][0], h), sp16_half(bo[0], h), acc[jj][b], 0, 0, 0);
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf8x, a[jj][s][h]), __builtin_bit_cast(bf8x, bo[h]),
                            acc[jj][b], 0, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        rstage = rstage + 1 == D ? 0 : rstage + 1;
        wstage = wstage + 1 == D ? 0 : wstage + 1;
    };

    if constexpr (AREG) {
        // ---- operands in registers, two sets, one chunk ahead ------------------------
        struct Ops {
            u4v a[NJ][KS][AH];
            unsigned idx[NJ][KS];
        };
        auto load_ops = [&](Ops& o, int c) {
            const int cc = c < p.nchunks ? c : p.nchunks - 1;   // past the end: a valid chunk, never used
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
                for (int s2 = 0; s2 < KS; ++s2) {
#pragma unroll
                    for (int h = 0; h < AH; ++h)
                        o.a[jj][s2][h] = __builtin_amdgcn_raw_buffer_load_b128(
                            wr, wvoff + wsoff[jj] + (unsigned)cc * WCH + (unsigned)(s2 * AH + h) * 1024, 0, 0);
                    if constexpr (SPARSE)
                        o.idx[jj][s2] = __builtin_amdgcn_raw_buffer_load_b32(
                            rr, (unsigned)(q * KS + s2) * 4 + isoff[jj] + (unsigned)cc * ICH, 0, 0);
                }
        };
        constexpr int RD = NM < 4 ? NM : 4;          // strip reads in flight
        auto chunk_r = [&](const Ops& o) {
            __builtin_amdgcn_s_barrier();            // the producers' loads of this chunk have landed
            const unsigned sbase = lds0 + (unsigned)(rstage * STAGE);
            unsigned raddr[KS][BH];
#pragma unroll
            for (int s2 = 0; s2 < KS; ++s2)
#pragma unroll
                for (int h = 0; h < BH; ++h) raddr[s2][h] = sbase + roff[s2][h];
            auto read_b = [&](int m, u4v (&dst)[BH]) {
                const int s2 = m / NBLK, b = m % NBLK;
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst[0]) : "v"(raddr[s2][0]), "n"(b * 16 * RB) : "memory");
                if constexpr (BH == 2)
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst[BH - 1]) : "v"(raddr[s2][BH - 1]), "n"(b * 16 * RB) : "memory");
            };
            u4v ring[RD][BH];
#pragma unroll
            for (int m = 0; m < RD - 1; ++m) read_b(m, ring[m]);
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int s2 = m / NBLK, b = m % NBLK;
                if (m + RD - 1 < NM) read_b(m + RD - 1, ring[(m + RD - 1) % RD]);
                // reads m .. min(m + RD, NM) - 1 are outstanding, BH instructions each; the oldest must be back
                const int later = ((m + RD - 1 < NM ? RD : NM - m) - 1) * BH;
                if (later == 6) NM_SP16_WAIT(6, ring[m % RD]);
                else if (later == 4) NM_SP16_WAIT(4, ring[m % RD]);
                else if (later == 3) NM_SP16_WAIT(3, ring[m % RD]);
                else if (later == 2) NM_SP16_WAIT(2, ring[m % RD]);
                else if (later == 1) NM_SP16_WAIT(1, ring[m % RD]);
                else NM_SP16_WAIT(0, ring[m % RD]);
                const u4v(&bo)[BH] = ring[m % RD];
#pragma unroll
                for (int jj = 0; jj < NJ; ++jj) {
                    if constexpr (SPARSE) {
                        const bf16x bv = __builtin_shufflevector(__builtin_bit_cast(bf8x, bo[0]),
                                                                 __builtin_bit_cast(bf8x, bo[BH - 1]), 0, 1, 2, 3, 4,
                                                                 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                        acc[jj][b] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(
                            __builtin_bit_cast(bf8x, o.a[jj][s2][0]), bv, acc[jj][b], (int)o.idx[jj][s2], 0, 0);
                    } else if constexpr (F8X) {
                        acc[jj][b] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                            sp16_pair(o.a[jj][s2][0], o.a[jj][s2][AH - 1]), sp16_pair(bo[0], bo[BH - 1]), acc[jj][b], 0, 0, 0, 0, 0, 0);
                    } else if constexpr (F8) {
#pragma unroll
                        for (int h = 0; h < 2; ++h)
                            acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(
                                sp16_half(o.a[jj][s2][0], h), sp16_half(bo[0], h), acc[jj][b], 0, 0, 0);
                    } else {
#pragma unroll
                        for (int h = 0; h < 2; ++h)
                            acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf8x, o.a[jj][s2][h]), __builtin_bit_cast(bf8x, bo[h]),
                                acc[jj][b], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            rstage = rstage + 1 == D ? 0 : rstage + 1;
        };
        Ops oa, ob;
        load_ops(oa, 0);
        int c = 0;
        for (; c + 1 < p.nchunks; c += 2) {
            load_ops(ob, c + 1);
            chunk_r(oa);
            load_ops(oa, c + 2);
            chunk_r(ob);
        }
        if (c < p.nchunks) chunk_r(oa);
    } else {
        for (int c = 0; c < p.nchunks; ++c) chunk(c);
    }

    // ---- epilogue: bias, ReLU, round to bf16, NHWC store ------------------------
    bf16_t* __restrict__ y = reinterpret_cast<bf16_t*>(p.y);
    if (tile_path) {
        // whole 128-byte lines through the LDS tile, once every wavefront is past its last strip read
        constexpr int PITCH = tile_pitch<bf16_t>(WGC);
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int rb = rb0 + jj;
            const int co = rb * 16 + q * 4;       // T is a multiple of 16: row block rb is channels 16 rb ..
            const bool row_live = rb < p.n_rowblocks && co < p.Cout;
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pl = wpix + b * 16 + n;
                const int pp = p0 + pl;
                // (bf16: the bias is already in the accumulator)
                tile_put4<bf16_t>(p, lds8 + pl * PITCH + ((wcx * NJ + jj) * 16 + q * 4) * 2,
                                  (unsigned)pp * (unsigned)p.Cout + (unsigned)co, row_live && pp < p.P,
                                  F8 ? acc[jj][b] * p.oscale + bb[jj] : acc[jj][b]);
            }
        }
        __syncthreads();
        tile_flush<bf16_t, BP, WGC>(p, lds8, p0, cblock * WGC);
        return;
    }
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        const int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) continue;
        const int j = rb / p.rbpt;
        const int sub = rb - j * p.rbpt;
        const int rit = sub * 16 + q * 4;
        const int co = j * p.tile + rit;
        if (fast) {
            if (rit >= p.tile || co >= p.Cout) continue;
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + b * 16 + n;
                if (pp >= p.P) continue;
                const f4 v = F8 ? acc[jj][b] * p.oscale + bb[jj] : acc[jj][b];   // bf16: the bias is already there
                emit4(p, y, (unsigned)pp * (unsigned)p.Cout + (unsigned)co, v);
            }
        } else {
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + b * 16 + n;
                if (pp >= p.P) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (rit + r >= p.tile || co + r >= p.Cout) continue;
                    float v = (F8 ? acc[jj][b][r] * p.oscale : acc[jj][b][r]) + (p.bias ? p.bias[co + r] : 0.f);
                    emit1(p, y, (unsigned)pp * (unsigned)p.Cout + (unsigned)(co + r), v);
                }
            }
        }
    }
}

template <int NBLK, int WP, int NJ, int CK, bool SPARSE, bool SPEC, bool AREG, bool F8>
int launch_sp16_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_sp16_kernel<NBLK, WP, NJ, CK, SPARSE, SPEC, AREG, F8>;
    constexpr size_t stage = sp16_stage_bytes(16 * NBLK * WP, CK, NJ, SPARSE, AREG, F8);
    if (F8 && (p.tile % 16 != 0 || p.Cout % 8 != 0 || p.Cin % CK != 0)) {
        set_error("internal: the fp8 kernel needs T %% 16 == 0, Cout %% 8 == 0 and whole chunks per tap");
        return NM_ERR_UNSUPPORTED;
    }
    // the most this kernel may ever be launched with: the full ring, or what the CU has
    constexpr size_t ring = kSp16Stages * stage > out_tile_bytes(16 * NBLK * WP, (4 / WP) * NJ * 16, 2)
                                ? kSp16Stages * stage : out_tile_bytes(16 * NBLK * WP, (4 / WP) * NJ * 16, 2);
    constexpr size_t most = ring < 160 * 1024 ? ring : 160 * 1024;
    {
        static unsigned long long done = 0;
        const int rc = allow_lds(reinterpret_cast<const void*>(kern), most, &done);
        if (rc != NM_OK) return rc;
    }
    // short K loops use (and allocate) fewer stages, which leaves room for more workgroups per CU;
    // the epilogue's output tile needs its share too
    constexpr size_t otile = out_tile_bytes(16 * NBLK * WP, (4 / WP) * NJ * 16, 2);
    size_t lds = stage * (size_t)(p.nchunks < kSp16Stages ? p.nchunks : kSp16Stages);
    if (lds < otile) lds = otile;
    if (lds > most) {
        set_error("internal: LDS %zu bytes exceed the CU's 160 KB", lds);
        return NM_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL(kern, dim3(p.wg_per_xcd * 8), dim3(SPEC ? 512 : 256), lds, s, p);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

}  // namespace nm
