// Fused im2col + packing + column-wise N:M contraction + bias/ReLU for gfx950.
//
// One workgroup (4 wavefronts of 64) produces BP = 16*NBLK*WP output pixels x
// (4/WP)*NJ*16 output channels.  The K axis is walked in chunks of CK rows of
// the im2col matrix (paper section 2.2); for each chunk the workgroup gathers
// rows k0..k0+CK-1 of the im2col matrix for its BP pixels straight from the
// NHWC feature map into LDS, laid out [row][pixel] -- the K-by-V strip of the
// paper's data packing (section 3.2, Alg. 2) with V = BP, built in one pass and
// never written to memory.  Each wavefront then contracts its row blocks
// against that strip as Alg. 1 does: for every kept column it reads the data
// row the index points at once and feeds it to all 16 output channels of the
// row block (a 16x16x4 fp32 MFMA covers 16 channels x 16 pixels x 4 kept
// columns).  The index of a kept column is a property of the column tile, so
// it is read once per wavefront quarter and reused for every pixel.
//
// MFMA operand roles (v_mfma_f32_16x16x4_f32, D = A*B + C):
//   A[i][k]  lane i + 16k  = weight of output channel i for kept column k
//   B[k][j]  lane j + 16k  = im2col value of kept column k at pixel j
//   D[i][j]  lane j + 16*(i/4), register i%4
// A wavefront's 16*NBLK pixels are cut into 64-pixel segments read with one
// 16-byte LDS load per lane (pixels 4j..4j+3 feed four MFMAs), then at most one
// 32-pixel piece (8-byte loads) and one 16-pixel piece (4-byte loads).
//
// On this machine every VALU, LDS or memory instruction a wavefront issues
// takes issue time away from its own MFMAs, so the loop is built to keep such
// instructions few: input addresses are per-tap registers plus a scalar,
// operand streams are buffer loads with scalar offsets, row offsets come
// ready-made from the operand table, and the operand registers ping-pong
// between two sets instead of being copied.
#pragma once

#include "nm_launch_decl.h"

namespace nm {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round to nearest even, NaN stays NaN: the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32), two values per instruction
typedef float f2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
__device__ inline unsigned pack_bf16(float lo, float hi)
{
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{lo, hi}, bf2v));
}
__device__ inline unsigned short to_bf16_bits(float v) { return (unsigned short)(pack_bf16(v, 0.f) & 0xffffu); }
__device__ inline void store4(float* p, f4 v) { *reinterpret_cast<f4*>(p) = v; }
__device__ inline void store4(bf16_t* p, f4 v)
{
    uint2 u;
    u.x = pack_bf16(v.x, v.y);
    u.y = pack_bf16(v.z, v.w);
    *reinterpret_cast<uint2*>(p) = u;
}
__device__ inline void store1(float* p, float v) { *p = v; }
__device__ inline void store1(bf16_t* p, float v) { p->v = to_bf16_bits(v); }
__device__ inline f4 load4(const float* p) { return *reinterpret_cast<const f4*>(p); }
__device__ inline f4 load4(const bf16_t* p)
{
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    return f4{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
              __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
}
__device__ inline float load1(const float* p) { return *p; }
__device__ inline float load1(const bf16_t* p) { return __uint_as_float((unsigned)p->v << 16); }

// max(v, 0) as one instruction per value (fmaxf costs a second one that quiets NaNs first;
// the hardware maximum already returns the number when the other operand is a NaN)
__device__ inline float relu1(float v)
{
    float r;
    asm("v_max_f32_e32 %0, 0, %1" : "=v"(r) : "v"(v));
    return r;
}
__device__ inline f4 relu4(f4 v) { return f4{relu1(v.x), relu1(v.y), relu1(v.z), relu1(v.w)}; }

// Tail of every epilogue: optional residual (a tensor shaped like the output,
// added before the activation), ReLU, cast, store.
// (offsets are element counts below 2^31, so 32-bit arithmetic is enough)
template <typename TOUT> __device__ inline void emit4(const ConvParams& p, TOUT* y, unsigned off, f4 v)
{
    if (p.res) v = v + load4(reinterpret_cast<const TOUT*>(p.res) + off);
    if (p.relu) v = relu4(v);
    store4(y + off, v);
}
template <typename TOUT> __device__ inline void emit1(const ConvParams& p, TOUT* y, unsigned off, float v)
{
    if (p.res) v += load1(reinterpret_cast<const TOUT*>(p.res) + off);
    if (p.relu) v = relu1(v);
    store1(y + off, v);
}

// ---- workgroup-wide output tile ---------------------------------------------
// A store straight from the MFMA accumulator layout touches 16 pixels x 32 bytes (bf16)
// or 64 bytes (fp32) per instruction, and streams of such partial-line writes reach
// about two thirds of the memory rate that whole 128-byte lines reach (measured with a
// load-then-store microbenchmark of the same tile sizes).  So where the layer allows
// (T a multiple of 16, 16-byte aligned pixel rows) the workgroup first assembles its
// output tile [pixel][channel] in LDS -- residual, ReLU and the cast applied on the way
// in, one rounding -- and then writes it out 16 bytes per lane with consecutive lanes
// on consecutive bytes of a pixel.  The row pitch is an odd number of 16-byte units.
template <typename TOUT> constexpr int tile_pitch(int wgc) { return wgc * (int)sizeof(TOUT) + 16; }
constexpr size_t out_tile_bytes(int bp, int wgc, int es) { return (size_t)bp * (wgc * es + 16); }

template <typename TOUT> __device__ inline bool tile_out_ok(const ConvParams& p)
{
    return (p.tile % 16 == 0) && ((p.Cout * (int)sizeof(TOUT)) % 16 == 0);
}
// four consecutive channels of one pixel into the tile; `goff` is the element offset of
// the same four values in the output (for the residual), `live` whether they exist
template <typename TOUT>
__device__ inline void tile_put4(const ConvParams& p, char* dst, unsigned goff, bool live, f4 v)
{
    if (p.res && live) v = v + load4(reinterpret_cast<const TOUT*>(p.res) + goff);
    if (p.relu) v = relu4(v);
    store4(reinterpret_cast<TOUT*>(dst), v);
}
// the tile [BP][WGC] (first pixel p0, first channel co0) from LDS to the NHWC output: a thread
// keeps its 16-byte column and walks down the rows, so one compare and one add per store
template <typename TOUT, int BP, int WGC>
__device__ inline void tile_flush(const ConvParams& p, const char* tile, int p0, int co0)
{
    constexpr int CPG = 16 / (int)sizeof(TOUT);      // channels per 16-byte granule
    constexpr int GPR = WGC / CPG;                   // granules per pixel
    constexpr int PITCH = tile_pitch<TOUT>(WGC);
    static_assert(GPR <= 256 && 256 % GPR == 0, "a row's granules divide the workgroup");
    constexpr int RSTEP = 256 / GPR;                 // rows covered by one pass of the workgroup
    constexpr int NG = (BP + RSTEP - 1) / RSTEP;
    const int r0 = (int)threadIdx.x / GPR, cg = (int)threadIdx.x % GPR;
    const int co = co0 + cg * CPG;
    if (co >= p.Cout) return;
    TOUT* __restrict__ y = reinterpret_cast<TOUT*>(p.y) + ((unsigned)(p0 + r0) * (unsigned)p.Cout + (unsigned)co);
    const char* src = tile + r0 * PITCH + cg * 16;
    const int rows_left = p.P - p0 - r0;             // rows r0 + k RSTEP with k RSTEP < rows_left exist
#pragma unroll
    for (int it = 0; it < NG; ++it) {
        if ((BP % RSTEP == 0 || r0 + it * RSTEP < BP) && it * RSTEP < rows_left) {
            const u4v v = *reinterpret_cast<const u4v*>(src + it * (RSTEP * PITCH));
            *reinterpret_cast<u4v*>(y + (unsigned)(it * RSTEP) * (unsigned)p.Cout) = v;
        }
    }
}

// Buffer loads: an offset at or beyond the descriptor's size returns zeros, which
// is how padding, ragged pixel tiles and partial chunks are filled without a branch.
constexpr unsigned kOOB = 0x80000000u;   // beyond any tensor this library accepts (< 2 GiB)

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* ptr, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(ptr), 0, (int)bytes, 0x00020000);
}
__device__ inline f4 buf_load4(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, const float*)
{
    const u4v v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return f4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
}
__device__ inline f4 buf_load4(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, const bf16_t*)
{
    const u2v u = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
    return f4{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
              __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
}
__device__ inline float buf_load1(__amdgpu_buffer_rsrc_t r, unsigned voff, const float*)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, 0, 0));
}
__device__ inline float buf_load1(__amdgpu_buffer_rsrc_t r, unsigned voff, const bf16_t*)
{
    return __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, voff, 0, 0) << 16);
}

// Per-lane operands of one (row block, chunk): SPC weights and, for this lane's
// quarter, the LDS row of each of the SPC k-steps.
template <int SPC> struct StepOps {
    float a[SPC];
    unsigned row[SPC];
};

template <int SPC>
__device__ inline void load_words(unsigned (&dst)[SPC], __amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff)
{
    if constexpr (SPC == 1) {
        dst[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
    } else if constexpr (SPC == 2) {
        const u2v v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        dst[0] = v.x; dst[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < SPC / 4; ++i) {
            const u4v v = __builtin_amdgcn_raw_buffer_load_b128(r, voff + 16 * i, soff, 0);
            dst[4 * i + 0] = v.x; dst[4 * i + 1] = v.y; dst[4 * i + 2] = v.z; dst[4 * i + 3] = v.w;
        }
    }
}

// x / d for a divisor d fixed at launch and x < 2^31: umulhi(2 x, mul) >> shift
// with shift = ceil(log2 d) and mul = floor(2^(31 + shift) / d) + 1.
__device__ inline unsigned fdiv(unsigned x, unsigned mul, unsigned shift)
{
    return __umulhi(x << 1, mul) >> shift;
}

// MODE 0: element-wise staging on the flat k axis; 1: 16-byte channel loads, every chunk
// runs SPC k-steps; 2: as 1, but each (column tile, chunk) runs only the k-steps that
// hold kept columns (their number rides in the upper half of the first row-table word).
template <int NBLK, int WP, int NJ, int CK, int SPC, int MODE, typename TIN, typename TOUT>
__global__ __launch_bounds__(256) void nm_conv_kernel(const ConvParams p)
{
    constexpr bool VEC = MODE != 0;
    constexpr bool VAR = MODE == 2;
    constexpr int BPW = 16 * NBLK;        // pixels per wavefront
    constexpr int BP = BPW * WP;          // pixels per workgroup
    constexpr int SP = strip_stride(BP, CK, VEC);
    constexpr int WC = 4 / WP;            // wavefronts along the row-block axis
    constexpr int ES = (int)sizeof(TIN);
    constexpr int NF = NBLK / 4;          // whole 64-pixel segments of a wavefront
    constexpr int R = NBLK % 4;           // MFMA blocks in the ragged tail: a pair, a single, or both
    constexpr int OFF2 = NF * 64;                     // first pixel of the 32-pixel piece
    constexpr int OFF1 = NF * 64 + (R >= 2 ? 32 : 0); // first pixel of the 16-pixel piece

    extern __shared__ float lds[];        // [2][CK][SP]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4;
    const int n = lane & 15;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // range of logical ids so that the workgroups sharing one pixel tile (they
    // differ only in the row-block group) hit the same L2.
    const int bid = blockIdx.x;
    const int logical = (bid & 7) * p.wg_per_xcd + (bid >> 3);
    if (logical >= p.n_wg) return;
    // K split (p.ksplit > 1): the workgroups of one output tile share the K axis, split
    // `ks` contracts chunks [c_begin, c_end) and leaves its partial sums in p.partial
    const int n_out_tiles = p.n_ptiles * p.n_cblocks;
    const int ks = p.ksplit > 1 ? logical / n_out_tiles : 0;
    const int otile = logical - ks * n_out_tiles;
    const int c_begin = p.ksplit > 1 ? ks * p.cps : 0;
    const int c_end = p.ksplit > 1 ? (c_begin + p.cps < p.nchunks ? c_begin + p.cps : p.nchunks) : p.nchunks;
    const int cblock = otile % p.n_cblocks;
    const int ptile = otile / p.n_cblocks;
    const int p0 = ptile * BP;

    const int wpx = wave % WP;            // position along pixels
    const int wcx = wave / WP;            // position along row blocks
    const int rb0 = (cblock * WC + wcx) * NJ;
    const int wpix = wpx * BPW;

    const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.x, p.x_bytes);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wfrag, p.wfrag_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.rows, p.rows_bytes);
    const TIN* const xtag = nullptr;

    // ---- staging geometry -------------------------------------------------
    // vector mode: item = (pixel, 4-channel quad); a thread keeps the same quad
    // and NIT pixels.  scalar mode: a thread keeps one pixel and walks rows.
    constexpr int QPR = CK / 4;
    constexpr int PSTEP = 256 / QPR;
    constexpr int NIT = VEC ? (BP * QPR + 255) / 256 : 1;
    static_assert(VEC || (256 % BP == 0 || BP % 256 == 0), "scalar staging keeps one pixel per thread");
    constexpr int NITS = VEC ? 1 : (BP * CK) / 256;   // scalar items per thread
    constexpr int NST = VEC ? NIT : NITS;             // staging items per thread and chunk

    const int quad = tid % QPR;
    const int pl0 = VEC ? tid / QPR : tid % BP;
    const int r0s = BP >= 256 ? 0 : __builtin_amdgcn_readfirstlane(tid / BP);
    int hi0[NIT], wi0[NIT];
    unsigned base[NIT];   // byte offset of (b, hi0, wi0, quad*4); wraps for border pixels, only used with valid taps
    unsigned voff[NIT];   // base + current tap, or kOOB when that tap falls outside the image
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int pl = pl0 + it * PSTEP;
        const int pp = p0 + pl;
        const bool live = (pp < p.P) & (pl < BP);
        const int b = (int)fdiv((unsigned)pp, p.howo_mul, p.howo_shift);
        const int rem = pp - b * HoWo;
        const int ho = (int)fdiv((unsigned)rem, p.wo_mul, p.wo_shift);
        const int wo = rem - ho * p.Wo;
        const int h0 = ho * p.sh - p.ph, w0 = wo * p.sw - p.pw;
        hi0[it] = live ? h0 : -(1 << 28);   // a dead pixel has every tap outside the image
        wi0[it] = w0;
        base[it] = (unsigned)(((b * p.H + h0) * p.W + w0) * p.Cin + (VEC ? quad * 4 : 0)) * ES;
    }

    f4 st[VEC ? NIT : 1];
    float sts[VEC ? 1 : NITS];

    // Fetch iterator: the chunk that the next fetch brings in, as (chunk id, tap
    // row, tap column, first channel); it runs two chunks ahead of the
    // contraction and stays on the last chunk once it gets there.
    int f_c = c_begin, f_kh = 0, f_kw = 0, f_ci0 = 0;
    if (VEC && c_begin > 0) {   // a later split starts inside the K axis
        const int tap = c_begin / p.ncpt;
        f_ci0 = (c_begin - tap * p.ncpt) * CK;
        f_kh = tap / p.Kw;
        f_kw = tap - f_kh * p.Kw;
    }
    auto retap = [&]() {   // per-pixel offsets of the tap (f_kh, f_kw)
        const int dhh = f_kh * p.dh, dww = f_kw * p.dw;
        const unsigned tapoff = (unsigned)((dhh * p.W + dww) * p.Cin) * ES;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int hi = hi0[it] + dhh, wi = wi0[it] + dww;
            const bool inb = ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            voff[it] = inb ? base[it] + tapoff : kOOB;
        }
    };
    auto fetch_item = [&](int it) {
        if constexpr (VEC) {
            // the channel offset of the chunk rides in the vector offset so that
            // the range check sees the whole address
            st[it] = buf_load4(xr, voff[it] + (unsigned)(f_ci0 * ES), 0, xtag);
        } else {
            // row r of the chunk is the same for the whole wavefront, so its
            // (tap row, tap column, channel) comes from a table through scalar loads
            const int r = r0s * NITS + it;
            const int k = f_c * CK + r;
            const unsigned e = p.ktab[k];
            const int dhh = (int)(e & 0xffu) * p.dh, dww = (int)((e >> 8) & 0xffu) * p.dw;
            const int ci = (int)(e >> 16);
            const int hi = hi0[0] + dhh, wi = wi0[0] + dww;
            const bool inb = (k < p.K) & ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            const unsigned off = base[0] + (unsigned)((dhh * p.W + dww) * p.Cin + ci) * ES;
            sts[it] = buf_load1(xr, inb ? off : kOOB, xtag);
        }
    };
    auto fetch_advance = [&]() {
        const int adv = f_c + 1 < c_end ? 1 : 0;
        f_c += adv;
        if constexpr (VEC) {
            const int nci = f_ci0 + CK;
            const int wrap = (adv && nci >= p.Cin) ? 1 : 0;
            f_ci0 = wrap ? 0 : (adv ? nci : f_ci0);
            if (wrap) {   // uniform, once per tap
                const int nkw = f_kw + 1;
                const int wrap2 = nkw == p.Kw ? 1 : 0;
                f_kw = wrap2 ? 0 : nkw;
                f_kh += wrap2;
                retap();
            }
        }
    };
    auto stash_value = [&](int it, float* dst, const f4& v4, float v1) {
        if constexpr (VEC) {
            // im2col row 4*quad + j of the chunk lives in LDS row j*QPR + quad: the quads a
            // wavefront writes together are then consecutive rows, which the row stride
            // chosen in strip_stride() spreads over the banks
            float* d = dst + quad * SP + pl0 + it * PSTEP;
            d[0] = v4.x;
            d[QPR * SP] = v4.y;
            d[2 * QPR * SP] = v4.z;
            d[3 * QPR * SP] = v4.w;
        } else {
            dst[(r0s * NITS + it) * SP + pl0] = v1;
        }
    };
    auto stash_item = [&](int it, float* dst) { stash_value(it, dst, st[VEC ? it : 0], sts[VEC ? 0 : it]); };

    // ---- operand streams ----------------------------------------------------
    // A wavefront whose row blocks lie beyond the last one still takes part in
    // staging and barriers; it computes on a clamped row block and stores nothing.
    const unsigned wvoff = (unsigned)lane * SPC * 4;   // lane part of the weight offset
    const unsigned rvoff = (unsigned)q * SPC * 4;      // quarter part of the row-table offset
    unsigned wsoff[NJ], rsoff[NJ];                     // scalar parts at chunk 0
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;
        const int j = rb / p.rbpt;
        wsoff[jj] = (unsigned)rb * p.nchunks * (64 * SPC * 4);
        rsoff[jj] = (unsigned)j * p.nchunks * (4 * SPC * 4);
    }
    auto load_ops = [&](StepOps<SPC>& o, int jj, int c) {
        unsigned w[SPC];
        load_words<SPC>(w, wr, wvoff, wsoff[jj] + (unsigned)c * (64 * SPC * 4));
#pragma unroll
        for (int s = 0; s < SPC; ++s) o.a[s] = __uint_as_float(w[s]);
        load_words<SPC>(o.row, rr, rvoff, rsoff[jj] + (unsigned)c * (4 * SPC * 4));
    };

    StepOps<SPC> opsA[NJ], opsB[NJ];

    // Prologue: bias and operands of chunk 0, then the strips of chunk 0 and of chunk 1
    // into registers, and only then chunk 0 into LDS: the first wait of the workgroup
    // covers one memory round trip, not three.
    const bool bias_first = (p.tile % 4 == 0) && (p.Cout % 4 == 0);   // the accumulators can start from it
    f4 bb0[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        bb0[jj] = f4{0.f, 0.f, 0.f, 0.f};
        const int rb = rb0 + jj;
        const int j = rb / p.rbpt;
        const int rit = (rb - j * p.rbpt) * 16 + q * 4;
        const int co = j * p.tile + rit;
        if (bias_first && p.bias && p.ksplit <= 1 && rb < p.n_rowblocks && rit < p.tile && co < p.Cout)
            bb0[jj] = *reinterpret_cast<const f4*>(p.bias + co);   // (with a K split the bias is added when the partial sums meet)
    }
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) load_ops(opsA[jj], jj, c_begin);
    if constexpr (VEC) retap();
#pragma unroll
    for (int it = 0; it < NST; ++it) fetch_item(it);
    fetch_advance();
    {
        f4 first4[VEC ? NIT : 1];
        float first1[VEC ? 1 : NITS];
#pragma unroll
        for (int it = 0; it < (VEC ? NIT : 1); ++it) first4[it] = st[it];
#pragma unroll
        for (int it = 0; it < (VEC ? 1 : NITS); ++it) first1[it] = sts[it];
#pragma unroll
        for (int it = 0; it < NST; ++it) fetch_item(it);
        fetch_advance();
#pragma unroll
        for (int it = 0; it < NST; ++it) stash_value(it, lds, first4[VEC ? it : 0], first1[VEC ? 0 : it]);
    }
    __syncthreads();

    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = bb0[jj];

    constexpr int TOT = NJ * SPC;          // k-steps per chunk for this wavefront
    constexpr int DEPTH = NBLK <= 4 ? 2 : 1;   // LDS reads run this many k-steps ahead
    constexpr int RING = DEPTH + 1;
    constexpr int NM = TOT * NBLK;         // MFMAs per chunk for this wavefront
    // Staging work of one iteration, cut into tasks that are dealt out behind the
    // MFMAs: load the operands of the next chunk, write item i of the strip held
    // in registers to LDS, fetch item i of the strip two chunks ahead, advance.
    constexpr int NTASK = 2 * NST + NJ + 1;

    // lane parts of the three kinds of LDS read (bytes)
    const unsigned lane128 = (unsigned)(wpix + n * 4) * 4;
    const unsigned lane64 = (unsigned)(wpix + OFF2 + n * 2) * 4;
    const unsigned lane32 = (unsigned)(wpix + OFF1 + n) * 4;

    // One chunk: registers `st` (chunk c+1, fetched one iteration ago) go to the
    // other LDS buffer; the fetch of chunk c+2 and the operands of chunk c+1 are
    // issued; chunk c is contracted out of LDS.  No branch except the per-tap
    // one.  Past the last chunk the same code re-fetches the last chunk and
    // writes it to the buffer nobody reads.
    auto chunk = [&](int c, const int parity, StepOps<SPC> (&cur)[NJ], StepOps<SPC> (&nxt)[NJ]) {
        const int cn = c + 1 < c_end ? c + 1 : c;
        float* const wbuf = lds + (parity ^ 1) * (CK * SP);
        const unsigned rbuf = (unsigned)(parity * (CK * SP) * 4);
        const unsigned l128 = lane128 + rbuf, l64 = lane64 + rbuf, l32 = lane32 + rbuf;
        auto task = [&](int i) {
            if (i < NJ) {
                load_ops(nxt[i], i, cn);
            } else if (i < NJ + NST) {
                stash_item(i - NJ, wbuf);
            } else if (i < NJ + 2 * NST) {
                fetch_item(i - NJ - NST);
            } else {
                fetch_advance();
            }
        };
        float bv[RING][NBLK];
        auto read_b = [&](int t, float (&dst)[NBLK]) {
            const int jj = t / SPC, s = t % SPC;
            const unsigned row = cur[jj].row[s];
            const char* base8 = reinterpret_cast<const char*>(lds);
#pragma unroll
            for (int seg = 0; seg < NF; ++seg) {
                const f4 v = *reinterpret_cast<const f4*>(base8 + (__umul24(row, SP * 4) + l128) + seg * 256);
                dst[seg * 4 + 0] = v.x; dst[seg * 4 + 1] = v.y; dst[seg * 4 + 2] = v.z; dst[seg * 4 + 3] = v.w;
            }
            if constexpr (R >= 2) {
                const f2 v = *reinterpret_cast<const f2*>(base8 + (__umul24(row, SP * 4) + l64));
                dst[NF * 4 + 0] = v.x; dst[NF * 4 + 1] = v.y;
            }
            if constexpr (R == 1 || R == 3)
                dst[NBLK - 1] = *reinterpret_cast<const float*>(base8 + (__umul24(row, SP * 4) + l32));
        };
        if constexpr (VAR) {
            // The first SMIN k-steps of a row block always run (slots past the kept
            // columns carry weight 0) and carry the staging tasks; the others run only
            // up to the count the table gives for this (tile, chunk).
            constexpr int SMIN = SPC / 4;
            constexpr int NMV = NJ * SMIN * NBLK;
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj) {
                const int ns = __builtin_amdgcn_readfirstlane((int)(cur[jj].row[0] >> 16));
                cur[jj].row[0] &= 0xffffu;
#pragma unroll
                for (int s = 0; s < DEPTH && s < SPC; ++s) read_b(jj * SPC + s, bv[s % RING]);
#pragma unroll
                for (int s = 0; s < SPC; ++s) {
                    if (s >= SMIN && s >= ns) break;
                    if (s + DEPTH < SPC) read_b(jj * SPC + s + DEPTH, bv[(s + DEPTH) % RING]);
                    __builtin_amdgcn_sched_barrier(0);
                    const float a = cur[jj].a[s];
#pragma unroll
                    for (int b = 0; b < NBLK; ++b) {
                        acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bv[s % RING][b], acc[jj][b], 0, 0, 0);
                        if (s < SMIN) {
                            const int m = (jj * SMIN + s) * NBLK + b;
#pragma unroll
                            for (int i = m * NTASK / NMV; i < (m + 1) * NTASK / NMV; ++i) task(i);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < DEPTH && t < TOT; ++t) read_b(t, bv[t % RING]);
#pragma unroll
            for (int t = 0; t < TOT; ++t) {
                // the LDS reads of k-step t+DEPTH lead the MFMAs of k-step t
                if (t + DEPTH < TOT) read_b(t + DEPTH, bv[(t + DEPTH) % RING]);
                __builtin_amdgcn_sched_barrier(0);
                const int jj = t / SPC, s = t % SPC;
                const float a = cur[jj].a[s];
#pragma unroll
                for (int b = 0; b < NBLK; ++b) {
                    const int m = t * NBLK + b;
                    acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bv[t % RING][b], acc[jj][b], 0, 0, 0);
#pragma unroll
                    for (int i = m * NTASK / NM; i < (m + 1) * NTASK / NM; ++i) task(i);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        __syncthreads();
    };

    // The loop branch costs about as much as two MFMAs, so short chunk bodies are
    // unrolled four times, long ones twice.
    int c = c_begin;
    if constexpr (NM <= 32) {
        for (; c + 3 < c_end; c += 4) {
            chunk(c, 0, opsA, opsB);
            chunk(c + 1, 1, opsB, opsA);
            chunk(c + 2, 0, opsA, opsB);
            chunk(c + 3, 1, opsB, opsA);
        }
    }
    for (; c + 1 < c_end; c += 2) {
        chunk(c, 0, opsA, opsB);
        chunk(c + 1, 1, opsB, opsA);
    }
    if (c < c_end) chunk(c, 0, opsA, opsB);

    // ---- epilogue: bias, ReLU, cast, NHWC store ------------------------------
    TOUT* __restrict__ y = reinterpret_cast<TOUT*>(p.y);
    const bool fast = (p.tile % 4 == 0) && (p.Cout % 4 == 0);
    auto pixel_of = [&](int b) {   // pixel (inside the wavefront's range) of MFMA block b for this lane
        if (b < 4 * NF) return (b >> 2) * 64 + n * 4 + (b & 3);
        if (R >= 2 && b < 4 * NF + 2) return OFF2 + n * 2 + (b - 4 * NF);
        return OFF1 + n;
    };
    constexpr int WGC = WC * NJ * 16;     // output channels of the workgroup
    if (p.ksplit > 1) {
        // partial sums of this split, fp32, laid out like the output: [split][pixel][channel];
        // bias, residual and activation are applied where the splits are added up
        float* __restrict__ part = p.partial + (size_t)ks * (size_t)p.P * (size_t)p.Cout;
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int rb = rb0 + jj;
            if (rb >= p.n_rowblocks) continue;
            const int j = rb / p.rbpt;
            const int rit = (rb - j * p.rbpt) * 16 + q * 4;
            const int co = j * p.tile + rit;
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + pixel_of(b);
                if (pp >= p.P) continue;
                float* dst = part + (size_t)pp * (size_t)p.Cout + co;
                if (fast) {
                    if (rit < p.tile && co < p.Cout) *reinterpret_cast<f4*>(dst) = acc[jj][b];
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (rit + r < p.tile && co + r < p.Cout) dst[r] = acc[jj][b][r];
                }
            }
        }
        return;
    }
    if (WGC * (int)sizeof(TOUT) >= 128 && tile_out_ok<TOUT>(p)) {
        // through the LDS tile (every wavefront is past its last strip read: the chunk ends with a barrier)
        constexpr int PITCH = tile_pitch<TOUT>(WGC);
        char* const tile = reinterpret_cast<char*>(lds);
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int rb = rb0 + jj;
            const int co = rb * 16 + q * 4;           // T is a multiple of 16: row block rb is channels 16 rb ..
            const bool row_live = rb < p.n_rowblocks && co < p.Cout;
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pl = wpix + pixel_of(b);
                const int pp = p0 + pl;
                tile_put4<TOUT>(p, tile + pl * PITCH + ((wcx * NJ + jj) * 16 + q * 4) * (int)sizeof(TOUT),
                                (unsigned)pp * (unsigned)p.Cout + (unsigned)co, row_live && pp < p.P,
                                acc[jj][b]);   // the bias is already in the accumulator
            }
        }
        __syncthreads();
        tile_flush<TOUT, BP, WGC>(p, tile, p0, cblock * WGC);
        return;
    }
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        const int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) continue;
        const int j = rb / p.rbpt;
        const int sub = rb - j * p.rbpt;
        const int rit = sub * 16 + q * 4;          // first of this lane's 4 rows inside the tile
        const int co = j * p.tile + rit;
        if (fast) {
            if (rit >= p.tile || co >= p.Cout) continue;
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + pixel_of(b);
                if (pp >= p.P) continue;
                emit4(p, y, (unsigned)pp * (unsigned)p.Cout + (unsigned)co, acc[jj][b]);   // bias included
            }
        } else {
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + pixel_of(b);
                if (pp >= p.P) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (rit + r >= p.tile || co + r >= p.Cout) continue;
                    float v = acc[jj][b][r] + (p.bias ? p.bias[co + r] : 0.f);
                    emit1(p, y, (unsigned)pp * (unsigned)p.Cout + (unsigned)(co + r), v);
                }
            }
        }
    }
}

template <int NBLK, int WP, int NJ, int CK, int SPC, int MODE, typename TIN, typename TOUT>
int launch_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_kernel<NBLK, WP, NJ, CK, SPC, MODE, TIN, TOUT>;
    constexpr size_t strip = (size_t)2 * CK * strip_stride(16 * NBLK * WP, CK, MODE != 0) * sizeof(float);
    constexpr size_t otile = out_tile_bytes(16 * NBLK * WP, (4 / WP) * NJ * 16, (int)sizeof(TOUT));
    constexpr size_t lds = strip > otile ? strip : otile;
    {
        static unsigned long long done = 0;
        const int rc = allow_lds(reinterpret_cast<const void*>(kern), lds, &done);
        if (rc != NM_OK) return rc;
    }
    hipLaunchKernelGGL(kern, dim3(p.wg_per_xcd * 8), dim3(256), lds, s, p);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

}  // namespace nm
