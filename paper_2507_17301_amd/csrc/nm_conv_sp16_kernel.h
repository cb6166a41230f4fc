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
#pragma once

#include "nm_conv_kernel.h"

namespace nm {

typedef __bf16 bf8x __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x __attribute__((ext_vector_type(16)));

// LDS row stride (bytes): CK channels plus 16, so that rows stay 16-byte
// aligned and the 16 pixels that a lane group reads with one 16-byte access
// start in 16 different bank quads.
constexpr int strip_sp16_stride(int CK) { return CK * 2 + 16; }
constexpr int strip_sp16_rows(int BP, int CK)
{
    const int opr = CK / 8, pstep = 256 / opr, nit = (BP * opr + 255) / 256;
    return nit * pstep > BP ? nit * pstep : BP;
}

template <int NBLK, int WP, int NJ, int CK, bool SPARSE>
__global__ __launch_bounds__(256) void nm_conv_sp16_kernel(const ConvParams p)
{
    constexpr int BPW = 16 * NBLK;
    constexpr int BP = BPW * WP;
    constexpr int S = strip_sp16_stride(CK);
    constexpr int WC = 4 / WP;
    constexpr int KS = CK / 64;                  // k-steps (64 channels) per chunk
    constexpr int AH = SPARSE ? 1 : 2;           // 16-byte A operands per k-step and row block
    static_assert(CK % 64 == 0, "a chunk is a whole number of 64-channel k-steps");

    extern __shared__ char lds8[];               // [2][ROWS][S]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

    // ---- staging: item = (pixel, 8-channel octet), 16 bytes ----------------
    constexpr int OPR = CK / 8;
    constexpr int PSTEP = 256 / OPR;
    constexpr int NIT = (BP * OPR + 255) / 256;
    constexpr int ROWS = strip_sp16_rows(BP, CK);
    const int oct = tid % OPR;
    const int pl0 = tid / OPR;
    int hi0[NIT], wi0[NIT];
    unsigned base[NIT], voff[NIT];
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
        base[it] = (unsigned)(((b * p.H + h0) * p.W + w0) * p.Cin + oct * 8) * 2;
    }
    u4v st[NIT];
    int f_c = 0, f_kh = 0, f_kw = 0, f_ci0 = 0;
    auto retap = [&]() {
        const int dhh = f_kh * p.dh, dww = f_kw * p.dw;
        const unsigned tapoff = (unsigned)((dhh * p.W + dww) * p.Cin) * 2;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int hi = hi0[it] + dhh, wi = wi0[it] + dww;
            const bool inb = ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            voff[it] = inb ? base[it] + tapoff : kOOB;
        }
    };
    auto fetch_item = [&](int it) {
        st[it] = __builtin_amdgcn_raw_buffer_load_b128(xr, voff[it] + (unsigned)(f_ci0 * 2), 0, 0);
    };
    auto fetch_advance = [&]() {
        const int adv = f_c + 1 < p.nchunks ? 1 : 0;
        f_c += adv;
        const int nci = f_ci0 + CK;
        const int wrap = (adv && nci >= p.Cin) ? 1 : 0;
        f_ci0 = wrap ? 0 : (adv ? nci : f_ci0);
        if (wrap) {
            const int nkw = f_kw + 1;
            const int wrap2 = nkw == p.Kw ? 1 : 0;
            f_kw = wrap2 ? 0 : nkw;
            f_kh += wrap2;
            retap();
        }
    };
    auto stash_item = [&](int it, char* dst) {
        *reinterpret_cast<u4v*>(dst + (pl0 + it * PSTEP) * S + oct * 16) = st[it];
    };

    // ---- operand streams ------------------------------------------------------
    // weights: [row block][chunk][k-step][AH][lane] x 16 bytes (8 bf16)
    // index operands (sparse): [column tile][chunk][lane group][k-step] x 4 bytes
    struct Ops {
        u4v a[KS][AH];
        unsigned idx[KS];
    };
    constexpr unsigned WCH = KS * AH * 1024;     // weight bytes per (row block, chunk)
    constexpr unsigned ICH = KS * 16;            // index bytes per (tile, chunk)
    const unsigned wvoff = (unsigned)lane * 16;
    const unsigned ivoff = (unsigned)q * KS * 4;
    unsigned wsoff[NJ], isoff[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;
        wsoff[jj] = (unsigned)rb * p.nchunks * WCH;
        isoff[jj] = (unsigned)(rb / p.rbpt) * p.nchunks * ICH;
    }
    auto load_ops = [&](Ops& o, int jj, int c) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int h = 0; h < AH; ++h)
                o.a[s][h] = __builtin_amdgcn_raw_buffer_load_b128(
                    wr, wvoff, wsoff[jj] + (unsigned)c * WCH + (unsigned)(s * AH + h) * 1024, 0);
        if constexpr (SPARSE) {
            const unsigned so = isoff[jj] + (unsigned)c * ICH;
            if constexpr (KS == 1) {
                o.idx[0] = __builtin_amdgcn_raw_buffer_load_b32(rr, ivoff, so, 0);
            } else if constexpr (KS == 2) {
                const u2v t = __builtin_amdgcn_raw_buffer_load_b64(rr, ivoff, so, 0);
                o.idx[0] = t.x; o.idx[1] = t.y;
            } else {
                static_assert(KS == 4, "index operands are fetched 1, 2 or 4 at a time");
                const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rr, ivoff, so, 0);
                o.idx[0] = t.x; o.idx[1] = t.y; o.idx[2] = t.z; o.idx[3] = t.w;
            }
        }
    };

    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = f4{0.f, 0.f, 0.f, 0.f};

    Ops opsA[NJ], opsB[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) load_ops(opsA[jj], jj, 0);
    retap();
#pragma unroll
    for (int it = 0; it < NIT; ++it) fetch_item(it);
    fetch_advance();
#pragma unroll
    for (int it = 0; it < NIT; ++it) stash_item(it, lds8);
#pragma unroll
    for (int it = 0; it < NIT; ++it) fetch_item(it);
    fetch_advance();
    __syncthreads();

    constexpr int NM = KS * NBLK;                // B operands (LDS reads) per chunk for this wavefront
    constexpr int NTASK = 2 * NIT + NJ + 1;
    // this lane's 32 bytes inside block 0, k-step 0
    const unsigned lanepix = (unsigned)((wpix + n) * S + q * 32);

    // One chunk: the strip of the next chunk goes from registers to the other
    // LDS buffer, the fetch two chunks ahead and the operands of the next chunk
    // are issued, all dealt out behind the matrix instructions of this chunk.
    auto chunk = [&](int c, const int parity, Ops (&cur)[NJ], Ops (&nxt)[NJ]) {
        const int cn = c + 1 < p.nchunks ? c + 1 : c;
        char* const wbuf = lds8 + (parity ^ 1) * (ROWS * S);
        const char* const rbase = lds8 + parity * (ROWS * S) + lanepix;
        auto task = [&](int i) {
            if (i < NJ) {
                load_ops(nxt[i], i, cn);
            } else if (i < NJ + NIT) {
                stash_item(i - NJ, wbuf);
            } else if (i < NJ + 2 * NIT) {
                fetch_item(i - NJ - NIT);
            } else {
                fetch_advance();
            }
        };
        auto read_b = [&](int m, u4v (&dst)[2]) {
            const int s = m / NBLK, b = m % NBLK;
            const char* a = rbase + b * 16 * S + s * 128;
            dst[0] = *reinterpret_cast<const u4v*>(a);
            dst[1] = *reinterpret_cast<const u4v*>(a + 16);
        };
        u4v ring[2][2];
        read_b(0, ring[0]);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const int s = m / NBLK, b = m % NBLK;
            if (m + 1 < NM) read_b(m + 1, ring[(m + 1) & 1]);
            const u4v(&bo)[2] = ring[m & 1];
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj) {
                if constexpr (SPARSE) {
                    const bf16x bv = __builtin_shufflevector(__builtin_bit_cast(bf8x, bo[0]),
                                                             __builtin_bit_cast(bf8x, bo[1]), 0, 1, 2, 3, 4,
                                                             5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                    acc[jj][b] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(
                        __builtin_bit_cast(bf8x, cur[jj].a[s][0]), bv, acc[jj][b], (int)cur[jj].idx[s], 0, 0);
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf8x, cur[jj].a[s][h]), __builtin_bit_cast(bf8x, bo[h]),
                            acc[jj][b], 0, 0, 0);
                }
            }
#pragma unroll
            for (int i = m * NTASK / NM; i < (m + 1) * NTASK / NM; ++i) task(i);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };

    int c = 0;
    for (; c + 1 < p.nchunks; c += 2) {
        chunk(c, 0, opsA, opsB);
        chunk(c + 1, 1, opsB, opsA);
    }
    if (c < p.nchunks) chunk(c, 0, opsA, opsB);

    // ---- epilogue: bias, ReLU, round to bf16, NHWC store ------------------------
    bf16_t* __restrict__ y = reinterpret_cast<bf16_t*>(p.y);
    const bool fast = (p.tile % 4 == 0) && (p.Cout % 4 == 0);
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
            f4 bb = {0.f, 0.f, 0.f, 0.f};
            if (p.bias) bb = *reinterpret_cast<const f4*>(p.bias + co);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + b * 16 + n;
                if (pp >= p.P) continue;
                f4 v = acc[jj][b] + bb;
                if (p.relu) {
                    v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f);
                    v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
                }
                store4(y + (size_t)pp * p.Cout + co, v);
            }
        } else {
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + b * 16 + n;
                if (pp >= p.P) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (rit + r >= p.tile || co + r >= p.Cout) continue;
                    float v = acc[jj][b][r] + (p.bias ? p.bias[co + r] : 0.f);
                    if (p.relu) v = fmaxf(v, 0.f);
                    store1(y + (size_t)pp * p.Cout + co + r, v);
                }
            }
        }
    }
}

template <int NBLK, int WP, int NJ, int CK, bool SPARSE>
int launch_sp16_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_sp16_kernel<NBLK, WP, NJ, CK, SPARSE>;
    constexpr size_t lds = (size_t)2 * strip_sp16_rows(16 * NBLK * WP, CK) * strip_sp16_stride(CK);
    if (lds > 64 * 1024) {
        static hipError_t once = hipFuncSetAttribute(
            reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (once != hipSuccess) {
            set_error("hipFuncSetAttribute(LDS %zu) failed: %s", lds, hipGetErrorString(once));
            return NM_ERR_HIP;
        }
    }
    hipLaunchKernelGGL(kern, dim3(p.wg_per_xcd * 8), dim3(256), lds, s, p);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

}  // namespace nm
