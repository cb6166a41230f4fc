// bf16 variant of the fused convolution: bf16 activations and bf16 (rounded)
// kept weights are multiplied on the bf16 matrix cores with fp32 accumulation.
//
// Same decomposition as the fp32 kernel (workgroup = BP pixels x row blocks,
// K walked in chunks, strip of the im2col matrix in LDS, contraction of
// Alg. 1 over the kept columns only), with what the bf16 MFMA changes:
//   * v_mfma_f32_16x16x32_bf16 wants, per lane, eight K-consecutive values of
//     one pixel (lane j + 16q holds K = 8q..8q+7 of column j).  After
//     compaction the kept columns are not contiguous, so the strip is laid out
//     [pixel][channel] and every lane gathers its eight kept values with
//     2-byte LDS reads; the eight channel offsets are a property of the column
//     tile and the wavefront quarter, come from the operand table, and are
//     added to the lane's pixel address once per k-step -- the pixel blocks of
//     the wavefront are then reached with immediate offsets.
//   * a k-step is 32 kept columns; a chunk of CK channels holds SPC k-steps.
//   * column tiles wider than 16 (T = 32) are two row blocks that share one
//     kept set, so SHARE = 2 feeds both from the same gathered operand.
#pragma once

#include "nm_conv_kernel.h"

namespace nm {

typedef short s8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));

// LDS row stride (bytes) of the bf16 strip: CK channels plus 4 bytes, so that
// the 16 pixels a wavefront quarter reads at one channel fall into 16 banks.
constexpr int strip16_stride(int CK) { return CK * 2 + 4; }

template <int NBLK, int WP, int NJ, int CK, int SPC, int SHARE>
__global__ __launch_bounds__(256) void nm_conv_bf16_kernel(const ConvParams p)
{
    constexpr int BPW = 16 * NBLK;
    constexpr int BP = BPW * WP;
    constexpr int S = strip16_stride(CK);        // bytes per pixel row of the strip
    constexpr int WC = 4 / WP;
    constexpr int NG = NJ / SHARE;               // groups of row blocks that share one gathered operand
    static_assert(NJ % SHARE == 0, "row blocks per wavefront must be a multiple of SHARE");

    extern __shared__ char lds8[];               // [2][BP][S]

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
    constexpr int OPR = CK / 8;                  // octets per pixel row
    constexpr int PSTEP = 256 / OPR;
    constexpr int NIT = (BP * OPR + 255) / 256;
    constexpr int ROWS = NIT * PSTEP > BP ? NIT * PSTEP : BP;   // pixel rows the staging threads write
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
        unsigned* d = reinterpret_cast<unsigned*>(dst + (pl0 + it * PSTEP) * S + oct * 16);
        d[0] = st[it].x; d[1] = st[it].y; d[2] = st[it].z; d[3] = st[it].w;
    };

    // ---- operand streams ------------------------------------------------------
    // per (row block, chunk, k-step): 8 bf16 weights per lane (16 bytes);
    // per (tile, chunk, k-step, quarter): 8 channel byte offsets (32 bytes)
    struct Ops {
        u4v a[SHARE][SPC];
        unsigned off[SPC][8];
    };
    const unsigned wvoff = (unsigned)lane * 16;
    const unsigned rvoff = (unsigned)q * 32;
    unsigned wsoff[NJ], rsoff[NG];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;
        wsoff[jj] = (unsigned)rb * p.nchunks * (SPC * 64 * 16);
        if (jj % SHARE == 0) rsoff[jj / SHARE] = (unsigned)(rb / p.rbpt) * p.nchunks * (SPC * 4 * 32);
    }
    auto load_ops = [&](Ops& o, int gi, int c) {
#pragma unroll
        for (int s = 0; s < SPC; ++s) {
#pragma unroll
            for (int h = 0; h < SHARE; ++h)
                o.a[h][s] = __builtin_amdgcn_raw_buffer_load_b128(
                    wr, wvoff, wsoff[gi * SHARE + h] + (unsigned)(c * SPC + s) * (64 * 16), 0);
            const unsigned so = rsoff[gi] + (unsigned)(c * SPC + s) * (4 * 32);
            const u4v lo = __builtin_amdgcn_raw_buffer_load_b128(rr, rvoff, so, 0);
            const u4v hi = __builtin_amdgcn_raw_buffer_load_b128(rr, rvoff + 16, so, 0);
            o.off[s][0] = lo.x; o.off[s][1] = lo.y; o.off[s][2] = lo.z; o.off[s][3] = lo.w;
            o.off[s][4] = hi.x; o.off[s][5] = hi.y; o.off[s][6] = hi.z; o.off[s][7] = hi.w;
        }
    };

    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = f4{0.f, 0.f, 0.f, 0.f};

    Ops opsA[NG], opsB[NG];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) load_ops(opsA[gi], gi, 0);
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

    constexpr int NM = NG * SPC * NBLK;          // gathered operands per chunk for this wavefront
    constexpr int NTASK = 2 * NIT + NG + 1;
    const unsigned lanepix = (unsigned)((wpix + n) * S);   // this lane's pixel row in block 0

    auto chunk = [&](int c, const int parity, Ops (&cur)[NG], Ops (&nxt)[NG]) {
        const int cn = c + 1 < p.nchunks ? c + 1 : c;
        char* const wbuf = lds8 + (parity ^ 1) * (ROWS * S);
        const char* const rbase = lds8 + parity * (ROWS * S) + lanepix;
        auto task = [&](int i) {
            if (i < NG) {
                load_ops(nxt[i], i, cn);
            } else if (i < NG + NIT) {
                stash_item(i - NG, wbuf);
            } else if (i < NG + 2 * NIT) {
                fetch_item(i - NG - NIT);
            } else {
                fetch_advance();
            }
        };
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
#pragma unroll
            for (int s = 0; s < SPC; ++s) {
                const char* ap[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) ap[e] = rbase + cur[gi].off[s][e];
#pragma unroll
                for (int b = 0; b < NBLK; ++b) {
                    s8v g;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        g[e] = *reinterpret_cast<const short*>(ap[e] + b * 16 * S);
                    const bf8v bop = __builtin_bit_cast(bf8v, g);
#pragma unroll
                    for (int h = 0; h < SHARE; ++h) {
                        const int jj = gi * SHARE + h;
                        acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf8v, cur[gi].a[h][s]), bop, acc[jj][b], 0, 0, 0);
                    }
                    const int m = (gi * SPC + s) * NBLK + b;
#pragma unroll
                    for (int i = m * NTASK / NM; i < (m + 1) * NTASK / NM; ++i) task(i);
                }
            }
        }
        __syncthreads();
    };

    int c = 0;
    for (; c + 1 < p.nchunks; c += 2) {
        chunk(c, 0, opsA, opsB);
        chunk(c + 1, 1, opsB, opsA);
    }
    if (c < p.nchunks) chunk(c, 0, opsA, opsB);

    // ---- epilogue ---------------------------------------------------------------
    bf16_t* __restrict__ y = reinterpret_cast<bf16_t*>(p.y);
    const bool fast = (p.tile % 4 == 0) && (p.Cout % 4 == 0);
    constexpr int WGC = WC * NJ * 16;            // output channels of the workgroup
    if (WGC * 2 >= 128 && tile_out_ok<bf16_t>(p)) {
        // whole 128-byte lines through the LDS tile (the last chunk ended with a barrier)
        constexpr int PITCH = tile_pitch<bf16_t>(WGC);
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int rb = rb0 + jj;
            const int co = rb * 16 + q * 4;       // T is a multiple of 16: row block rb is channels 16 rb ..
            const bool row_live = rb < p.n_rowblocks && co < p.Cout;
            f4 bb = {0.f, 0.f, 0.f, 0.f};
            if (p.bias && row_live) bb = *reinterpret_cast<const f4*>(p.bias + co);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pl = wpix + b * 16 + n;
                const int pp = p0 + pl;
                tile_put4<bf16_t>(p, lds8 + pl * PITCH + ((wcx * NJ + jj) * 16 + q * 4) * 2,
                                  (unsigned)pp * (unsigned)p.Cout + (unsigned)co, row_live && pp < p.P,
                                  acc[jj][b] + bb);
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
            f4 bb = {0.f, 0.f, 0.f, 0.f};
            if (p.bias) bb = *reinterpret_cast<const f4*>(p.bias + co);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + b * 16 + n;
                if (pp >= p.P) continue;
                f4 v = acc[jj][b] + bb;
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
                    float v = acc[jj][b][r] + (p.bias ? p.bias[co + r] : 0.f);
                    emit1(p, y, (unsigned)pp * (unsigned)p.Cout + (unsigned)(co + r), v);
                }
            }
        }
    }
}

template <int NBLK, int WP, int NJ, int CK, int SPC, int SHARE>
int launch16_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_bf16_kernel<NBLK, WP, NJ, CK, SPC, SHARE>;
    constexpr int BP = 16 * NBLK * WP;
    constexpr int OPR = CK / 8, PSTEP = 256 / OPR, NIT = (BP * OPR + 255) / 256;
    constexpr int ROWS = NIT * PSTEP > BP ? NIT * PSTEP : BP;
    constexpr size_t strip = (size_t)2 * ROWS * strip16_stride(CK);
    constexpr size_t otile = out_tile_bytes(BP, (4 / WP) * NJ * 16, 2);
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
