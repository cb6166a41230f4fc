// bf16 convolution for layers with very few input channels (the 7x7 first
// layer of the ResNets: Cin = 3, paper section 4.1.2 keeps it dense).
//
// With Cin this small the im2col row of a pixel is not made of channel runs
// worth fetching, but for a fixed kernel row kh the Kw * Cin values
// x[b][hi][wi0 .. wi0 + Kw - 1][0 .. Cin - 1] are one contiguous run in NHWC.
// The strip therefore holds, per pixel, Kh runs of GR 16-byte granules (the run
// starts d = 0 or 1 elements early so that it is 4-byte aligned, and is padded
// to whole granules), padded to KS 64-element k-steps; the weights are laid
// out to match, zero in every padding slot.  K grows from Kh*Kw*Cin to
// KS*64 (147 -> 192 for the 7x7x3 layer), which the bf16 matrix cores absorb
// easily; in exchange the whole strip arrives through 16-byte loads straight
// into LDS and the contraction is the dense one of the gather-free kernel.
//
// A run may hang over the left or right image border (there the neighbouring
// image row would be read) or over the ends of the tensor.  Those granules --
// a few per image row -- are instead assembled element by element with guarded
// loads by the thread that owns them and written over the granule before the
// workgroup starts contracting.
//
// One chunk only: the whole (padded) K of a pixel tile is resident at once.
#pragma once

#include "nm_conv_sp16_kernel.h"

namespace nm {

// granule position swizzle for rows of 8 * KS granules (see the gather-free kernel)
__device__ inline int run16_swz(int row, int KS) { return (KS & 1) ? ((row & 7) ^ ((row >> 3) & 1)) : (row & 15); }

// strip [BP][KS*64] bf16, then the dense weights of the workgroup's row blocks: one copy per
// group of waves that work on the same row blocks (WC = 4 / WP groups)
constexpr int run16_lds_bytes(int BP, int WP, int NJ, int KS) { return BP * KS * 128 + (4 / WP) * NJ * KS * 2048; }

template <int NBLK, int WP, int NJ, int KS>
__global__ __launch_bounds__(256) void nm_conv_run16_kernel(const ConvParams p)
{
    constexpr int BPW = 16 * NBLK;
    constexpr int BP = BPW * WP;
    constexpr int WC = 4 / WP;
    constexpr int GPR = 8 * KS;                  // granules per pixel row of the strip
    constexpr int RB = GPR * 16;                 // bytes per pixel row
    constexpr int AW = NJ * KS * 2048;           // weight bytes per group of waves sharing row blocks

    extern __shared__ __attribute__((aligned(16))) char lds8[];   // [BP][RB] strip, then [WC][AW] weights

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

    // ---- weights of this wave's row blocks: [row block][k-step][half][lane] x 16 bytes.
    // The WP waves that share the row blocks split the loads between them.
#pragma unroll
    for (int li = 0; li < NJ * KS * 2; ++li) {
        if (WP > 1 && li % WP != wpx) continue;              // wave-uniform
        const int jj = li / (KS * 2), sh = li % (KS * 2);
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;
        const unsigned vo = (unsigned)lane * 16 + ((unsigned)rb * KS * 2 + sh) * 1024;
        char* d = lds8 + BP * RB + wcx * AW + li * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (lds_ptr_t)d, 16, vo, 0, 0, 0);
    }

    // ---- strip: wave-wide loads of 64 granules; load i is issued by wave i % 4
    constexpr int NW = BP * GPR / 64;
    constexpr int NIT = (NW + 3) / 4;
    const int HoWo = p.Ho * p.Wo;
    const int GR = p.run_gr, dsh = p.run_d;
    const int KwC = p.Kw * p.Cin;
    u4v fix[NIT];
    bool need[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        need[it] = false;
        fix[it] = u4v{0u, 0u, 0u, 0u};
        if (NW % 4 != 0 && wave + 4 * it >= NW) continue;     // wave-uniform
        const int G = (wave + 4 * it) * 64 + lane;            // granule slot of the strip this lane fills
        const int pl = G / GPR;
        const int g = (G % GPR) ^ run16_swz(pl, KS);          // the granule that belongs at that slot
        const int kh = (int)fdiv((unsigned)g, p.gr_mul, p.gr_shift), gi = g - kh * GR;
        const int pp = p0 + pl;
        const int b = (int)fdiv((unsigned)pp, p.howo_mul, p.howo_shift);
        const int rem = pp - b * HoWo;
        const int ho = (int)fdiv((unsigned)rem, p.wo_mul, p.wo_shift);
        const int wo = rem - ho * p.Wo;
        const int hi = ho * p.sh - p.ph + kh * p.dh;
        const int wi0 = wo * p.sw - p.pw;
        const bool rowok = (pp < p.P) & (kh < p.Kh) & ((unsigned)hi < (unsigned)p.H);
        // first element of the granule in the tensor, and which of its 8 elements are real taps
        const int e0 = gi * 8 - dsh;                          // position in the run of element 0
        // (32-bit: the tensor has fewer than 2^30 elements and rows that pass `rowok` lie inside it)
        const int start = ((b * p.H + hi) * p.W + wi0) * p.Cin + e0;
        // columns the real taps of this granule touch: elements max(e0,0) .. min(e0+7, KwC-1)
        const int lo = e0 > 0 ? e0 : 0, hi_e = e0 + 7 < KwC - 1 ? e0 + 7 : KwC - 1;
        const bool any = lo <= hi_e;
        const int wlo = wi0 + (int)fdiv((unsigned)lo, p.cin_mul, p.cin_shift);
        const int whi = wi0 + (any ? (int)fdiv((unsigned)hi_e, p.cin_mul, p.cin_shift) : 0);
        const bool inside = (wlo >= 0) & (whi < p.W) & (start >= 0) & ((unsigned)start + 8u <= p.x_elems);
        const bool dma = rowok & any & inside;
        need[it] = rowok & any & !inside;
        const unsigned off = dma ? (unsigned)start * 2u : kOOB;
        char* dst = lds8 + (wave + 4 * it) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (lds_ptr_t)dst, 16, off, 0, 0, 0);
        if (need[it]) {
            // border granule: element by element, zero where the column is outside the image
            unsigned short v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int er = e0 + e;
                const int wi = wi0 + (er >= 0 ? (int)fdiv((unsigned)er, p.cin_mul, p.cin_shift) : -1);
                const bool ok = (er >= 0) & (er < KwC) & ((unsigned)wi < (unsigned)p.W);
                v[e] = __builtin_amdgcn_raw_buffer_load_b16(xr, ok ? (unsigned)(start + e) * 2u : kOOB, 0, 0);
            }
            fix[it] = u4v{(unsigned)v[0] | ((unsigned)v[1] << 16), (unsigned)v[2] | ((unsigned)v[3] << 16),
                          (unsigned)v[4] | ((unsigned)v[5] << 16), (unsigned)v[6] | ((unsigned)v[7] << 16)};
        }
    }

    // bias of this lane's rows
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

    // all loads of this thread have landed; then the border granules go over the zeros
    NM_WAIT_VMCNT(0);
#pragma unroll
    for (int it = 0; it < NIT; ++it)
        if (need[it]) *reinterpret_cast<u4v*>(lds8 + (wave + 4 * it) * 1024 + lane * 16) = fix[it];
    __syncthreads();

    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = bb[jj];   // start from the bias

    const char* const abase = lds8 + BP * RB + wcx * AW + lane * 16;
    const int sw = run16_swz(n, KS);             // rows of block b are 16 b + n: same swizzle for every block
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        u4v a[NJ][2];
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                a[jj][h] = *reinterpret_cast<const u4v*>(abase + ((jj * KS + s) * 2 + h) * 1024);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const char* row = lds8 + (wpix + b * 16 + n) * RB;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const u4v bo = *reinterpret_cast<const u4v*>(row + (((s * 8 + q * 2 + h) ^ sw) * 16));
#pragma unroll
                for (int jj = 0; jj < NJ; ++jj)
                    acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf8x, a[jj][h]), __builtin_bit_cast(bf8x, bo), acc[jj][b], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: bias, ReLU, round to bf16, NHWC store ------------------------
    bf16_t* __restrict__ y = reinterpret_cast<bf16_t*>(p.y);
    constexpr int WGC = WC * NJ * 16;            // output channels of the workgroup
    if (WGC * 2 >= 128 && fast && tile_out_ok<bf16_t>(p)) {
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
                tile_put4<bf16_t>(p, lds8 + pl * PITCH + ((wcx * NJ + jj) * 16 + q * 4) * 2,
                                  (unsigned)pp * (unsigned)p.Cout + (unsigned)co, row_live && pp < p.P,
                                  acc[jj][b]);   // the bias is already in the accumulator
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
                const f4 v = acc[jj][b];   // the bias is already in the accumulator
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

template <int NBLK, int WP, int NJ, int KS>
int launch_run16_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_run16_kernel<NBLK, WP, NJ, KS>;
    constexpr size_t work = run16_lds_bytes(16 * NBLK * WP, WP, NJ, KS);
    constexpr size_t otile = out_tile_bytes(16 * NBLK * WP, (4 / WP) * NJ * 16, 2);
    constexpr size_t lds = work > otile ? work : otile;
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
