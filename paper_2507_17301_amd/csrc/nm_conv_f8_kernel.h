// fp8 (E4M3) convolution: activations and kept weights one byte each, exact products, fp32
// accumulation, bf16 output.  The second workload beside fp32 / bf16: it halves the bytes of
// the activations once more, which is what bounds the bf16 layers.
//
// Matrix instruction: the dense v_mfma_f32_16x16x32_fp8_fp8 on the zero-filled weights of the
// column tile (two per 64-channel k-step).  Its operands are 8 bytes per lane with
//   A: lane i + 16 q holds row i, K positions 8 q .. 8 q + 7
//   B: lane n + 16 q holds column n, K positions 8 q .. 8 q + 7
//   D: lane n + 16 q register r is row 4 q + r, column n
// (checked on the device against a plain matrix product of small integers).  Which channel a
// K position stands for is free as long as A and B agree: lane group q takes channels
// 16 q .. 16 q + 15 of the k-step, the first eight for the first instruction, the other eight
// for the second, so that a lane's share of the activations is 16 contiguous bytes of a
// pixel's NHWC row -- one 16-byte load -- and the weights are laid out to match by nm_prune.
// (The sparse fp8 instruction of the same shape pairs lanes and K positions differently from
// its bf16 sibling; its layout is not used here.)
//
// Both operands stream from global memory into registers, two register sets, one chunk
// ahead; there is no LDS staging and no workgroup barrier.  A wavefront owns 16 NBLK pixels x
// 16 NJ output channels from its first instruction to its last; the epilogue turns the
// accumulator layout into whole 128-byte lines through a wavefront-private LDS tile.
// The loads of a lane group touch 16 different pixel rows, 64 bytes of each: per byte moved
// this costs the L1 more than staged, coalesced rows would, and it is what bounds the kernel;
// with one byte per element it moves half the bytes of a bf16 kernel of the same form.
#pragma once

#include "nm_conv_kernel.h"

namespace nm {

constexpr int f8_pitch(int NJ) { return NJ * 32 + 16; }                 // bytes per pixel row of the bf16 output tile
constexpr int f8_lds_bytes(int NBLK, int NJ) { return 4 * 16 * NBLK * f8_pitch(NJ); }

template <int NBLK, int NJ> struct F8Stage {
    u4v b[NBLK];
    u4v a[NJ];
};

template <int NBLK, int WP, int NJ>
__global__ __launch_bounds__(256) void nm_conv_f8_kernel(const ConvParams p)
{
    constexpr int BPW = 16 * NBLK;
    constexpr int BP = BPW * WP;
    constexpr int WC = 4 / WP;
    constexpr unsigned WCH = 1024;               // weight bytes per (row block, chunk)
    typedef F8Stage<NBLK, NJ> Stage;

    extern __shared__ __attribute__((aligned(16))) char lds8[];

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
    const int wpx = wave % WP, wcx = wave / WP;
    const int rb0 = (cblock * WC + wcx) * NJ;
    const int wpix = ptile * BP + wpx * BPW;     // first pixel of this wavefront
    if (rb0 >= p.n_rowblocks) return;            // no row block at all (there is no barrier to miss)

    const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.x, p.x_bytes);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wfrag, p.wfrag_bytes);

    // ---- this lane's pixel in every block (byte offsets: one byte per element) ----
    int hi0[NBLK], wi0[NBLK];
    unsigned base[NBLK], voff[NBLK];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
        const int pp = wpix + b * 16 + n;
        const bool live = pp < p.P;
        const int img = (int)fdiv((unsigned)pp, p.howo_mul, p.howo_shift);
        const int rem = pp - img * HoWo;
        const int ho = (int)fdiv((unsigned)rem, p.wo_mul, p.wo_shift);
        const int wo = rem - ho * p.Wo;
        const int h0 = ho * p.sh - p.ph, w0 = wo * p.sw - p.pw;
        hi0[b] = live ? h0 : -(1 << 28);         // a dead pixel has every tap outside the image
        wi0[b] = w0;
        base[b] = (unsigned)(((img * p.H + h0) * p.W + w0) * p.Cin + q * 16);
    }
    int f_c = 0, f_kh = 0, f_kw = 0, f_ci0 = 0;  // fetch iterator: chunk f_c = tap (f_kh, f_kw), channels f_ci0 .. + 63
    auto retap = [&]() {
        const int dhh = f_kh * p.dh, dww = f_kw * p.dw;
        const unsigned tapoff = (unsigned)((dhh * p.W + dww) * p.Cin);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int hi = hi0[b] + dhh, wi = wi0[b] + dww;
            const bool inb = ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            voff[b] = inb ? base[b] + tapoff : kOOB;
        }
    };
    unsigned wsoff[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;   // its results are never stored
        wsoff[jj] = (unsigned)rb * p.nchunks * WCH + (unsigned)lane * 16;
    }
    // every load of the current fetch chunk, then step the iterator (never stepped past the last chunk's loads)
    auto fetch = [&](Stage& st) {
        const unsigned cio = (unsigned)f_ci0;    // kOOB + cio stays out of range: cio < Cin <= 2^16, x below 2 GiB
#pragma unroll
        for (int b = 0; b < NBLK; ++b) st.b[b] = __builtin_amdgcn_raw_buffer_load_b128(xr, voff[b] + cio, 0, 0);
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
            st.a[jj] = __builtin_amdgcn_raw_buffer_load_b128(wr, wsoff[jj] + (unsigned)f_c * WCH, 0, 0);
        ++f_c;
        f_ci0 += 64;
        if (f_ci0 >= p.Cin) {                    // wave-uniform
            f_ci0 = 0;
            if (++f_kw == p.Kw) { f_kw = 0; ++f_kh; }
            retap();
        }
    };
    auto half = [](const u4v& v, int h) -> long {
        const unsigned long long lo = h ? v.z : v.x, hi = h ? v.w : v.y;
        return (long)(lo | (hi << 32));
    };
    auto contract = [&](const Stage& st, f4 (&acc)[NJ][NBLK]) {
#pragma unroll
        for (int b = 0; b < NBLK; ++b)
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(half(st.a[jj], h), half(st.b[b], h),
                                                                            acc[jj][b], 0, 0, 0);
    };

    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = f4{0.f, 0.f, 0.f, 0.f};

    // ---- K loop: two register sets, one chunk ahead ------------------------------
    Stage s0, s1;
    retap();
    fetch(s0);
    int c = 0;
    for (; c + 2 < p.nchunks; c += 2) {
        fetch(s1);
        contract(s0, acc);
        fetch(s0);
        contract(s1, acc);
    }
    if (p.nchunks - c == 2) {
        fetch(s1);
        contract(s0, acc);
        contract(s1, acc);
    } else {
        contract(s0, acc);
    }

    // ---- epilogue: back to the weights' scale, bias, residual, ReLU, bf16, whole lines out
    // (the host launches this kernel only for T % 16 == 0 and Cout % 8 == 0: row block rb is
    //  channels 16 rb .., and the channels beyond Cout come in whole groups of 8)
    constexpr int PITCH = f8_pitch(NJ);
    char* const tile = lds8 + wave * (BPW * PITCH);
    const bf16_t* res = reinterpret_cast<const bf16_t*>(p.res);
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        const int co = (rb0 + jj) * 16 + q * 4;
        f4 bb = f4{0.f, 0.f, 0.f, 0.f};
        if (p.bias && co < p.Cout) bb = *reinterpret_cast<const f4*>(p.bias + co);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int pl = b * 16 + n;
            const int pp = wpix + pl;
            f4 v = acc[jj][b] * p.oscale + bb;
            if (res && pp < p.P && co < p.Cout) v = v + load4(res + ((unsigned)pp * (unsigned)p.Cout + (unsigned)co));
            if (p.relu) v = relu4(v);
            store4(reinterpret_cast<bf16_t*>(tile + pl * PITCH + (jj * 16 + q * 4) * 2), v);
        }
    }
    // the tile is private to this wavefront and LDS executes a wavefront's instructions in
    // order; the compiler must not move the reads above the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int GPR = NJ * 2;                  // 16-byte granules per pixel row of the tile
    constexpr int RSTEP = 64 / GPR;              // rows per wave-wide store
    static_assert(64 % GPR == 0, "a row's granules divide the wavefront");
    const int g = lane % GPR, r0 = lane / GPR;
    const int cg = rb0 * 16 + g * 8;             // first channel of this lane's granule
    if (cg < p.Cout) {
        bf16_t* __restrict__ y = reinterpret_cast<bf16_t*>(p.y);
#pragma unroll
        for (int it = 0; it < BPW / RSTEP; ++it) {
            const int pl = it * RSTEP + r0;
            const int pp = wpix + pl;
            if (pp < p.P) {
                const u4v v = *reinterpret_cast<const u4v*>(tile + pl * PITCH + g * 16);
                *reinterpret_cast<u4v*>(y + ((unsigned)pp * (unsigned)p.Cout + (unsigned)cg)) = v;
            }
        }
    }
}

template <int NBLK, int WP, int NJ>
int launch_f8_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_f8_kernel<NBLK, WP, NJ>;
    constexpr size_t lds = f8_lds_bytes(NBLK, NJ);
    {
        static unsigned long long done = 0;
        const int rc = allow_lds(reinterpret_cast<const void*>(kern), lds, &done);
        if (rc != NM_OK) return rc;
    }
    if (p.tile % 16 != 0 || p.Cout % 8 != 0 || p.Cin % 64 != 0) {
        set_error("internal: the fp8 kernel needs T %% 16 == 0, Cout %% 8 == 0, Cin %% 64 == 0");
        return NM_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL(kern, dim3(p.wg_per_xcd * 8), dim3(256), lds, s, p);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

}  // namespace nm
