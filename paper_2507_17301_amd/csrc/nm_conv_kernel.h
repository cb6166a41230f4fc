// Fused im2col + packing + column-wise N:M contraction + bias/ReLU for gfx950.
//
// One workgroup (4 wavefronts of 64) produces BP output pixels x (4/WP)*NJ*16
// output channels.  The K axis is walked in chunks of CK rows of the im2col
// matrix (paper section 2.2); for each chunk the workgroup gathers
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
// A lane's 16-byte LDS read returns four consecutive pixels of one row, which
// feed four MFMAs; so MFMA block e of a 64-pixel segment owns pixels 4j + e.
#pragma once

#include "nm_launch_decl.h"

namespace nm {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));



template <typename T> struct elem;
template <> struct elem<float> { static constexpr nm_dtype_t dt = NM_F32; };
template <> struct elem<bf16_t> { static constexpr nm_dtype_t dt = NM_BF16; };

__device__ inline f4 load4(const float* p) { return *reinterpret_cast<const f4*>(p); }
__device__ inline f4 load4(const bf16_t* p)
{
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    f4 r;
    r.x = __uint_as_float(u.x << 16);
    r.y = __uint_as_float(u.x & 0xffff0000u);
    r.z = __uint_as_float(u.y << 16);
    r.w = __uint_as_float(u.y & 0xffff0000u);
    return r;
}
__device__ inline float load1(const float* p) { return *p; }
__device__ inline float load1(const bf16_t* p) { return __uint_as_float((unsigned)p->v << 16); }

__device__ inline unsigned short to_bf16_bits(float v)
{
    unsigned u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ inline void store4(float* p, f4 v) { *reinterpret_cast<f4*>(p) = v; }
__device__ inline void store4(bf16_t* p, f4 v)
{
    uint2 u;
    u.x = (unsigned)to_bf16_bits(v.x) | ((unsigned)to_bf16_bits(v.y) << 16);
    u.y = (unsigned)to_bf16_bits(v.z) | ((unsigned)to_bf16_bits(v.w) << 16);
    *reinterpret_cast<uint2*>(p) = u;
}
__device__ inline void store1(float* p, float v) { *p = v; }
__device__ inline void store1(bf16_t* p, float v) { p->v = to_bf16_bits(v); }

// Per-lane operand fetch for one (row block, chunk): SPC weights and the SPC
// LDS rows (one byte each) of this lane's quarter.
template <int SPC> struct StepOps {
    float a[SPC];
    unsigned rw[(SPC + 3) / 4];
};

template <int SPC>
__device__ inline void load_ops(StepOps<SPC>& o, const float* __restrict__ wf,
                                const unsigned char* __restrict__ rows)
{
    if constexpr (SPC == 1) {
        o.a[0] = wf[0];
    } else if constexpr (SPC == 2) {
        const f2 v = *reinterpret_cast<const f2*>(wf);
        o.a[0] = v.x; o.a[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < SPC / 4; ++i) {
            const f4 v = *reinterpret_cast<const f4*>(wf + 4 * i);
            o.a[4 * i + 0] = v.x; o.a[4 * i + 1] = v.y; o.a[4 * i + 2] = v.z; o.a[4 * i + 3] = v.w;
        }
    }
#pragma unroll
    for (int i = 0; i < (SPC + 3) / 4; ++i) o.rw[i] = reinterpret_cast<const unsigned*>(rows)[i];
}

// Buffer loads: an offset at or beyond the descriptor's size returns zeros, which
// is how padding, ragged pixel tiles and partial chunks are filled without a branch.
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
constexpr unsigned kOOB = 0x80000000u;   // beyond any tensor this library accepts (< 2 GiB)

__device__ inline f4 buf_load4(__amdgpu_buffer_rsrc_t r, unsigned off, const float*)
{
    const u4v v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
    return f4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
}
__device__ inline f4 buf_load4(__amdgpu_buffer_rsrc_t r, unsigned off, const bf16_t*)
{
    const u2v u = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
    return f4{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
              __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
}
__device__ inline float buf_load1(__amdgpu_buffer_rsrc_t r, unsigned off, const float*)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
}
__device__ inline float buf_load1(__amdgpu_buffer_rsrc_t r, unsigned off, const bf16_t*)
{
    return __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0) << 16);
}


template <int BP, int WP, int NJ, int CK, int SPC, bool VEC, typename TIN, typename TOUT>
__global__ __launch_bounds__(256) void nm_conv_kernel(const ConvParams p)
{
    constexpr int SP = BP + 4;            // LDS row stride (floats); rows stay 16-byte aligned
    constexpr int BPW = BP / WP;          // pixels per wavefront
    constexpr int NSEG = BPW / 64;        // 64-pixel segments per wavefront
    constexpr int NBLK = NSEG * 4;        // 16-pixel MFMA blocks per wavefront
    constexpr int WC = 4 / WP;            // wavefronts along the row-block axis
    constexpr int ROWB = SPC < 4 ? 4 : SPC;
    constexpr int ES = (int)sizeof(TIN);
    static_assert(BPW % 64 == 0 && NSEG >= 1, "a wavefront owns whole 64-pixel segments");

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
    const int cblock = logical % p.n_cblocks;
    const int ptile = logical / p.n_cblocks;
    const int p0 = ptile * BP;

    const int wpx = wave % WP;            // position along pixels
    const int wcx = wave / WP;            // position along row blocks
    const int rb0 = (cblock * WC + wcx) * NJ;
    const int wpix = wpx * BPW;

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(p.x), 0, (int)p.x_bytes, 0x00020000);
    const TIN* const xtag = nullptr;

    // ---- staging geometry -------------------------------------------------
    // vector mode: item = (pixel, 4-channel quad); a thread keeps the same quad
    // and NIT pixels.  scalar mode: a thread keeps one pixel and walks rows.
    constexpr int QPR = CK / 4;
    constexpr int NIT = VEC ? (BP * QPR) / 256 : 1;
    constexpr int PSTEP = 256 / QPR;
    static_assert(!VEC || (BP * QPR) % 256 == 0, "staging items must divide evenly");
    static_assert(VEC || (256 % BP == 0 || BP % 256 == 0), "scalar staging keeps one pixel per thread");
    constexpr int NITS = VEC ? 1 : (BP * CK) / 256;   // scalar items per thread
    constexpr int RSTEP = BP >= 256 ? 1 : 256 / BP;

    const int quad = tid % QPR;
    const int pl0 = VEC ? tid / QPR : tid % BP;
    const int r0s = BP >= 256 ? 0 : __builtin_amdgcn_readfirstlane(tid / BP);
    int hi0[NIT], wi0[NIT];
    unsigned base[NIT];                   // byte offset of (b, hi0, wi0, quad*4); may wrap, used only with valid taps
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int pp = p0 + pl0 + it * PSTEP;
        if (pp < p.P) {
            const int b = pp / HoWo;
            const int rem = pp - b * HoWo;
            const int ho = rem / p.Wo;
            const int wo = rem - ho * p.Wo;
            hi0[it] = ho * p.sh - p.ph;
            wi0[it] = wo * p.sw - p.pw;
            base[it] = (unsigned)(((b * p.H + hi0[it]) * p.W + wi0[it]) * p.Cin + (VEC ? quad * 4 : 0)) * ES;
        } else {
            hi0[it] = -(1 << 28);   // every tap lands outside the image
            wi0[it] = 0;
            base[it] = 0;
        }
    }

    constexpr int NST = VEC ? NIT : NITS;   // staging items per thread and chunk
    f4 st[VEC ? NIT : 1];
    float sts[VEC ? 1 : NITS];

    // Fetch iterator: the chunk that the next fetch brings in, as (chunk id, tap
    // row, tap column, first channel); it runs two chunks ahead of the
    // contraction and stays on the last chunk once it gets there.
    int f_c = 0, f_kh = 0, f_kw = 0, f_ci0 = 0;
    auto fetch_item = [&](int it) {
        if constexpr (VEC) {
            const int dhh = f_kh * p.dh, dww = f_kw * p.dw;
            const unsigned choff = (unsigned)((dhh * p.W + dww) * p.Cin + f_ci0) * ES;
            const bool cok = f_ci0 + quad * 4 < p.Cin;
            const int hi = hi0[it] + dhh, wi = wi0[it] + dww;
            const bool inb = cok & ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            st[it] = buf_load4(xr, inb ? base[it] + choff : kOOB, xtag);
        } else {
            const int r = r0s + it * RSTEP;
            const int k = f_c * CK + r;
            const int tap = k / p.Cin;
            const int ci = k - tap * p.Cin;
            const int kh = tap / p.Kw;
            const int kw = tap - kh * p.Kw;
            const int dhh = kh * p.dh, dww = kw * p.dw;
            const int hi = hi0[0] + dhh, wi = wi0[0] + dww;
            const bool inb = (k < p.K) & ((unsigned)hi < (unsigned)p.H) & ((unsigned)wi < (unsigned)p.W);
            const unsigned off = base[0] + (unsigned)((dhh * p.W + dww) * p.Cin + ci) * ES;
            sts[it] = buf_load1(xr, inb ? off : kOOB, xtag);
        }
    };
    auto fetch_advance = [&]() {
        const int adv = f_c + 1 < p.nchunks ? 1 : 0;
        f_c += adv;
        if constexpr (VEC) {
            const int nci = f_ci0 + CK;
            const int wrap = (adv && nci >= p.Cin) ? 1 : 0;
            f_ci0 = wrap ? 0 : (adv ? nci : f_ci0);
            const int nkw = f_kw + wrap;
            const int wrap2 = nkw == p.Kw ? 1 : 0;
            f_kw = wrap2 ? 0 : nkw;
            f_kh += wrap2;
        }
    };
    auto stash_item = [&](int it, int buf) {
        float* dst = lds + buf * (CK * SP);
        if constexpr (VEC) {
            float* d = dst + (quad * 4) * SP + pl0 + it * PSTEP;
            d[0] = st[it].x;
            d[SP] = st[it].y;
            d[2 * SP] = st[it].z;
            d[3 * SP] = st[it].w;
        } else {
            dst[(r0s + it * RSTEP) * SP + pl0] = sts[it];
        }
    };

    // ---- operand streams ----------------------------------------------------
    // A wavefront whose row blocks lie beyond the last one still takes part in
    // staging and barriers; it computes on a clamped row block and stores nothing.
    const float* wfp[NJ];
    const unsigned char* rwp[NJ];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        int rb = rb0 + jj;
        if (rb >= p.n_rowblocks) rb = p.n_rowblocks - 1;
        const int j = rb / p.rbpt;
        wfp[jj] = p.wfrag + ((size_t)rb * p.nchunks * 64 + lane) * SPC;
        rwp[jj] = p.rows + ((size_t)j * p.nchunks * 4 + q) * ROWB;
    }

    f4 acc[NJ][NBLK];
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) acc[jj][b] = f4{0.f, 0.f, 0.f, 0.f};

    StepOps<SPC> cur[NJ], nxt[NJ];

    // Prologue: operands of chunk 0, strip of chunk 0 into LDS, strip of chunk 1
    // into registers.  The operand loads go out first so that the wait for the
    // strip also covers them.
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) load_ops<SPC>(cur[jj], wfp[jj], rwp[jj]);
#pragma unroll
    for (int it = 0; it < NST; ++it) fetch_item(it);
    fetch_advance();
#pragma unroll
    for (int it = 0; it < NST; ++it) stash_item(it, 0);
#pragma unroll
    for (int it = 0; it < NST; ++it) fetch_item(it);
    fetch_advance();
    __syncthreads();

    constexpr int TOT = NJ * SPC;          // k-steps per chunk for this wavefront
    constexpr int DEPTH = NSEG == 1 ? 2 : 1;   // LDS reads run this many k-steps ahead
    constexpr int RING = DEPTH + 1;
    constexpr int NM = TOT * NBLK;         // MFMAs per chunk for this wavefront
    // Staging work of one iteration, cut into tasks that are dealt out behind the
    // MFMAs: write item i of the strip held in registers to LDS, fetch item i of
    // the strip two chunks ahead, load the operands of the next chunk, advance.
    constexpr int NTASK = 2 * NST + NJ + 1;

    // Steady state, one iteration per chunk c, no branch inside:
    //   registers `st` (chunk c+1, fetched one iteration ago) go to the other LDS
    //   buffer; the fetch of chunk c+2 and the operands of chunk c+1 are issued;
    //   chunk c is contracted out of LDS.  Past the last chunk the same code
    //   re-fetches the last chunk and writes it to the buffer nobody reads.
    for (int c = 0; c < p.nchunks; ++c) {
        const int cn = c + 1 < p.nchunks ? c + 1 : c;
        const int nb = (c + 1) & 1;
        auto task = [&](int i) {
            if (i < NST) {
                stash_item(i, nb);
            } else if (i < 2 * NST) {
                fetch_item(i - NST);
            } else if (i < 2 * NST + NJ) {
                const int jj = i - 2 * NST;
                load_ops<SPC>(nxt[jj], wfp[jj] + (size_t)cn * 64 * SPC, rwp[jj] + (size_t)cn * 4 * ROWB);
            } else {
                fetch_advance();
            }
        };

        const float* buf = lds + (c & 1) * (CK * SP) + wpix + n * 4;
        f4 bv[RING][NSEG];
        auto read_b = [&](int t, f4 (&dst)[NSEG]) {
            const int jj = t / SPC, s = t % SPC;
            const unsigned ro = (cur[jj].rw[s >> 2] >> (8 * (s & 3))) & 0xffu;
            const float* bp = buf + ro * SP;
#pragma unroll
            for (int seg = 0; seg < NSEG; ++seg) dst[seg] = *reinterpret_cast<const f4*>(bp + seg * 64);
        };
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
                acc[jj][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bv[t % RING][b >> 2][b & 3], acc[jj][b], 0, 0, 0);
                // a slice of the staging work issues while this MFMA occupies the matrix pipe
#pragma unroll
                for (int i = m * NTASK / NM; i < (m + 1) * NTASK / NM; ++i) task(i);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) cur[jj] = nxt[jj];
        __syncthreads();
    }

    // ---- epilogue: bias, ReLU, cast, NHWC store ------------------------------
    TOUT* __restrict__ y = reinterpret_cast<TOUT*>(p.y);
    const bool fast = (p.tile % 4 == 0) && (p.Cout % 4 == 0);
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
            f4 bb = {0.f, 0.f, 0.f, 0.f};
            if (p.bias) bb = *reinterpret_cast<const f4*>(p.bias + co);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int pp = p0 + wpix + (b >> 2) * 64 + n * 4 + (b & 3);
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
                const int pp = p0 + wpix + (b >> 2) * 64 + n * 4 + (b & 3);
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

template <int BP, int WP, int NJ, int CK, int SPC, bool VEC, typename TIN, typename TOUT>
int launch_t(const ConvParams& p, hipStream_t s)
{
    auto kern = nm_conv_kernel<BP, WP, NJ, CK, SPC, VEC, TIN, TOUT>;
    constexpr size_t lds = (size_t)2 * CK * (BP + 4) * sizeof(float);
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
