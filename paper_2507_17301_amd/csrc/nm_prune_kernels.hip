// Pruning, packing and operand-table kernels (gfx950).
//
// Column-wise N:M selection with L1-norm importance (paper section 3.1), the
// compressed weight + index array (section 2.1, inputs of Alg. 1), and the
// repacking of both into the order the convolution kernel consumes.
#include "nm_internal.h"

namespace nm {

namespace {

constexpr int kPruneThreads = 256;

// One workgroup handles `gpb` groups of one column tile (gpb*M columns, or one
// group of M > 256 columns).  Per column: L1 norm over the tile's rows in fp64,
// rows ascending (adds only, so the sum is reproducible bit for bit); then the
// rank of the column inside its group (number of columns that beat it, a lower
// index beating an equal norm); ranks < N survive.  Kept positions are written
// ascending.
__global__ __launch_bounds__(kPruneThreads) void prune_select_kernel(
    const float* __restrict__ w, int cout, int K, int N, int M, int T, int G, int gpb,
    int32_t* __restrict__ idx)
{
    extern __shared__ double sm_score[];
    const int cols = gpb * M;
    unsigned char* keep = reinterpret_cast<unsigned char*>(sm_score + cols);
    const int j = blockIdx.y;
    const int g0 = blockIdx.x * gpb;
    const int r0 = j * T;
    const int r1 = min(r0 + T, cout);

    for (int i = threadIdx.x; i < cols; i += kPruneThreads) {
        const int lg = i / M, c = i - lg * M;
        const int g = g0 + lg;
        double s = 0.0;
        if (g < G) {
            const float* col = w + (size_t)g * M + c;
            for (int r = r0; r < r1; ++r) s += fabs((double)col[(size_t)r * K]);
        }
        sm_score[i] = s;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cols; i += kPruneThreads) {
        const int lg = i / M, c = i - lg * M;
        const double mine = sm_score[i];
        const double* grp = sm_score + lg * M;
        int rank = 0;
        for (int c2 = 0; c2 < M; ++c2) {
            const double o = grp[c2];
            rank += (o > mine || (o == mine && c2 < c)) ? 1 : 0;
        }
        keep[i] = rank < N ? 1 : 0;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cols; i += kPruneThreads) {
        const int lg = i / M, c = i - lg * M;
        const int g = g0 + lg;
        if (g >= G || !keep[i]) continue;
        const unsigned char* grp = keep + lg * M;
        int pos = 0;
        for (int c2 = 0; c2 < c; ++c2) pos += grp[c2];
        idx[((size_t)j * G + g) * N + pos] = g * M + c;
    }
}

__device__ inline float round_bf16_rne(float v)
{
    unsigned u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xffff0000u);
}

// fp32 -> fp8 E4M3 code (the OCP "e4m3fn" format: bias 7, 3 mantissa bits, subnormals,
// largest value 448), round to nearest, ties to even, in integer arithmetic on the fp32
// bit pattern.  |v| <= 448 here by construction of the weight scale.
__device__ inline unsigned e4m3_code(float v)
{
    const unsigned u = __float_as_uint(v), sign = (u >> 24) & 0x80u;
    const unsigned a = u & 0x7fffffffu;
    const int e = (int)(a >> 23) - 127;            // leading bit at 2^e
    if (a == 0u || e < -10) return sign;           // below half of the smallest step 2^-9
    const unsigned man = (a & 0x7fffffu) | 0x800000u;   // |v| = man * 2^(e - 23)
    const int E = e < -6 ? -6 : e;                 // binade whose spacing 2^(E - 3) applies
    const int shift = 20 + (E - e);                // |v| / 2^(E - 3) = man / 2^shift
    const unsigned q0 = man >> shift, rem = man & ((1u << shift) - 1u), half = 1u << (shift - 1);
    const unsigned q = q0 + ((rem > half || (rem == half && (q0 & 1u))) ? 1u : 0u);
    // normal numbers: q in 8 .. 16, and q = 16 carries into the exponent field by itself;
    // below 2^-6: q in 0 .. 8 is the subnormal's mantissa (8 = the smallest normal)
    return e >= -6 ? sign | (unsigned)(((E + 7) << 3) + (int)q - 8) : sign | q;
}
__device__ inline float e4m3_value(unsigned code)
{
    const int ex = (int)((code >> 3) & 15u), m = (int)(code & 7u);
    const float a = ex == 0 ? ldexpf((float)m, -9) : ldexpf((float)(8 + m), ex - 10);
    return (code & 0x80u) ? -a : a;
}

// kept values -> the E4M3 value they are stored as under the layer's power-of-two scale, in place
__global__ void quantize_e4m3_kernel(float* __restrict__ vals, size_t n, float scale, float inv_scale)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        vals[i] = e4m3_value(e4m3_code(vals[i] * scale)) * inv_scale;
}

// vals[j][kk][t] = w[j*T + t][idx[j][kk]] (zero beyond Cout), optionally
// rounded to bf16.
__global__ void pack_values_kernel(const float* __restrict__ w, const int32_t* __restrict__ idx,
                                   int cout, int K, int kprime, int T, int n_tiles, int to_bf16,
                                   float* __restrict__ vals)
{
    const size_t total = (size_t)n_tiles * kprime * T;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int t = (int)(i % T);
        const size_t jk = i / T;
        const int j = (int)(jk / kprime);
        const int r = j * T + t;
        float v = 0.f;
        if (r < cout) v = w[(size_t)r * K + idx[jk]];
        if (to_bf16) v = round_bf16_rne(v);
        vals[i] = v;
    }
}

__device__ inline void chunk_of(int k, int cin, int CK, int vec, int ncpt, int* c, int* r)
{
    if (vec) {
        const int tap = k / cin, ci = k - tap * cin;
        *c = tap * ncpt + ci / CK;
        *r = ci % CK;
    } else {
        *c = k / CK;
        *r = k % CK;
    }
}

// One workgroup per column tile.  Kept columns are ascending in k, hence
// grouped by chunk; the i-th kept column of a chunk becomes quarter i % 4 of
// k-step i / 4 of that chunk.  Outputs (zero-initialised by the caller):
//   rows [j][c][q][SPC] u32      LDS row (strip_row() in vector mode) of the kept column used by quarter q in step s
//   wfrag[rb][c][lane][SPC]      weight for MFMA A-operand lane (q*16 + t)
// err[0] is set if a chunk holds more than 4*SPC kept columns.
__global__ __launch_bounds__(256) void build_prepack_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ vals, int kprime, int T, int rbpt,
    int cin, int CK, int vec, int ncpt, int nchunks, int SPC, int with_counts,
    uint32_t* __restrict__ rows, float* __restrict__ wfrag, int* __restrict__ err)
{
    extern __shared__ int sm_int[];
    int* cnt = sm_int;             // [nchunks]
    int* first = sm_int + nchunks; // [nchunks]
    const int j = blockIdx.x;
    const int32_t* idxj = idx + (size_t)j * kprime;
    for (int c = threadIdx.x; c < nchunks; c += blockDim.x) cnt[c] = 0;
    __syncthreads();
    for (int kk = threadIdx.x; kk < kprime; kk += blockDim.x) {
        int c, r;
        chunk_of(idxj[kk], cin, CK, vec, ncpt, &c, &r);
        atomicAdd(&cnt[c], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int c = 0; c < nchunks; ++c) {
            first[c] = run;
            run += cnt[c];
            if (cnt[c] > 4 * SPC) err[0] = 1;
        }
    }
    __syncthreads();
    for (int kk = threadIdx.x; kk < kprime; kk += blockDim.x) {
        int c, r;
        chunk_of(idxj[kk], cin, CK, vec, ncpt, &c, &r);
        const int i = kk - first[c];
        const int step = i >> 2, q = i & 3;
        if (step >= SPC) continue;
        rows[(((size_t)j * nchunks + c) * 4 + q) * SPC + step] = (uint32_t)(vec ? strip_row(r, CK) : r);
        for (int sub = 0; sub < rbpt; ++sub) {
            const size_t rb = (size_t)j * rbpt + sub;
            for (int t = 0; t < 16; ++t) {
                const int tt = sub * 16 + t;
                const float v = tt < T ? vals[((size_t)j * kprime + kk) * T + tt] : 0.f;
                wfrag[((rb * nchunks + c) * 64 + q * 16 + t) * SPC + step] = v;
            }
        }
    }
    if (with_counts) {
        // number of k-steps that hold kept columns, in the upper half of each quarter's first word
        __syncthreads();
        for (int i = threadIdx.x; i < nchunks * 4; i += blockDim.x) {
            const int c = i >> 2, q = i & 3;
            rows[(((size_t)j * nchunks + c) * 4 + q) * SPC] |= (uint32_t)((cnt[c] + 3) >> 2) << 16;
        }
    }
}

// The same for the bf16 MFMA kernel: a k-step is 32 kept columns, column i of a
// chunk is element i % 8 of quarter (i % 32) / 8 of step i / 32.  Outputs
// (zero-initialised by the caller):
//   rows [j][c][s][q][8] u32     byte offset (k - k0) * 2 of the column inside the strip's pixel row
//   wfrag[rb][c][s][lane][8]     bf16 weight for MFMA A-operand lane (q*16 + t), element e
__global__ __launch_bounds__(256) void build_prepack16_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ vals, int kprime, int T, int rbpt,
    int cin, int CK, int ncpt, int nchunks, int SPC,
    uint32_t* __restrict__ rows, unsigned short* __restrict__ wfrag, int* __restrict__ err)
{
    extern __shared__ int sm_int[];
    int* cnt = sm_int;
    int* first = sm_int + nchunks;
    const int j = blockIdx.x;
    const int32_t* idxj = idx + (size_t)j * kprime;
    for (int c = threadIdx.x; c < nchunks; c += blockDim.x) cnt[c] = 0;
    __syncthreads();
    for (int kk = threadIdx.x; kk < kprime; kk += blockDim.x) {
        int c, r;
        chunk_of(idxj[kk], cin, CK, 1, ncpt, &c, &r);
        atomicAdd(&cnt[c], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int c = 0; c < nchunks; ++c) {
            first[c] = run;
            run += cnt[c];
            if (cnt[c] > 32 * SPC) err[0] = 1;
        }
    }
    __syncthreads();
    for (int kk = threadIdx.x; kk < kprime; kk += blockDim.x) {
        int c, r;
        chunk_of(idxj[kk], cin, CK, 1, ncpt, &c, &r);
        const int i = kk - first[c];
        const int step = i >> 5, q = (i & 31) >> 3, e = i & 7;
        if (step >= SPC) continue;
        rows[((((size_t)j * nchunks + c) * SPC + step) * 4 + q) * 8 + e] = (uint32_t)r * 2u;
        for (int sub = 0; sub < rbpt; ++sub) {
            const size_t rb = (size_t)j * rbpt + sub;
            for (int t = 0; t < 16; ++t) {
                const int tt = sub * 16 + t;
                const float v = tt < T ? vals[((size_t)j * kprime + kk) * T + tt] : 0.f;
                // the values are already bf16-representable (rounded at pack time): keep the top half
                wfrag[((((rb * nchunks + c) * SPC + step) * 64) + q * 16 + t) * 8 + e] =
                    (unsigned short)(__float_as_uint(v) >> 16);
            }
        }
    }
}

// Operand tables of the gather-free bf16 kernel.  One thread per (row block,
// chunk, k-step, half, lane) writes that lane's 8 A-operand values.
//   sparse: element ea of lane i + 16 qa belongs to the aligned group of 4
//     columns that starts at channel 16 (2 (qa % 2) + ea / 4) + 8 (qa / 2) +
//     4 ((ea % 4) / 2) of the k-step; its two slots take the group's kept
//     columns in ascending order, a group with fewer than two is padded with a
//     zero weight at a free position (positions stay ascending); the 2-bit
//     positions go to field ea of the lane group's index operand.
//   dense: element e of lane i + 16 q, half h is channel 16 q + 8 h + e of the
//     k-step, its weight or 0.
__device__ inline int lower_bound_idx(const int32_t* a, int n, int key)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(256) void build_prepack_sp16_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ vals, int kprime, int T, int rbpt,
    int n_rowblocks, int cin, int CK, int ncpt, int nchunks, int sparse,
    uint32_t* __restrict__ rows, unsigned short* __restrict__ wfrag, int* __restrict__ err)
{
    const int KS = CK / 64, AH = sparse ? 1 : 2;
    const size_t total = (size_t)n_rowblocks * nchunks * KS * AH * 64;
    for (size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
         id += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(id % 64);
        size_t r = id / 64;
        const int h = (int)(r % AH); r /= AH;
        const int s = (int)(r % KS); r /= KS;
        const int c = (int)(r % nchunks);
        const int rb = (int)(r / nchunks);
        const int i = lane & 15, qa = lane >> 4;
        const int j = rb / rbpt, sub = rb - j * rbpt;
        const int t = sub * 16 + i;                       // row inside the column tile
        const int32_t* idxj = idx + (size_t)j * kprime;
        const int tap = c / ncpt, ci0 = (c - tap * ncpt) * CK;
        const int kstep0 = tap * cin + ci0 + s * 64;      // flat k of the k-step's first channel
        unsigned short out[8];
        if (sparse) {
            unsigned fields = 0;
            for (int pair = 0; pair < 4; ++pair) {        // elements 2 pair, 2 pair + 1 share a group
                const int ea = 2 * pair;
                const int k0 = kstep0 + 16 * (2 * (qa % 2) + ea / 4) + 8 * (qa / 2) + 4 * ((ea % 4) / 2);
                const int lb = lower_bound_idx(idxj, kprime, k0);
                int cnt = 0, pos[2] = {0, 0}, kk[2] = {-1, -1};
                for (int u = lb; u < kprime && idxj[u] < k0 + 4; ++u) {
                    if (cnt < 2) { pos[cnt] = idxj[u] - k0; kk[cnt] = u; }
                    ++cnt;
                }
                if (cnt > 2) err[0] = 1;
                if (cnt == 0) {
                    pos[0] = 0; pos[1] = 1;
                } else if (cnt == 1) {
                    if (pos[0] == 3) { pos[1] = 3; kk[1] = kk[0]; pos[0] = 0; kk[0] = -1; }
                    else pos[1] = 3;
                }
                for (int e = 0; e < 2; ++e) {
                    float v = 0.f;
                    if (kk[e] >= 0 && t < T) v = vals[((size_t)j * kprime + kk[e]) * T + t];
                    out[ea + e] = (unsigned short)(__float_as_uint(v) >> 16);   // already bf16-representable
                }
                fields |= (unsigned)(pos[0] | (pos[1] << 2)) << (4 * pair);
            }
            if (i == 0 && sub == 0) rows[(((size_t)j * nchunks + c) * 4 + qa) * KS + s] = fields;
        } else {
            for (int e = 0; e < 8; ++e) {
                const int k = kstep0 + 16 * qa + 8 * h + e;
                const int lb = lower_bound_idx(idxj, kprime, k);
                float v = 0.f;
                if (lb < kprime && idxj[lb] == k && t < T) v = vals[((size_t)j * kprime + lb) * T + t];
                out[e] = (unsigned short)(__float_as_uint(v) >> 16);
            }
        }
        unsigned short* dst = wfrag + id * 8;
        for (int e = 0; e < 8; ++e) dst[e] = out[e];
    }
}

// Operand table of the kernel-row-run kernel: element E = 64 s + 16 q + 8 h + e of
// a pixel's padded K axis is position E % (8 GR) - par of the run of kernel row
// E / (8 GR); positions outside [0, Kw*Cin) and rows >= Kh are padding (weight 0).
__global__ __launch_bounds__(256) void build_prepack_run16_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ vals, int kprime, int T, int rbpt,
    int n_rowblocks, int Kh, int KwC, int KS, int GR, int par, unsigned short* __restrict__ wfrag)
{
    const size_t total = (size_t)n_rowblocks * KS * 2 * 64;
    for (size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
         id += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(id % 64);
        size_t r = id / 64;
        const int h = (int)(r % 2); r /= 2;
        const int s = (int)(r % KS);
        const int rb = (int)(r / KS);
        const int i = lane & 15, q = lane >> 4;
        const int j = rb / rbpt, sub = rb - j * rbpt;
        const int t = sub * 16 + i;
        const int32_t* idxj = idx + (size_t)j * kprime;
        unsigned short* dst = wfrag + id * 8;
        for (int e = 0; e < 8; ++e) {
            const int E = 64 * s + 16 * q + 8 * h + e;
            const int kh = E / (8 * GR);
            const int pos = E - kh * 8 * GR - par;
            float v = 0.f;
            if (kh < Kh && pos >= 0 && pos < KwC && t < T) {
                const int k = kh * KwC + pos;
                const int lb = lower_bound_idx(idxj, kprime, k);
                if (lb < kprime && idxj[lb] == k) v = vals[((size_t)j * kprime + lb) * T + t];
            }
            dst[e] = (unsigned short)(__float_as_uint(v) >> 16);
        }
    }
}

__global__ void build_mask_kernel(const int32_t* __restrict__ idx, int cout, int K, int kprime,
                                  int T, int n_tiles, unsigned char* __restrict__ mask)
{
    const size_t total = (size_t)n_tiles * kprime * T;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int t = (int)(i % T);
        const size_t jk = i / T;
        const int j = (int)(jk / kprime);
        const int r = j * T + t;
        if (r < cout) mask[(size_t)r * K + idx[jk]] = 1;
    }
}

__device__ inline unsigned hash32(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

__global__ void fill_random_kernel(void* dst, size_t n, int bf16, unsigned seed)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
        const unsigned h = hash32((unsigned)i * 2654435761u + seed);
        const float v = (float)(h >> 8) * (1.0f / 16777216.0f);   // [0,1)
        if (bf16 == 2)
            reinterpret_cast<unsigned char*>(dst)[i] = (unsigned char)e4m3_code(v);
        else if (bf16)
            reinterpret_cast<unsigned short*>(dst)[i] =
                (unsigned short)(__float_as_uint(round_bf16_rne(v)) >> 16);
        else
            reinterpret_cast<float*>(dst)[i] = v;
    }
}

// Operand table of the fp8 kernel (dense instruction on zero-filled weights): one thread per
// (row block, 64-channel chunk, lane) writes that lane's 16 A-operand bytes: byte e of lane
// i + 16 q is channel 16 q + e of the chunk (bytes 0-7 feed the first 16x16x32 instruction of
// the k-step, bytes 8-15 the second), the weight's E4M3 code under the layer's scale, or 0.
__global__ __launch_bounds__(256) void build_prepack_f8_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ vals, int kprime, int T, int rbpt,
    int n_rowblocks, int cin, int ncpt, int nchunks, float scale, unsigned char* __restrict__ wfrag)
{
    const size_t total = (size_t)n_rowblocks * nchunks * 64;
    for (size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
         id += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(id % 64);
        const size_t r = id / 64;
        const int c = (int)(r % nchunks), rb = (int)(r / nchunks);
        const int i = lane & 15, q = lane >> 4;
        const int j = rb / rbpt, t = (rb - j * rbpt) * 16 + i;
        const int32_t* idxj = idx + (size_t)j * kprime;
        const int tap = c / ncpt, k0 = tap * cin + (c - tap * ncpt) * 64 + 16 * q;
        unsigned w4[4] = {0u, 0u, 0u, 0u};
        for (int e = 0; e < 16; ++e) {
            const int k = k0 + e;
            const int lb = lower_bound_idx(idxj, kprime, k);
            float v = 0.f;
            if (lb < kprime && idxj[lb] == k && t < T) v = vals[((size_t)j * kprime + lb) * T + t];
            w4[e >> 2] |= e4m3_code(v * scale) << (8 * (e & 3));
        }
        unsigned* dst = reinterpret_cast<unsigned*>(wfrag + id * 16);
        dst[0] = w4[0]; dst[1] = w4[1]; dst[2] = w4[2]; dst[3] = w4[3];
    }
}

int grid_for(size_t total, int threads)
{
    size_t g = (total + threads - 1) / threads;
    if (g > 65535u * 16u) g = 65535u * 16u;
    if (g < 1) g = 1;
    return (int)g;
}

}  // namespace

int run_prune(const float* d_w, nm_packed* wp, hipStream_t s)
{
    const int M = wp->m;
    const int gpb = M <= kPruneThreads ? kPruneThreads / M : 1;
    const size_t lds = (size_t)gpb * M * (sizeof(double) + 1);
    if (lds > 64 * 1024) {
        NM_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(prune_select_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    dim3 grid((wp->G + gpb - 1) / gpb, wp->n_tiles);
    hipLaunchKernelGGL(prune_select_kernel, grid, dim3(kPruneThreads), lds, s, d_w, wp->cout,
                       wp->K, wp->n, M, wp->tile, wp->G, gpb, wp->d_idx);
    NM_HIP_CHECK(hipGetLastError());
    const size_t total = (size_t)wp->n_tiles * wp->kprime * wp->tile;
    hipLaunchKernelGGL(pack_values_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s, d_w,
                       wp->d_idx, wp->cout, wp->K, wp->kprime, wp->tile, wp->n_tiles,
                       wp->value_dtype == NM_BF16 ? 1 : 0, wp->d_vals);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_build_prepack(nm_packed* wp, Prepack& pp, hipStream_t s)
{
    const ChunkGeom& g = pp.geom;
    int* d_err = nullptr;
    NM_HIP_CHECK(hipMalloc(&d_err, sizeof(int)));
    NM_HIP_CHECK(hipMemsetAsync(d_err, 0, sizeof(int), s));
    const size_t lds = (size_t)2 * g.nchunks * sizeof(int);
    if (pp.kind == 6 || pp.kind == 7) {
        // the table is made of 64-channel k-steps whatever the variant's chunk size
        const int ncpt64 = wp->cin / 64, nk64 = wp->K / 64;
        const size_t total = (size_t)wp->n_rowblocks * nk64 * 64;
        hipLaunchKernelGGL(build_prepack_f8_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s, wp->d_idx,
                           wp->d_vals, wp->kprime, wp->tile, wp->rbpt, wp->n_rowblocks, wp->cin, ncpt64,
                           nk64, wp->scale, reinterpret_cast<unsigned char*>(pp.d_wfrag));
    } else if (pp.kind == 0 || pp.kind == 5)
        hipLaunchKernelGGL(build_prepack_kernel, dim3(wp->n_tiles), dim3(256), lds, s, wp->d_idx,
                           wp->d_vals, wp->kprime, wp->tile, wp->rbpt, wp->cin, g.CK, g.vec, g.ncpt,
                           g.nchunks, pp.SPC, pp.kind == 5 ? 1 : 0, pp.d_rows, pp.d_wfrag, d_err);
    else if (pp.kind == 4) {
        const int KwC = wp->kw * wp->cin, GR = (pp.par + KwC + 7) / 8;
        const size_t total = (size_t)wp->n_rowblocks * pp.SPC * 2 * 64;
        hipLaunchKernelGGL(build_prepack_run16_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s,
                           wp->d_idx, wp->d_vals, wp->kprime, wp->tile, wp->rbpt, wp->n_rowblocks, wp->kh,
                           KwC, pp.SPC, GR, pp.par, reinterpret_cast<unsigned short*>(pp.d_wfrag));
    } else if (pp.kind >= 2) {
        const size_t total = (size_t)wp->n_rowblocks * g.nchunks * pp.SPC * (pp.kind == 2 ? 1 : 2) * 64;
        hipLaunchKernelGGL(build_prepack_sp16_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s,
                           wp->d_idx, wp->d_vals, wp->kprime, wp->tile, wp->rbpt, wp->n_rowblocks, wp->cin,
                           g.CK, g.ncpt, g.nchunks, pp.kind == 2 ? 1 : 0, pp.d_rows,
                           reinterpret_cast<unsigned short*>(pp.d_wfrag), d_err);
    } else
        hipLaunchKernelGGL(build_prepack16_kernel, dim3(wp->n_tiles), dim3(256), lds, s, wp->d_idx,
                           wp->d_vals, wp->kprime, wp->tile, wp->rbpt, wp->cin, g.CK, g.ncpt, g.nchunks,
                           pp.SPC, pp.d_rows, reinterpret_cast<unsigned short*>(pp.d_wfrag), d_err);
    hipError_t e = hipGetLastError();
    int h_err = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&h_err, d_err, sizeof(int), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(d_err);
    if (e != hipSuccess) {
        set_error("build_prepack failed: %s", hipGetErrorString(e));
        return NM_ERR_HIP;
    }
    if (h_err) {
        set_error("internal: a K chunk holds more kept columns than the operand table allows");
        return NM_ERR_UNSUPPORTED;
    }
    return NM_OK;
}

int run_quantize_e4m3(nm_packed* wp, hipStream_t s)
{
    const size_t n = (size_t)wp->n_tiles * wp->kprime * wp->tile;
    hipLaunchKernelGGL(quantize_e4m3_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, wp->d_vals, n, wp->scale,
                       1.0f / wp->scale);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_build_mask(const nm_packed* wp, unsigned char* d_mask, hipStream_t s)
{
    NM_HIP_CHECK(hipMemsetAsync(d_mask, 0, (size_t)wp->cout * wp->K, s));
    const size_t total = (size_t)wp->n_tiles * wp->kprime * wp->tile;
    hipLaunchKernelGGL(build_mask_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s, wp->d_idx,
                       wp->cout, wp->K, wp->kprime, wp->tile, wp->n_tiles, d_mask);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_fill_random(void* d, size_t n_elems, nm_dtype_t dt, uint32_t seed, hipStream_t s)
{
    hipLaunchKernelGGL(fill_random_kernel, dim3(grid_for(n_elems, 256)), dim3(256), 0, s, d,
                       n_elems, dt == NM_BF16 ? 1 : (dt == NM_F8E4M3 ? 2 : 0), seed);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

}  // namespace nm
