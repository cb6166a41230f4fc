// The pooling layers between the convolutions of a ResNet: 3x3/2 max pooling
// after the first layer and global average pooling before the classifier.
// Both are plain HBM-bound passes over NHWC tensors: one thread handles 4
// consecutive channels (8 or 16 bytes) of one output position, so that a
// wavefront reads and writes contiguous runs.
#include "nm_conv_kernel.h"

namespace nm {
namespace {

inline int grid_for_items(size_t items)
{
    size_t g = (items + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    return g < 1 ? 1 : (int)g;
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(const T* __restrict__ x, T* __restrict__ y, int B,
                                                      int H, int W, int C, int k, int stride, int pad,
                                                      int Ho, int Wo)
{
    const int C4 = (C + 3) / 4;
    const size_t total = (size_t)B * Ho * Wo * C4;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int c4 = (int)(i % C4);
        size_t r = i / C4;
        const int wo = (int)(r % Wo); r /= Wo;
        const int ho = (int)(r % Ho);
        const int b = (int)(r / Ho);
        const int c0 = c4 * 4;
        const bool vec = (C % 4 == 0);
        f4 m = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        for (int kh = 0; kh < k; ++kh) {
            const int hi = ho * stride - pad + kh;
            if ((unsigned)hi >= (unsigned)H) continue;
            for (int kw = 0; kw < k; ++kw) {
                const int wi = wo * stride - pad + kw;
                if ((unsigned)wi >= (unsigned)W) continue;
                const T* px = x + ((size_t)(b * H + hi) * W + wi) * C + c0;
                if (vec) {
                    const f4 v = load4(px);
                    m.x = fmaxf(m.x, v.x); m.y = fmaxf(m.y, v.y);
                    m.z = fmaxf(m.z, v.z); m.w = fmaxf(m.w, v.w);
                } else {
                    for (int e = 0; e < 4 && c0 + e < C; ++e) m[e] = fmaxf(m[e], load1(px + e));
                }
            }
        }
        T* py = y + ((size_t)(b * Ho + ho) * Wo + wo) * C + c0;
        if (vec) {
            store4(py, m);
        } else {
            for (int e = 0; e < 4 && c0 + e < C; ++e) store1(py + e, m[e]);
        }
    }
}

// one workgroup per (image, 64-channel slab): 4 wavefronts split the positions,
// lanes run along the channels; fp32 partial sums meet in LDS
template <typename T>
__global__ __launch_bounds__(256) void avgpool_kernel(const T* __restrict__ x, T* __restrict__ y, int HW, int C)
{
    __shared__ float part[4][64];
    const int b = blockIdx.y;
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int wv = threadIdx.x >> 6;
    float s = 0.f;
    if (c < C)
        for (int i = wv; i < HW; i += 4) s += load1(x + ((size_t)b * HW + i) * C + c);
    part[wv][threadIdx.x & 63] = s;
    __syncthreads();
    if (wv == 0 && c < C) {
        const float t = ((part[0][threadIdx.x] + part[1][threadIdx.x]) + part[2][threadIdx.x]) + part[3][threadIdx.x];
        store1(y + (size_t)b * C + c, t / (float)HW);
    }
}

// im2col written out: one thread per (pixel, run of V channels of one tap), V elements = 16 bytes
// when the channel count allows, else one element
template <typename T, int V>
__global__ __launch_bounds__(256) void im2col_kernel(const T* __restrict__ x, T* __restrict__ a, int B, int H,
                                                     int W, int C, int Kh, int Kw, int sh, int sw, int ph, int pw,
                                                     int dh, int dw, int Ho, int Wo)
{
    const int CV = C / V;
    const size_t total = (size_t)B * Ho * Wo * Kh * Kw * CV;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int cv = (int)(i % CV);
        size_t r = i / CV;
        const int kw_ = (int)(r % Kw); r /= Kw;
        const int kh_ = (int)(r % Kh); r /= Kh;
        const int wo = (int)(r % Wo); r /= Wo;
        const int ho = (int)(r % Ho);
        const int b = (int)(r / Ho);
        const int hi = ho * sh - ph + kh_ * dh, wi = wo * sw - pw + kw_ * dw;
        const bool in = ((unsigned)hi < (unsigned)H) & ((unsigned)wi < (unsigned)W);
        T* dst = a + i * V;     // (pixel, tap, channel run) is exactly the order of a[p][k]
        if constexpr (V == 1) {
            T z; if constexpr (sizeof(T) == 4) z = 0; else z.v = 0;
            dst[0] = in ? x[((size_t)(b * H + hi) * W + wi) * C + cv] : z;
        } else {
            u4v v = {0u, 0u, 0u, 0u};
            if (in) v = *reinterpret_cast<const u4v*>(x + ((size_t)(b * H + hi) * W + wi) * C + cv * V);
            *reinterpret_cast<u4v*>(dst) = v;
        }
    }
}

// The traffic of a layer and nothing else: read nx 16-byte units, write ny, both spread over
// every thread of the grid in grid-stride order (whole 1 KB runs per wavefront), four loads in
// flight per thread before the first use.  What is read only steers a store that never happens.
__global__ __launch_bounds__(256) void stream_floor_kernel(const u4v* __restrict__ x, size_t nx,
                                                           u4v* __restrict__ y, size_t ny)
{
    const size_t step = (size_t)gridDim.x * blockDim.x;
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned acc = 0;
    size_t i = i0;
    for (; i + 3 * step < nx; i += 4 * step) {
        const u4v a = x[i], b = x[i + step], c = x[i + 2 * step], d = x[i + 3 * step];
        acc += (a.x ^ b.y) + (c.z ^ d.w);
    }
    for (; i < nx; i += step) acc += x[i].x;
    const u4v v = {1u, 2u, 3u, 4u};
    for (size_t j = i0; j < ny; j += step) y[j] = v;
    if (acc == 0x9e3779b9u && ny > 0 && i0 == 0) y[0].x = acc;   // keeps the loads alive
}

// Where the partial sums of a K split meet: one thread per 4 consecutive channels of one
// pixel (or per element when Cout is not a multiple of 4) adds the splits in ascending order,
// then bias, residual, activation, one rounding.
template <typename TOUT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ConvParams p)
{
    const size_t total = (size_t)p.P * p.Cout;
    TOUT* __restrict__ y = reinterpret_cast<TOUT*>(p.y);
    if (p.Cout % 4 == 0) {
        const size_t n4 = total / 4;
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
            f4 v = *reinterpret_cast<const f4*>(p.partial + i * 4);
            for (int s = 1; s < p.ksplit; ++s) v = v + *reinterpret_cast<const f4*>(p.partial + (size_t)s * total + i * 4);
            if (p.bias) v = v + *reinterpret_cast<const f4*>(p.bias + (i * 4) % (size_t)p.Cout);
            emit4(p, y, (unsigned)(i * 4), v);
        }
    } else {
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
            float v = p.partial[i];
            for (int s = 1; s < p.ksplit; ++s) v += p.partial[(size_t)s * total + i];
            if (p.bias) v += p.bias[i % (size_t)p.Cout];
            emit1(p, y, (unsigned)i, v);
        }
    }
}

}  // namespace

int run_splitk_reduce(const ConvParams& p, nm_dtype_t ydt, hipStream_t s)
{
    const size_t total = (size_t)p.P * p.Cout;
    const size_t items = p.Cout % 4 == 0 ? total / 4 : total;
    const int grid = grid_for_items(items);
    if (ydt == NM_F32)
        hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3(grid), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL(splitk_reduce_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, p);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_stream_floor(const void* x, size_t x_bytes, void* y, size_t y_bytes, hipStream_t s)
{
    const size_t nx = x_bytes / 16, ny = y_bytes / 16;
    const size_t most = nx > ny ? nx : ny;
    // enough workgroups to fill every CU several times over, never more threads than units
    int grid = (int)((most + 255) / 256);
    if (grid > 256 * 8) grid = 256 * 8;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(stream_floor_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<const u4v*>(x), nx,
                       reinterpret_cast<u4v*>(y), ny);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_im2col(const void* x, nm_dtype_t dt, int B, int H, int W, int C, int Kh, int Kw, int sh, int sw,
               int ph, int pw, int dh, int dw, int Ho, int Wo, void* a, hipStream_t s)
{
    const int V = dt == NM_F32 ? 4 : 8;
    const bool vec = (C % V == 0);
    const size_t total = (size_t)B * Ho * Wo * Kh * Kw * (vec ? C / V : C);
    const unsigned grid = (unsigned)std::min<size_t>((total + 255) / 256, 1u << 20);
#define NM_IM2COL(T, VV)                                                                                    \
    hipLaunchKernelGGL((im2col_kernel<T, VV>), dim3(grid), dim3(256), 0, s, (const T*)x, (T*)a, B, H, W, C, Kh, \
                       Kw, sh, sw, ph, pw, dh, dw, Ho, Wo)
    if (dt == NM_F32) { if (vec) NM_IM2COL(float, 4); else NM_IM2COL(float, 1); }
    else { if (vec) NM_IM2COL(bf16_t, 8); else NM_IM2COL(bf16_t, 1); }
#undef NM_IM2COL
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_maxpool(const void* x, nm_dtype_t dt, int B, int H, int W, int C, int k, int stride, int pad,
                int Ho, int Wo, void* y, hipStream_t s)
{
    const size_t total = (size_t)B * Ho * Wo * ((C + 3) / 4);
    const unsigned grid = (unsigned)std::min<size_t>((total + 255) / 256, 1u << 20);
    if (dt == NM_F32)
        hipLaunchKernelGGL(maxpool_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)x, (float*)y, B, H,
                           W, C, k, stride, pad, Ho, Wo);
    else
        hipLaunchKernelGGL(maxpool_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, B,
                           H, W, C, k, stride, pad, Ho, Wo);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

int run_avgpool(const void* x, nm_dtype_t dt, int B, int HW, int C, void* y, hipStream_t s)
{
    const dim3 grid((C + 63) / 64, B);
    if (dt == NM_F32)
        hipLaunchKernelGGL(avgpool_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (float*)y, HW, C);
    else
        hipLaunchKernelGGL(avgpool_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, HW, C);
    NM_HIP_CHECK(hipGetLastError());
    return NM_OK;
}

}  // namespace nm
