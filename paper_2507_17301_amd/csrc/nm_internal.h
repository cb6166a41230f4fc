// Internal declarations shared by the translation units of libnmconv.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <string>
#include <vector>

#include "nm_conv.h"

namespace nm {

void set_error(const char* fmt, ...);

#define NM_HIP_CHECK(expr)                                                        \
    do {                                                                          \
        hipError_t e__ = (expr);                                                  \
        if (e__ != hipSuccess) {                                                  \
            nm::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), \
                          __FILE__, __LINE__);                                    \
            return NM_ERR_HIP;                                                    \
        }                                                                         \
    } while (0)

// ---------------------------------------------------------------------------
// K chunking.  The K axis is cut into chunks of at most CK consecutive k; one
// chunk of the im2col matrix (rows k0 .. k0+len-1, all pixels of the
// workgroup's pixel tile) is resident in LDS at a time.
//   vector mode (Cin % 4 == 0): a chunk never crosses a kernel tap, so it is
//     `len` consecutive input channels of one tap and is fetched with 16-byte
//     loads.  ncpt = ceil(Cin / CK) chunks per tap.
//   scalar mode (any Cin): chunks are cut on the flat k axis.
// ---------------------------------------------------------------------------
struct ChunkGeom {
    int vec;      // 1 = vector mode
    int CK;       // rows per chunk
    int ncpt;     // chunks per tap (vector mode)
    int nchunks;  // total
};

inline ChunkGeom make_chunk_geom(int cin, int K, int CK, int vec)
{
    ChunkGeom g;
    g.vec = vec;
    g.CK = CK;
    if (vec) {
        g.ncpt = (cin + CK - 1) / CK;
        g.nchunks = (K / cin) * g.ncpt;
    } else {
        g.ncpt = 0;
        g.nchunks = (K + CK - 1) / CK;
    }
    return g;
}

// Operand tables for one chunk geometry (device memory, built once in nm_prune).
// The contraction of one column tile is cut into k-steps of four kept columns
// (the K depth of one 16x16x4 MFMA).  Every chunk owns exactly SPC k-steps per
// tile; the i-th kept column of the chunk is quarter i % 4 of step i / 4, and
// unused slots carry weight 0 and row 0.
struct Prepack {
    int kind = 0;                     // 0: fp32 MFMA kernel, 1: bf16 MFMA gather kernel, 2/3: gather-free bf16 kernel,
                                      // 4: bf16 kernel-row runs, 5: fp32 MFMA kernel with per-chunk step counts,
                                      // 6, 7: fp8 kernels (dense instruction on zero-filled weights), register-streaming
                                      // and LDS-staged
    ChunkGeom geom{};
    int SPC = 0;                      // k-steps per chunk (1, 2, 4 or 8)
    // kind 0: a k-step is 4 kept columns
    //   d_rows  [n_tiles][nchunks][4][SPC] u32        LDS row (k - k0) that quarter q reads in step s
    //   d_wfrag [n_rowblocks][nchunks][64][SPC] fp32  MFMA A-operand lane values
    // kind 5: as kind 0 with SPC = CK / 4; bits 16.. of d_rows[j][c][q][0] hold the number of
    //   k-steps that carry kept columns of (tile j, chunk c)
    // kind 1: a k-step is 32 kept columns
    //   d_rows  [n_tiles][nchunks][SPC][4][8] u32     byte offset (k - k0) * 2 of the 8 columns of quarter q
    //   d_wfrag [n_rowblocks][nchunks][SPC][64][8] bf16  MFMA A-operand lane values
    // kind 2 (sparse matrix instruction) and 3 (dense instruction, zero-filled weights):
    //   a k-step is 64 consecutive channels of one tap; SPC = CK / 64
    //   d_rows  [n_tiles][nchunks][4][SPC] u32        kind 2: index operand of lane group q in k-step s
    //   d_wfrag [n_rowblocks][nchunks][SPC][AH][64][8] bf16   A-operand lane values, AH = 1 (kind 2) or 2 (kind 3)
    // kind 4 (contiguous kernel-row runs, layers with very few input channels): one chunk of SPC
    //   64-element k-steps; per pixel Kh runs of GR granules, each starting `par` elements early
    //   d_wfrag [n_rowblocks][SPC][2][64][8] bf16   A-operand lane values, zero in padding slots
    // kind 6 and 7 (fp8 E4M3, dense instruction): a k-step is 64 channels of one tap, a chunk CK / 64 of them
    //   d_wfrag [n_rowblocks][K / 64][64][16] bytes   lane i + 16 q, byte e = channel 16 q + e of the k-step
    int par = 0;                      // kind 4: 0 or 1 elements of lead-in per run (alignment of the run start)
    uint32_t* d_rows = nullptr;
    float* d_wfrag = nullptr;
    size_t rows_bytes = 0, wfrag_bytes = 0;
    uint32_t* d_ktab = nullptr;       // scalar mode only: [nchunks*CK] (kh | kw << 8 | ci << 16) per im2col row
};

// LDS row stride (floats) of the im2col strip: the pixel tile, widened to what
// the staging threads write (a multiple of 16), plus 4.  Rows stay 16-byte
// aligned, and the stride is 4 times an odd number: the 8 (CK = 32) or 16
// (CK = 64) consecutive LDS rows that a wavefront's transposing writes touch
// start in different groups of four banks.
constexpr int strip_stride(int BP, int CK, bool vec)
{
    const int pstep = 256 / (CK / 4);
    const int nit = (BP * (CK / 4) + 255) / 256;
    const int cols = vec && nit * pstep > BP ? nit * pstep : BP;
    return cols + 4;
}

// Vector mode stores im2col row r of a chunk (r = 4 * quad + j) in LDS row j * (CK / 4) + quad.
constexpr int strip_row(int r, int CK) { return (r & 3) * (CK / 4) + (r >> 2); }

}  // namespace nm

struct nm_packed {
    int cout, kh, kw, cin, K;
    int n, m, tile;
    int G, kprime, n_tiles;
    int rbpt;         // 16-row blocks per column tile = ceil(tile / 16)
    int n_rowblocks;  // n_tiles * rbpt
    nm_dtype_t value_dtype;
    int device;
    float scale = 1.f;   // fp8 handles: the stored E4M3 value is weight * scale (a power of two)
    int sig = 0;      // hash of the operand tables built for this handle (part of the tuning-cache key)
    int32_t* d_idx = nullptr;   // [n_tiles][kprime]
    float* d_vals = nullptr;    // [n_tiles][kprime][tile]
    std::vector<int32_t> h_idx; // host copy of d_idx
    std::vector<nm::Prepack> prepacks;
};

namespace nm {

// ---------------------------------------------------------------------------
// Convolution kernel parameters (passed by value).
// ---------------------------------------------------------------------------
struct ConvParams {
    const void* x;
    void* y;
    const float* bias;
    const void* res;        // residual tensor shaped and typed like y, added before the activation, or null
    const float* wfrag;
    const uint32_t* rows;
    const uint32_t* ktab;   // scalar mode: [nchunks*CK] (kh | kw << 8 | ci << 16) of each im2col row
    int B, H, W, Cin, Cout, Kh, Kw, Ho, Wo;
    int sh, sw, ph, pw, dh, dw;
    int relu;
    int P;             // B*Ho*Wo
    int K;
    int nchunks, ncpt;
    int tile, rbpt, n_rowblocks;
    int n_ptiles, n_cblocks, n_wg;   // pixel tiles, row-block groups, product
    int wg_per_xcd;
    // launch-time divisors as multiply-shift pairs (x / d = umulhi(x, mul) >> shift, mul == 0: d == 1)
    unsigned howo_mul, howo_shift, wo_mul, wo_shift;
    int run_gr, run_d; // kind 4: granules per kernel-row run, lead-in elements of a run
    unsigned gr_mul, gr_shift, cin_mul, cin_shift;   // kind 4: multiply-shift pairs for / run_gr and / Cin
    unsigned x_elems;  // elements of x
    unsigned x_bytes;  // size of x in bytes (< 2 GiB), the range of the buffer descriptor
    unsigned wfrag_bytes, rows_bytes;
    // K split (fp32 MFMA kernel): ksplit workgroups share one output tile, each contracts cps
    // chunks and writes its partial sums to partial[split][P][Cout] (fp32); a second kernel adds
    // them up and applies bias, residual and activation.  ksplit <= 1: no split, partial unused.
    float* partial;
    int ksplit, cps;
    float oscale;      // fp8: factor that takes the accumulator back to the weights' own scale (1 / handle scale)
};

struct VariantDesc {
    const char* name;
    int BP;    // pixels per workgroup = 16 * NBLK * WP
    int NBLK;  // 16-pixel MFMA blocks per wavefront
    int WP;    // waves along the pixel axis (the other 4/WP split the row blocks)
    int NJ;    // row blocks (16 output channels each) per wave
    int CK;    // K rows per LDS chunk
    int SPC;   // k-steps per chunk
    int vec;   // chunk mode: 1 = 16-byte channel loads, 0 = element-wise on flat k
    int kind;  // 0 = fp32 MFMA kernel (fp32 or bf16 I/O), 1 = bf16 MFMA gather kernel (bf16 I/O, bf16 weights),
               // 2 = bf16 sparse-matrix-instruction kernel, 3 = bf16 dense kernel on zero-filled weights,
               // 4 = bf16 dense kernel on contiguous kernel-row runs (very few input channels),
               // 5 = fp32 MFMA kernel that runs only the k-steps holding kept columns of each (tile, chunk)
               // 6 = fp8 E4M3 kernel (fp8 activations, bf16 output): dense instruction on zero-filled weights
    int share; // kind 1: row blocks fed from one gathered operand
    int ksplit; // kinds 0, 5: workgroups that share the K axis of one output tile (1 = no split)
    int areg;  // kinds 2, 3, 7: 1 = weights and index words go straight to registers, the LDS stages hold the strip alone
    int spec;  // kinds 2, 3, 7: 1 = four producer wavefronts issue the loads (512 threads)
};

// Allows kernel `fn` more than 64 KB of dynamic LDS on the current device; done once per
// (kernel, device) -- `done` is the caller's per-kernel bit set, one bit per device ordinal.
int allow_lds(const void* fn, size_t bytes, unsigned long long* done);

int variant_count();
const VariantDesc& variant_desc(int v);
// Launches variant v; x/y dtypes select the instantiation.
int launch_conv(int v, nm_dtype_t xdt, nm_dtype_t ydt, const ConvParams& p, hipStream_t s);

// prune-side kernels (nm_prune_kernels.hip)
int run_prune(const float* d_w, nm_packed* wp, hipStream_t s);
int run_build_prepack(nm_packed* wp, Prepack& pp, hipStream_t s);   // any kind
int run_build_mask(const nm_packed* wp, uint8_t* d_mask, hipStream_t s);
int run_quantize_e4m3(nm_packed* wp, hipStream_t s);   // d_vals -> the E4M3 values they are stored as (needs wp->scale)
int run_fill_random(void* d, size_t n_elems, nm_dtype_t dt, uint32_t seed, hipStream_t s);

// pooling kernels (nm_pool_kernels.hip)
int run_maxpool(const void* x, nm_dtype_t dt, int B, int H, int W, int C, int k, int stride, int pad,
                int Ho, int Wo, void* y, hipStream_t s);
int run_avgpool(const void* x, nm_dtype_t dt, int B, int HW, int C, void* y, hipStream_t s);
// adds up the partial sums of a K split: y = act(sum_s partial[s] + bias + residual)
int run_splitk_reduce(const ConvParams& p, nm_dtype_t ydt, hipStream_t s);
// Static scratch of nm_conv2d_static (nm_scratch.hip): device address of the current
// device's copy, looked up once per device; never allocates.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
int static_scratch(int dev, float** out);
int run_stream_floor(const void* x, size_t x_bytes, void* y, size_t y_bytes, hipStream_t s);
int run_im2col(const void* x, nm_dtype_t dt, int B, int H, int W, int C, int Kh, int Kw, int sh, int sw,
               int ph, int pw, int dh, int dw, int Ho, int Wo, void* a, hipStream_t s);

}  // namespace nm
