/*
 * nm_conv.h -- C ABI of libnmconv: 2-D convolution with column-wise,
 * tile-level N:M pruned weights on one MI355X (gfx950).
 *
 * The operations follow the paper "Efficient Column-Wise N:M Pruning on
 * RISC-V CPU": column-wise N:M pruning with L1-norm importance (section 3.1,
 * Fig. 3c), the compressed weight + index array (section 2.1, inputs of
 * Alg. 1), the tiled contraction over the kept columns (Alg. 1), the fused
 * im2col + data packing that feeds it (section 3.2, Alg. 2) and the
 * profile-every-candidate tuning of the kernel parameters (section 3.3).
 * Bias, ReLU, stride/padding/dilation and bf16 follow their usual definitions.
 *
 * Notation: x[B][H][W][Cin] (NHWC); w[Cout][Kh][Kw][Cin] (OHWI) read as the
 * matrix W[Cout][K], K = Kh*Kw*Cin, k = (kh*Kw + kw)*Cin + ci; T = tile size
 * (output channels per column tile); G = K/M groups; K' = G*N kept columns
 * per tile; n_tiles = ceil(Cout/T).
 *
 * All functions return NM_OK (0) or a negative nm_status_t; no exception
 * crosses this boundary.  nm_last_error() returns a thread-local description
 * of the last failure on the calling thread.  Every function that touches the
 * GPU uses the calling thread's current HIP device.  Without a usable GPU the
 * functions that compute return NM_ERR_HIP: there is no CPU fallback.
 */
#ifndef NM_CONV_H
#define NM_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NM_OK = 0,
    NM_ERR_ARG = -1,         /* null pointer, n < 1, n > m, tile < 1, K % m != 0, non-finite weight, ... */
    NM_ERR_SHAPE = -2,       /* output height or width < 1, a tensor of more than 2^31 - 1 elements, or x of 2 GiB or more */
    NM_ERR_UNSUPPORTED = -3, /* no GPU kernel for this tile size / dtype pair / variant id */
    NM_ERR_ALLOC = -4,       /* host or device allocation failed */
    NM_ERR_HIP = -5,         /* a HIP call failed (no device, launch failure, ...) */
    NM_ERR_IO = -6           /* cache file could not be read or written */
} nm_status_t;

/* Element types.  A plain int at the boundary, so that a caller's out-of-range
 * value is an NM_ERR_ARG and not undefined behaviour inside the library. */
typedef int nm_dtype_t;
enum { NM_F32 = 0, NM_BF16 = 1,
       NM_F8E4M3 = 2   /* fp8, 4 exponent bits (bias 7), 3 mantissa bits, subnormals, no infinity, largest
                          value 448 (the OCP "e4m3fn" format); one byte per element */
};

/* Packed, pruned weights of one layer.  Opaque, owned by the library, immutable
 * after creation, bound to the device that was current in nm_prune. */
typedef struct nm_packed nm_packed_t;

const char* nm_last_error(void);

/* Number of kernel variants the tuner chooses from (ids 0 .. count-1), and a
 * short static description of one ("NB8_WP1_NJ2_CK32_SPC4_V1").  NULL for a bad id. */
int nm_variant_count(void);
const char* nm_variant_name(int variant);

/*
 * nm_prune -- column-wise N:M pruning (section 3.1) and packing (section 2.1).
 *
 * For every tile j of `tile` consecutive output channels (the last tile may be
 * shorter) and every group g of m consecutive k, the L1 norm of each column
 * over the tile's existing rows is accumulated in fp64 in ascending row order;
 * the n columns with the largest norm are kept, the lower k winning among
 * equal norms; exactly n are kept even if a kept column is all zero.  Kept
 * values are compacted to vals[j][g*n + i][t] (zero for rows beyond Cout) and
 * the kept absolute k stored ascending in idx[j][g][i].  n == m keeps
 * everything (dense layer).  Selection, compaction and the repacking into the
 * kernels' operand order all run on the GPU.
 *
 *   w_ohwi_host  host pointer, [cout][kh][kw][cin] fp32, caller-owned, only read
 *   value_dtype  NM_F32: values kept as fp32.  NM_BF16: kept values are rounded
 *                to bf16 (nearest even) after selection; selection itself
 *                always uses the fp32 weights.  NM_F8E4M3: kept values are stored
 *                as E4M3 under one power-of-two scale per layer -- the largest
 *                2^e with max|kept w| * 2^e <= 448 -- rounded to nearest even; the
 *                weight the convolution uses is the stored value times 2^-e
 *                (nm_packed_scale returns 2^e; needs cin % 64 == 0, tile % 16 == 0,
 *                cout % 8 == 0)
 *   out          receives the handle; free it with nm_packed_free
 *
 * Errors: NM_ERR_ARG (null, sizes < 1, n > m, (kh*kw*cin) % m != 0, m > 16384,
 * a NaN or infinite weight), NM_ERR_ALLOC, NM_ERR_HIP.  Synchronous.
 */
int nm_prune(const float* w_ohwi_host, int cout, int kh, int kw, int cin,
             int n, int m, int tile, nm_dtype_t value_dtype, nm_packed_t** out);

int nm_packed_free(nm_packed_t* wp);

/* Sizes of the canonical exports below.  Any out pointer may be NULL. */
int nm_packed_dims(const nm_packed_t* wp, int* n_tiles, int* groups, int* n, int* kprime);

/* Canonical exports into caller-allocated host buffers (for checking and for
 * saving pruned weights):
 *   idx  [n_tiles][groups][n] int32, absolute k, ascending
 *   vals [n_tiles][kprime][tile] fp32 (bf16 handles: the rounded values, widened)
 *   mask [cout][K] uint8, 1 = kept                                            */
int nm_packed_indices(const nm_packed_t* wp, int32_t* idx_host);
int nm_packed_values(const nm_packed_t* wp, float* vals_host);
int nm_packed_mask(const nm_packed_t* wp, uint8_t* mask_host);
/* The power-of-two scale of an fp8 handle (1 for fp32 and bf16 handles). */
int nm_packed_scale(const nm_packed_t* wp, float* scale);

/*
 * nm_conv2d -- y = relu?( conv(x, W_pruned) + bias ), computed as the
 * contraction of Alg. 1 over the kept columns only:
 *   y[p][j*T + t] = sum_{kk < K'} A[idx[j][kk]][p] * vals[j][kk][t] + bias
 * where A[k][p] is the im2col matrix of section 2.2 (zero outside the image),
 * p = (b*Hout + ho)*Wout + wo.  A is never written to memory: its kept rows
 * are gathered from x into on-chip storage inside the kernel (the fused
 * im2col + packing of section 3.2).
 *
 *   x_dev     device pointer, NHWC [b][h][w][cin] of x_dtype, 16-byte aligned,
 *             caller-owned, only read
 *   wp        handle from nm_prune on the same device; its cin must equal cin
 *   bias_dev  device pointer [cout] fp32, or NULL
 *   relu      0 or 1
 *   y_dev     device pointer, NHWC [b][hout][wout][cout] of y_dtype, 16-byte
 *             aligned, caller-allocated, fully overwritten,
 *             hout = (h + 2*pad_h - dil_h*(kh-1) - 1)/stride_h + 1 (same for w)
 *   hip_stream  hipStream_t (NULL = default stream)
 *
 * fp32 inputs are multiplied in fp32 on the matrix cores with fp32
 * accumulation; bf16 inputs are multiplied exactly and accumulated in fp32;
 * bf16 outputs are rounded to nearest even once.  Dtype pairs: fp32 -> fp32,
 * bf16 -> bf16, and E4M3 -> bf16 (x of NM_F8E4M3 with a handle whose values are
 * NM_F8E4M3: products exact, fp32 accumulation, the accumulator scaled back by the
 * handle's 2^-e before bias and activation, bf16 output; no residual dtype other
 * than bf16).  The call only enqueues work
 * on the stream and never synchronises -- with one exception: a K-split variant
 * (name ending in "_S<n>", only ever chosen by the tuner or the test hook) keeps
 * its partial sums in a library-owned workspace per device, and the first call
 * that needs a larger one than exists allocates it (nm_autotune sizes it for the
 * shapes it tunes; under stream capture such a call fails with NM_ERR_ALLOC
 * instead; nm_conv2d_static never allocates).  Calls that overlap on one device
 * and both run a K-split variant race on that workspace.  The kernel variant is
 * the one nm_autotune cached for this shape, else nm_force_variant's, else a
 * deterministic default.  Errors: NM_ERR_ARG, NM_ERR_SHAPE, NM_ERR_UNSUPPORTED,
 * NM_ERR_HIP.
 */
int nm_conv2d(const void* x_dev, nm_dtype_t x_dtype, int b, int h, int w, int cin,
              const nm_packed_t* wp, const float* bias_dev,
              int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
              int relu, void* y_dev, nm_dtype_t y_dtype, void* hip_stream);

/*
 * nm_conv2d_res -- nm_conv2d with a residual input, for the convolution that
 * closes a residual block (the networks of section 4 are ResNets):
 *   y = relu?( conv(x, W_pruned) + bias + residual )
 * The sum is formed in fp32 in the kernel's epilogue, so the block's skip
 * connection costs one extra read of `residual` and no extra pass over y.
 *   residual_dev  device pointer shaped and typed like y ([b][hout][wout][cout]
 *                 of y_dtype), 16-byte aligned, only read, must not overlap y;
 *                 NULL makes the call identical to nm_conv2d
 * Everything else as for nm_conv2d (same variant choice, same tuning cache).
 */
int nm_conv2d_res(const void* x_dev, nm_dtype_t x_dtype, int b, int h, int w, int cin,
                  const nm_packed_t* wp, const float* bias_dev, const void* residual_dev,
                  int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                  int relu, void* y_dev, nm_dtype_t y_dtype, void* hip_stream);

/*
 * nm_conv2d_static -- nm_conv2d_res for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results, same variant choice.  The one thing nm_conv2d may allocate is the
 * workspace for the partial sums of a K-split variant (a variant whose name ends in "_S<n>":
 * n workgroups share the K axis of an output tile; chosen by the tuner for layers with too
 * few output tiles to fill the chip); this entry point keeps those sums in a fixed buffer of
 * 16 MiB that is part of the library's device image instead, and calls no allocating routine.
 * A K-split variant whose partial sums (n * P * cout * 4 bytes) exceed 16 MiB is refused
 * with NM_ERR_SHAPE and a message that names both sizes.  Every call on a GPU shares that
 * GPU's buffer: calls that overlap on one GPU (different streams) race; calls on one stream
 * do not.  Nothing needs to be cleared between calls (every partial sum is written before it
 * is read).
 */
int nm_conv2d_static(const void* x_dev, nm_dtype_t x_dtype, int b, int h, int w, int cin,
                     const nm_packed_t* wp, const float* bias_dev, const void* residual_dev,
                     int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                     int relu, void* y_dev, nm_dtype_t y_dtype, void* hip_stream);

/*
 * The two pooling layers a ResNet needs around its convolutions, so that a whole
 * network can run on device tensors through this library (section 4 measures
 * whole networks).  NHWC, fp32 or bf16 (same dtype in and out), enqueue-only.
 *
 * nm_maxpool2d: y[b][ho][wo][c] = max over the k x k window at stride `stride`
 *   with `pad` rows/columns of padding that never win (windows lie inside the
 *   padded image; hout = (h + 2*pad - k)/stride + 1, same for w).
 * nm_avgpool_global: y[b][c] = mean over all h*w positions (fp32 sum).
 * Errors: NM_ERR_ARG (null, sizes < 1, pad >= k, unknown dtype), NM_ERR_SHAPE
 * (empty output), NM_ERR_HIP.
 */
int nm_maxpool2d(const void* x_dev, nm_dtype_t dtype, int b, int h, int w, int c,
                 int k, int stride, int pad, void* y_dev, void* hip_stream);
int nm_avgpool_global(const void* x_dev, nm_dtype_t dtype, int b, int h, int w, int c,
                      void* y_dev, void* hip_stream);

/*
 * nm_im2col -- the im2col matrix of section 2.2 written out to memory, for the
 * unfused comparison of section 4.3 (im2col and packing as separate passes
 * against the fused kernel).  nm_conv2d never calls it.
 *   a_dev[p][k] = x[b][ho*stride_h - pad_h + kh*dil_h][wo*stride_w - pad_w + kw*dil_w][ci]
 *                 or 0 outside the image,  p = (b*Hout + ho)*Wout + wo,
 *                 k = (kh*kw_ + kw)*cin + ci   (the k order nm_prune uses)
 * so a_dev is the NHWC tensor [b][hout][wout][kh*kw*cin] on which a 1x1
 * convolution with the same weights, read as [cout][1][1][kh*kw*cin], gives
 * the same result.  Same dtype in and out; enqueue-only.
 * Errors: NM_ERR_ARG, NM_ERR_SHAPE, NM_ERR_HIP.
 */
int nm_im2col(const void* x_dev, nm_dtype_t dtype, int b, int h, int w, int cin, int kh, int kw,
              int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
              void* a_dev, void* hip_stream);

/*
 * nm_stream_floor -- a measuring stick, not part of the method: one kernel that reads the
 * first x_bytes of x_dev and writes the first y_bytes of y_dev (whole 16-byte units; a
 * remainder below 16 bytes is left alone), and computes nothing.  Launched with a layer's
 * input and output sizes it shows what the layer's own traffic costs on this device in the
 * same launch sequence -- the part of a layer's time that no convolution kernel can remove
 * (section 3.2 argues from memory traffic; this puts a measured number under it).
 * The contents written to y are unspecified.  Pointers 16-byte aligned; enqueue-only.
 */
int nm_stream_floor(const void* x_dev, size_t x_bytes, void* y_dev, size_t y_bytes, void* hip_stream);

/*
 * nm_autotune -- per-layer choice of the fastest kernel variant (section 3.3:
 * every candidate is run on the target and the fastest kept).  Runs each legal
 * variant for this shape on library-allocated scratch tensors (pseudo-random
 * input; a ring of input/output sets of about 768 MB so that, as inside a
 * network, no launch finds its tensors in the last-level cache), times it with
 * HIP events on `hip_stream`, stores the winner in the process-wide cache keyed
 * by (shape, N:M, T, dtypes, bias / activation flags, the device's architecture and CU
 * count, and which operand tables the handle carries -- layers of one shape whose
 * kept sets need different k-steps per chunk do not share an entry) and returns it.
 * Synchronous.  A cached shape returns immediately with the cached result.
 * With the environment variable NM_TUNE_VERBOSE set, the time of every candidate
 * is printed to stderr, fastest first.
 *   chosen_variant, best_ms   may be NULL
 */
int nm_autotune(nm_dtype_t x_dtype, int b, int h, int w, int cin,
                const nm_packed_t* wp, int has_bias,
                int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                int relu, nm_dtype_t y_dtype, void* hip_stream,
                int* chosen_variant, float* best_ms);

/*
 * nm_autotune_tile -- the tuner also chooses the tile size T (section 3.3 spans
 * T in [1, 32]; the accuracy study of section 4.4 has a configuration whose T is
 * picked per layer by profiling).  For every candidate T the weights are pruned
 * at that T (nm_prune) and the convolution is tuned for the given shape
 * (nm_autotune, which also caches the variant); the handle of the fastest
 * candidate is returned and the others are freed.  T changes which weights
 * survive, so the candidates are different models: the choice is a
 * deployment-time trade that the paper pairs with retraining.
 *   w_host .. m, value_dtype   as nm_prune
 *   tiles[n_candidates]        host array of candidate T, tried in order (ties keep the earlier)
 *   x_dtype .. hip_stream      as nm_autotune
 *   out                        receives the winning handle, owned by the caller (nm_packed_free)
 *   best_tile                  may be NULL
 *   ms_per_candidate           host array [n_candidates] of each candidate's best time, or NULL
 * Synchronous.  Any error of nm_prune or nm_autotune for any candidate fails the
 * call and frees every handle; *out is then NULL.
 */
int nm_autotune_tile(const float* w_host, int cout, int kh, int kw, int cin, int n, int m,
                     const int* tiles, int n_candidates, nm_dtype_t value_dtype,
                     nm_dtype_t x_dtype, int b, int h, int w, int has_bias,
                     int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                     int relu, nm_dtype_t y_dtype, void* hip_stream,
                     nm_packed_t** out, int* best_tile, float* ms_per_candidate);

/* Frees the workspaces that K-split variants grew (one per device that ran one); the next
 * call that needs one allocates it again.  Waits for the kernels still using them. */
int nm_workspace_free(void);

/* Tuning cache: text file, one line per entry; the first line names the device it was
 * written on.  Loading merges into the cache; entries made on another kind of device
 * are kept but never match. */
int nm_cache_save(const char* path);
int nm_cache_load(const char* path);
int nm_cache_clear(void);
int nm_cache_size(void);

/* Test hook: variant >= 0 makes every nm_conv2d use that variant (an illegal
 * one for a shape gives NM_ERR_UNSUPPORTED); -1 restores the normal choice. */
int nm_force_variant(int variant_or_minus1);

/* The variant id the calling thread's last successful nm_conv2d / nm_conv2d_res launched
 * (-1 before the first): what actually ran, whether it came from the tuning cache, the
 * test hook or the default. */
int nm_last_variant(void);

/* Whether `variant` can run this layer (1), cannot (0), or bad arguments (<0). */
int nm_variant_legal(int variant, const nm_packed_t* wp, nm_dtype_t x_dtype, nm_dtype_t y_dtype);

#ifdef __cplusplus
}
#endif
#endif /* NM_CONV_H */
