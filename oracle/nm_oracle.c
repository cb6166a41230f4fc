/*
 * CPU oracle for column-wise, tile-level N:M pruned 2-D convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the GPU library and must never be linked or
 * called from the product path.  Floating point is accumulated in fp64.
 *
 * What it defines (paper section 3.1, Fig. 3c, Alg. 1 inputs; section 2.2):
 *   - the weight tensor w[Cout][Kh][Kw][Cin] (OHWI) is read as a matrix
 *     W[Cout][K], K = Kh*Kw*Cin, k = (kh*Kw + kw)*Cin + ci  (the "filter
 *     matrix" whose rows are flattened kernels);
 *   - rows are cut into tiles of T consecutive output channels; inside a tile
 *     every column (the T weights that share one k) is one pruning unit;
 *   - columns are grouped M at a time along k; in every group the N columns
 *     with the largest L1 norm (sum of |w| over the tile's rows) are kept and
 *     the others are removed for all rows of the tile at once;
 *   - the compressed form is the kept values W'[tile][G*N][T] plus the kept
 *     column positions Idx[tile][G*N];
 *   - the convolution result is by definition the direct convolution with the
 *     pruned-then-zero-filled dense weights (the tiled kernel of Alg. 1 visits
 *     only kept columns, so it reaches exactly this result up to rounding
 *     order).
 *
 * Readings where the paper is silent:
 *   - exactly N columns are kept per group (N = (1 - sparsity) * M);
 *   - the L1 norm is accumulated in double, rows in ascending order;
 *   - equal norms: the lower k wins;
 *   - the last tile may have fewer than T rows (Cout % T != 0): only existing
 *     rows contribute to the norm, packed values are zero padded to T;
 *   - K % M != 0 is rejected.
 *
 * Build:  gcc -O2 -fPIC -shared -pthread -o libnm_oracle.so nm_oracle.c
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)

/* ------------------------------------------------------------------------- */
/* Pruning: section 3.1 (column-wise N:M, L1-norm importance).               */
/* ------------------------------------------------------------------------- */

/*
 * w      [Cout][K] fp32 weight matrix (OHWI flattened).
 * mask   [Cout][K] out, 1 = kept, 0 = pruned.
 * idx    [n_tiles][G][N] out, absolute k of the kept columns, ascending.
 * wz     [Cout][K] out, w with pruned entries set to +0.0f.
 * Returns ORACLE_OK or ORACLE_ERR_ARG (bad sizes, non-finite weight).
 */
int oracle_prune(const float* w, int cout, int K, int N, int M, int T,
                 uint8_t* mask, int32_t* idx, float* wz)
{
    if (!w || !mask || !idx || !wz) return ORACLE_ERR_ARG;
    if (cout < 1 || K < 1 || N < 1 || M < 1 || T < 1 || N > M) return ORACLE_ERR_ARG;
    if (K % M != 0) return ORACLE_ERR_ARG;
    for (long i = 0; i < (long)cout * K; ++i)
        if (!isfinite(w[i])) return ORACLE_ERR_ARG;

    const int G = K / M;
    const int n_tiles = (cout + T - 1) / T;
    double* score = (double*)malloc(sizeof(double) * (size_t)M);
    uint8_t* taken = (uint8_t*)malloc((size_t)M);
    if (!score || !taken) { free(score); free(taken); return ORACLE_ERR_ARG; }

    memset(mask, 0, (size_t)cout * K);

    for (int j = 0; j < n_tiles; ++j) {
        const int r0 = j * T;
        const int r1 = (r0 + T < cout) ? r0 + T : cout;
        for (int g = 0; g < G; ++g) {
            /* L1 norm of each column of the group over the tile's rows */
            for (int c = 0; c < M; ++c) {
                double s = 0.0;
                for (int r = r0; r < r1; ++r)
                    s += fabs((double)w[(long)r * K + (long)g * M + c]);
                score[c] = s;
                taken[c] = 0;
            }
            /* N rounds of "take the largest remaining"; strict > keeps the
             * lowest column among equals */
            for (int n = 0; n < N; ++n) {
                int best = -1;
                for (int c = 0; c < M; ++c) {
                    if (taken[c]) continue;
                    if (best < 0 || score[c] > score[best]) best = c;
                }
                taken[best] = 1;
            }
            /* kept positions in ascending k */
            int n = 0;
            for (int c = 0; c < M; ++c) {
                if (!taken[c]) continue;
                idx[((long)j * G + g) * N + n] = g * M + c;
                ++n;
                for (int r = r0; r < r1; ++r)
                    mask[(long)r * K + (long)g * M + c] = 1;
            }
        }
    }
    for (long i = 0; i < (long)cout * K; ++i)
        wz[i] = mask[i] ? w[i] : 0.0f;

    free(score);
    free(taken);
    return ORACLE_OK;
}

/*
 * The compressed weights and their index array (section 2.1; the inputs W[T,N]
 * and Idx[N] of Alg. 1, repeated over groups):
 *   vals[j][kk][t] = w[j*T + t][ idx[j][kk] ],  kk = g*N + n,  zero when the
 *   row j*T + t does not exist.
 */
int oracle_pack(const float* w, int cout, int K, int N, int M, int T,
                const int32_t* idx, float* vals)
{
    if (!w || !idx || !vals || K % M != 0) return ORACLE_ERR_ARG;
    const int G = K / M;
    const int kprime = G * N;
    const int n_tiles = (cout + T - 1) / T;
    for (int j = 0; j < n_tiles; ++j)
        for (int kk = 0; kk < kprime; ++kk)
            for (int t = 0; t < T; ++t) {
                const int r = j * T + t;
                const int k = idx[(long)j * kprime + kk];
                vals[((long)j * kprime + kk) * T + t] =
                    (r < cout) ? w[(long)r * K + k] : 0.0f;
            }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Convolution: section 2.2 (convolution as patch matrix x filter matrix),   */
/* written as the direct seven-loop sum so that no im2col matrix, no tiling  */
/* and no reordering is involved.                                            */
/* ------------------------------------------------------------------------- */

/* round-to-nearest-even fp32 -> bf16, returned as the exactly representable
 * float (standard definition; inputs are finite here) */
static float round_to_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return v; /* NaN stays NaN */
    const uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    float r;
    memcpy(&r, &u, 4);
    return r;
}

/* fp32 -> fp8 E4M3 (the OCP "e4m3fn" format: 4 exponent bits with bias 7, 3 mantissa bits,
 * subnormals, no infinity, largest finite value 448), round to nearest, ties to even,
 * returned as the exactly representable float.  Written from the format's definition: the
 * spacing of representable values is 2^(E-3) in the binade 2^E <= |v| < 2^(E+1), E >= -6,
 * and 2^-9 below 2^-6; rounding |v| to a multiple of that spacing with ties to the even
 * multiple is round-to-nearest-even, because the multiples that are even are exactly the
 * values with an even mantissa field.  Beyond the largest finite value the format has no
 * number to round to: the result is NaN (no saturation), as in the reference conversion. */
static float round_to_e4m3(float v)
{
    if (v != v) return v;
    const double a = fabs((double)v);
    if (a == 0.0) return v;
    int e;
    (void)frexp(a, &e);                 /* a = f * 2^e with 0.5 <= f < 1: leading bit at 2^(e-1) */
    int E = e - 1;
    if (E < -6) E = -6;
    const double ulp = ldexp(1.0, E - 3);
    const double r = nearbyint(a / ulp) * ulp;   /* default rounding mode: ties to even; a / ulp is exact */
    if (r > 448.0) return (float)NAN;
    return (float)(v < 0 ? -r : r);
}

/* elementwise rounding of n floats to E4M3-representable floats */
void oracle_round_e4m3(const float* in, float* out, long n)
{
    for (long i = 0; i < n; ++i) out[i] = round_to_e4m3(in[i]);
}

/* elementwise RNE rounding of n floats to bf16-representable floats */
void oracle_round_bf16(const float* in, float* out, long n)
{
    for (long i = 0; i < n; ++i) out[i] = round_to_bf16(in[i]);
}

typedef struct {
    const float* x;
    const float* w;
    const float* bias;
    const float* res;        /* residual shaped like y, or NULL */
    float* y;
    int B, H, W, Cin, Cout, Kh, Kw;
    int sh, sw, ph, pw, dh, dw;
    int Ho, Wo;
    int relu, out_bf16;
    long row_begin, row_end; /* rows are (b, ho) pairs */
} conv_job;

/* one output element: y[b][ho][wo][co] */
static float conv_point(const conv_job* J, int b, int ho, int wo, int co)
{
    double acc = 0.0;
    for (int kh = 0; kh < J->Kh; ++kh) {
        const int hi = ho * J->sh - J->ph + kh * J->dh;
        if (hi < 0 || hi >= J->H) continue;           /* zero padding */
        for (int kw = 0; kw < J->Kw; ++kw) {
            const int wi = wo * J->sw - J->pw + kw * J->dw;
            if (wi < 0 || wi >= J->W) continue;       /* zero padding */
            const float* xp = J->x + (((long)b * J->H + hi) * J->W + wi) * J->Cin;
            const float* wp = J->w + (((long)co * J->Kh + kh) * J->Kw + kw) * J->Cin;
            for (int ci = 0; ci < J->Cin; ++ci)
                acc += (double)xp[ci] * (double)wp[ci];
        }
    }
    if (J->bias) acc += (double)J->bias[co];
    if (J->res)                                        /* skip connection, before the activation */
        acc += (double)J->res[(((long)b * J->Ho + ho) * J->Wo + wo) * J->Cout + co];
    if (J->relu && acc < 0.0) acc = 0.0;
    float r = (float)acc;                              /* one rounding */
    if (J->out_bf16) r = round_to_bf16(r);
    return r;
}

static void* conv_rows(void* arg)
{
    const conv_job* J = (const conv_job*)arg;
    for (long row = J->row_begin; row < J->row_end; ++row) {
        const int b = (int)(row / J->Ho);
        const int ho = (int)(row % J->Ho);
        for (int wo = 0; wo < J->Wo; ++wo)
            for (int co = 0; co < J->Cout; ++co)
                J->y[(((long)b * J->Ho + ho) * J->Wo + wo) * J->Cout + co] =
                    conv_point(J, b, ho, wo, co);
    }
    return NULL;
}

static int fill_job(conv_job* J, const float* x, int B, int H, int W, int Cin,
                    const float* w, int Cout, int Kh, int Kw, const float* bias,
                    int sh, int sw, int ph, int pw, int dh, int dw,
                    int relu, int out_bf16, float* y)
{
    if (!x || !w || !y) return ORACLE_ERR_ARG;
    if (B < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1 || Kh < 1 || Kw < 1) return ORACLE_ERR_ARG;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1) return ORACLE_ERR_ARG;
    const int eh = H + 2 * ph - dh * (Kh - 1) - 1;
    const int ew = W + 2 * pw - dw * (Kw - 1) - 1;
    if (eh < 0 || ew < 0) return ORACLE_ERR_ARG;
    J->x = x; J->w = w; J->bias = bias; J->res = NULL; J->y = y;
    J->B = B; J->H = H; J->W = W; J->Cin = Cin; J->Cout = Cout; J->Kh = Kh; J->Kw = Kw;
    J->sh = sh; J->sw = sw; J->ph = ph; J->pw = pw; J->dh = dh; J->dw = dw;
    J->Ho = eh / sh + 1;
    J->Wo = ew / sw + 1;
    J->relu = relu; J->out_bf16 = out_bf16;
    return ORACLE_OK;
}

/*
 * Direct convolution, NHWC input x[B][H][W][Cin], OHWI weights
 * w[Cout][Kh][Kw][Cin] (already zero filled where pruned), optional bias and
 * ReLU, output y[B][Ho][Wo][Cout] fp32 (optionally rounded to bf16 values).
 * The (b, ho) rows are split over nthreads host threads; each output element
 * is computed by exactly one thread with the same arithmetic, so the result
 * does not depend on nthreads.
 */
int oracle_conv2d(const float* x, int B, int H, int W, int Cin,
                  const float* w, int Cout, int Kh, int Kw, const float* bias,
                  int sh, int sw, int ph, int pw, int dh, int dw,
                  int relu, int out_bf16, float* y, int nthreads)
{
    conv_job base;
    int rc = fill_job(&base, x, B, H, W, Cin, w, Cout, Kh, Kw, bias,
                      sh, sw, ph, pw, dh, dw, relu, out_bf16, y);
    if (rc != ORACLE_OK) return rc;
    const long rows = (long)B * base.Ho;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > rows) nthreads = (int)rows;
    if (nthreads > 256) nthreads = 256;

    conv_job jobs[256];
    pthread_t th[256];
    for (int t = 0; t < nthreads; ++t) {
        jobs[t] = base;
        jobs[t].row_begin = rows * t / nthreads;
        jobs[t].row_end = rows * (t + 1) / nthreads;
    }
    if (nthreads == 1) {
        conv_rows(&jobs[0]);
        return ORACLE_OK;
    }
    for (int t = 0; t < nthreads; ++t)
        if (pthread_create(&th[t], NULL, conv_rows, &jobs[t]) != 0) return ORACLE_ERR_ARG;
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
    return ORACLE_OK;
}

/*
 * The convolution that closes a residual block:
 *   y = relu?( conv(x, w) + bias + residual ), residual[B][Ho][Wo][Cout],
 * the whole sum in double, one rounding.  Single-threaded.
 */
int oracle_conv2d_res(const float* x, int B, int H, int W, int Cin,
                      const float* w, int Cout, int Kh, int Kw, const float* bias,
                      const float* residual,
                      int sh, int sw, int ph, int pw, int dh, int dw,
                      int relu, int out_bf16, float* y)
{
    conv_job J;
    int rc = fill_job(&J, x, B, H, W, Cin, w, Cout, Kh, Kw, bias,
                      sh, sw, ph, pw, dh, dw, relu, out_bf16, y);
    if (rc != ORACLE_OK) return rc;
    J.res = residual;
    J.row_begin = 0;
    J.row_end = (long)B * J.Ho;
    conv_rows(&J);
    return ORACLE_OK;
}

/*
 * Max pooling, NHWC, k x k window, padding never wins:
 *   y[b][ho][wo][c] = max over the in-image positions of the window.
 */
int oracle_maxpool2d(const float* x, int B, int H, int W, int C, int k, int stride, int pad, float* y)
{
    if (!x || !y || B < 1 || H < 1 || W < 1 || C < 1 || k < 1 || stride < 1 || pad < 0 || pad >= k)
        return ORACLE_ERR_ARG;
    if (H + 2 * pad < k || W + 2 * pad < k) return ORACLE_ERR_ARG;
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    for (int b = 0; b < B; ++b)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < C; ++c) {
                    int have = 0;
                    float m = 0.f;
                    for (int kh = 0; kh < k; ++kh) {
                        const int hi = ho * stride - pad + kh;
                        if (hi < 0 || hi >= H) continue;
                        for (int kw = 0; kw < k; ++kw) {
                            const int wi = wo * stride - pad + kw;
                            if (wi < 0 || wi >= W) continue;
                            const float v = x[(((long)b * H + hi) * W + wi) * C + c];
                            if (!have || v > m) { m = v; have = 1; }
                        }
                    }
                    y[(((long)b * Ho + ho) * Wo + wo) * C + c] = m;
                }
    return ORACLE_OK;
}

/* Global average pooling: y[b][c] = mean of x[b][.][.][c], summed in double, one rounding. */
int oracle_avgpool_global(const float* x, int B, int H, int W, int C, int out_bf16, float* y)
{
    if (!x || !y || B < 1 || H < 1 || W < 1 || C < 1) return ORACLE_ERR_ARG;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            for (long i = 0; i < (long)H * W; ++i) s += (double)x[((long)b * H * W + i) * C + c];
            float r = (float)(s / (double)((long)H * W));
            if (out_bf16) r = round_to_bf16(r);
            y[(long)b * C + c] = r;
        }
    return ORACLE_OK;
}

/*
 * The im2col matrix of section 2.2 written out: a[p][k], p = (b*Ho + ho)*Wo + wo,
 * k = (kh*Kw + kw)*Cin + ci, zero outside the image.
 */
int oracle_im2col(const float* x, int B, int H, int W, int Cin, int Kh, int Kw,
                  int sh, int sw, int ph, int pw, int dh, int dw, float* a)
{
    if (!x || !a || B < 1 || H < 1 || W < 1 || Cin < 1 || Kh < 1 || Kw < 1) return ORACLE_ERR_ARG;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1) return ORACLE_ERR_ARG;
    const int eh = H + 2 * ph - dh * (Kh - 1) - 1, ew = W + 2 * pw - dw * (Kw - 1) - 1;
    if (eh < 0 || ew < 0) return ORACLE_ERR_ARG;
    const int Ho = eh / sh + 1, Wo = ew / sw + 1;
    const long K = (long)Kh * Kw * Cin;
    for (int b = 0; b < B; ++b)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                float* row = a + (((long)b * Ho + ho) * Wo + wo) * K;
                for (int kh = 0; kh < Kh; ++kh)
                    for (int kw = 0; kw < Kw; ++kw) {
                        const int hi = ho * sh - ph + kh * dh, wi = wo * sw - pw + kw * dw;
                        const int in = hi >= 0 && hi < H && wi >= 0 && wi < W;
                        for (int ci = 0; ci < Cin; ++ci)
                            row[((long)kh * Kw + kw) * Cin + ci] =
                                in ? x[(((long)b * H + hi) * W + wi) * Cin + ci] : 0.f;
                    }
            }
    return ORACLE_OK;
}

/*
 * The same definition evaluated only at npts listed output positions
 * pts[i] = {b, ho, wo, co}; out[i] receives y[b][ho][wo][co].  Used to check
 * full-size layers whose whole output would take the CPU too long.
 */
int oracle_conv2d_points(const float* x, int B, int H, int W, int Cin,
                         const float* w, int Cout, int Kh, int Kw, const float* bias,
                         int sh, int sw, int ph, int pw, int dh, int dw,
                         int relu, int out_bf16,
                         const int32_t* pts, long npts, float* out)
{
    conv_job J;
    float dummy;
    int rc = fill_job(&J, x, B, H, W, Cin, w, Cout, Kh, Kw, bias,
                      sh, sw, ph, pw, dh, dw, relu, out_bf16, &dummy);
    if (rc != ORACLE_OK || !pts || !out) return ORACLE_ERR_ARG;
    for (long i = 0; i < npts; ++i) {
        const int b = pts[4 * i + 0], ho = pts[4 * i + 1];
        const int wo = pts[4 * i + 2], co = pts[4 * i + 3];
        if (b < 0 || b >= B || ho < 0 || ho >= J.Ho || wo < 0 || wo >= J.Wo ||
            co < 0 || co >= Cout)
            return ORACLE_ERR_ARG;
        out[i] = conv_point(&J, b, ho, wo, co);
    }
    return ORACLE_OK;
}

int oracle_out_size(int H, int W, int Kh, int Kw, int sh, int sw, int ph, int pw,
                    int dh, int dw, int* Ho, int* Wo)
{
    const int eh = H + 2 * ph - dh * (Kh - 1) - 1;
    const int ew = W + 2 * pw - dw * (Kw - 1) - 1;
    if (eh < 0 || ew < 0 || sh < 1 || sw < 1) return ORACLE_ERR_ARG;
    *Ho = eh / sh + 1;
    *Wo = ew / sw + 1;
    return ORACLE_OK;
}
