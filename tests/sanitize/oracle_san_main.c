/*
 * Address- and undefined-behaviour-sanitizer run of the CPU oracle (host code
 * only).  Built by tests/test_sanitizers.py as
 *   gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all \
 *       oracle/nm_oracle.c tests/sanitize/oracle_san_main.c -lm -pthread
 * Every buffer is allocated at its exact size, so a read or write one element
 * outside what the functions document trips the sanitizer; ragged tiles, odd
 * geometries, paddings larger than the kernel reach, strides and dilations,
 * several threads and the argument-error paths are all exercised.  A few
 * invariants are checked on the way so that the run is also a smoke test.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_prune(const float* w, int cout, int K, int N, int M, int T, uint8_t* mask, int32_t* idx, float* wz);
int oracle_pack(const float* w, int cout, int K, int N, int M, int T, const int32_t* idx, float* vals);
void oracle_round_bf16(const float* in, float* out, long n);
int oracle_conv2d(const float* x, int B, int H, int W, int Cin, const float* w, int Cout, int Kh, int Kw,
                  const float* bias, int sh, int sw, int ph, int pw, int dh, int dw, int relu, int out_bf16,
                  float* y, int nthreads);
int oracle_conv2d_res(const float* x, int B, int H, int W, int Cin, const float* w, int Cout, int Kh, int Kw,
                      const float* bias, const float* residual, int sh, int sw, int ph, int pw, int dh, int dw,
                      int relu, int out_bf16, float* y);
int oracle_conv2d_points(const float* x, int B, int H, int W, int Cin, const float* w, int Cout, int Kh, int Kw,
                         const float* bias, int sh, int sw, int ph, int pw, int dh, int dw, int relu,
                         int out_bf16, const int32_t* pts, long npts, float* out);
int oracle_maxpool2d(const float* x, int B, int H, int W, int C, int k, int stride, int pad, float* y);
int oracle_avgpool_global(const float* x, int B, int H, int W, int C, int out_bf16, float* y);
int oracle_im2col(const float* x, int B, int H, int W, int Cin, int Kh, int Kw, int sh, int sw, int ph, int pw,
                  int dh, int dw, float* a);
int oracle_out_size(int H, int W, int Kh, int Kw, int sh, int sw, int ph, int pw, int dh, int dw, int* Ho, int* Wo);

static unsigned long long rng_state = 88172645463325252ull;
static float rnd(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (float)((rng_state >> 40) & 0xffff) / 32768.0f - 1.0f;
}
static float* randoms(long n)
{
    float* p = (float*)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    for (long i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c);       \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

static void prune_case(int cout, int K, int N, int M, int T)
{
    const int G = K / M, nt = (cout + T - 1) / T;
    float* w = randoms((long)cout * K);
    uint8_t* mask = (uint8_t*)malloc((size_t)cout * K);
    int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)nt * G * N);
    float* wz = (float*)malloc(sizeof(float) * (size_t)cout * K);
    float* vals = (float*)malloc(sizeof(float) * (size_t)nt * G * N * T);
    CHECK(oracle_prune(w, cout, K, N, M, T, mask, idx, wz) == 0);
    CHECK(oracle_pack(w, cout, K, N, M, T, idx, vals) == 0);
    for (int r = 0; r < cout; ++r)
        for (int g = 0; g < G; ++g) {
            int kept = 0;
            for (int c = 0; c < M; ++c) kept += mask[(long)r * K + g * M + c];
            CHECK(kept == N);
        }
    for (int j = 0; j < nt; ++j)
        for (int g = 0; g < G; ++g)
            for (int n = 0; n < N; ++n) {
                const int k = idx[((long)j * G + g) * N + n];
                CHECK(k >= g * M && k < g * M + M);
                CHECK(n == 0 || k > idx[((long)j * G + g) * N + n - 1]);
            }
    free(w); free(mask); free(idx); free(wz); free(vals);
}

static void conv_case(int B, int H, int W, int Cin, int Cout, int Kh, int Kw, int sh, int sw, int ph, int pw,
                      int dh, int dw, int threads)
{
    int Ho = 0, Wo = 0;
    CHECK(oracle_out_size(H, W, Kh, Kw, sh, sw, ph, pw, dh, dw, &Ho, &Wo) == 0);
    float* x = randoms((long)B * H * W * Cin);
    float* w = randoms((long)Cout * Kh * Kw * Cin);
    float* bias = randoms(Cout);
    const long ny = (long)B * Ho * Wo * Cout;
    float* y = (float*)malloc(sizeof(float) * (size_t)ny);
    float* y1 = (float*)malloc(sizeof(float) * (size_t)ny);
    float* res = randoms(ny);
    CHECK(oracle_conv2d(x, B, H, W, Cin, w, Cout, Kh, Kw, bias, sh, sw, ph, pw, dh, dw, 1, 0, y, threads) == 0);
    CHECK(oracle_conv2d(x, B, H, W, Cin, w, Cout, Kh, Kw, NULL, sh, sw, ph, pw, dh, dw, 0, 1, y1, 1) == 0);
    CHECK(oracle_conv2d(x, B, H, W, Cin, w, Cout, Kh, Kw, bias, sh, sw, ph, pw, dh, dw, 1, 0, y1, 1) == 0);
    CHECK(memcmp(y, y1, sizeof(float) * (size_t)ny) == 0);   /* the thread count changes nothing */
    CHECK(oracle_conv2d_res(x, B, H, W, Cin, w, Cout, Kh, Kw, bias, res, sh, sw, ph, pw, dh, dw, 1, 1, y1) == 0);
    /* the last output element and the first, one by one */
    int32_t pts[8] = {B - 1, Ho - 1, Wo - 1, Cout - 1, 0, 0, 0, 0};
    float two[2];
    CHECK(oracle_conv2d_points(x, B, H, W, Cin, w, Cout, Kh, Kw, bias, sh, sw, ph, pw, dh, dw, 1, 0, pts, 2, two) == 0);
    CHECK(two[0] == y[ny - 1] && two[1] == y[0]);
    int32_t bad[4] = {B, 0, 0, 0};
    CHECK(oracle_conv2d_points(x, B, H, W, Cin, w, Cout, Kh, Kw, bias, sh, sw, ph, pw, dh, dw, 1, 0, bad, 1, two) != 0);
    float* a = (float*)malloc(sizeof(float) * (size_t)((long)B * Ho * Wo * Kh * Kw * Cin));
    CHECK(oracle_im2col(x, B, H, W, Cin, Kh, Kw, sh, sw, ph, pw, dh, dw, a) == 0);
    free(x); free(w); free(bias); free(y); free(y1); free(res); free(a);
}

static void pool_case(int B, int H, int W, int C, int k, int stride, int pad)
{
    float* x = randoms((long)B * H * W * C);
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    float* y = (float*)malloc(sizeof(float) * (size_t)((long)B * Ho * Wo * C));
    CHECK(oracle_maxpool2d(x, B, H, W, C, k, stride, pad, y) == 0);
    float* m = (float*)malloc(sizeof(float) * (size_t)(B * C));
    CHECK(oracle_avgpool_global(x, B, H, W, C, 0, m) == 0);
    CHECK(oracle_avgpool_global(x, B, H, W, C, 1, m) == 0);
    free(x); free(y); free(m);
}

int main(void)
{
    /* prune + pack: ragged last tile, T = 1, T > cout, M = K, N = M, M not a power of two */
    prune_case(37, 48, 2, 4, 16);
    prune_case(5, 24, 1, 8, 1);
    prune_case(3, 36, 3, 6, 32);
    prune_case(20, 40, 20, 40, 8);
    prune_case(16, 12, 4, 4, 16);
    prune_case(1, 4, 1, 4, 16);
    /* argument errors come back as codes, not as accesses */
    float one = 1.0f;
    uint8_t m1;
    int32_t i1;
    CHECK(oracle_prune(&one, 1, 5, 1, 4, 1, &m1, &i1, &one) != 0);   /* K % M != 0 */
    CHECK(oracle_prune(NULL, 1, 4, 1, 4, 1, &m1, &i1, &one) != 0);
    CHECK(oracle_pack(&one, 1, 5, 1, 4, 1, &i1, &one) != 0);
    int ho, wo;
    CHECK(oracle_out_size(2, 2, 5, 5, 1, 1, 0, 0, 1, 1, &ho, &wo) != 0);
    CHECK(oracle_out_size(8, 8, 3, 3, 0, 1, 1, 1, 1, 1, &ho, &wo) != 0);

    /* bf16 rounding: ordinary values, ties, the largest finite value, zeros */
    float in[6] = {1.00390625f, 1.01171875f, 3.3895314e38f, -0.0f, 1e-40f, 65504.0f}, out[6];
    oracle_round_bf16(in, out, 6);
    CHECK(out[0] == 1.0f && out[1] == 1.015625f);

    /* convolutions: one pixel, padding beyond the kernel's reach, strides, dilation, 1x1, 7x7 on 3 channels,
       non-square everything, more threads than rows */
    conv_case(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 4);
    conv_case(2, 5, 7, 3, 4, 3, 3, 1, 1, 1, 1, 1, 1, 3);
    conv_case(1, 9, 8, 2, 5, 3, 2, 2, 3, 2, 1, 2, 2, 16);
    conv_case(3, 6, 6, 4, 6, 1, 1, 2, 2, 0, 0, 1, 1, 2);
    conv_case(1, 12, 12, 3, 2, 7, 7, 2, 2, 3, 3, 1, 1, 5);
    conv_case(1, 4, 4, 1, 1, 3, 3, 1, 1, 5, 5, 1, 1, 300);
    conv_case(2, 3, 10, 5, 3, 1, 4, 1, 2, 0, 3, 1, 3, 2);

    pool_case(2, 7, 6, 3, 3, 2, 1);
    pool_case(1, 1, 1, 5, 1, 1, 0);
    pool_case(1, 8, 8, 2, 5, 3, 2);
    puts("oracle sanitizer run: ok");
    return 0;
}
