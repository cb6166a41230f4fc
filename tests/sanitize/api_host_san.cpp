// Address- and undefined-behaviour-sanitizer run of the library's host layer
// (csrc/nm_api.hip: argument checks, geometry, operand-table planning, variant
// choice, the tuner's loop, the tuning cache and its file format) with no GPU.
// Built by tests/test_sanitizers.py from nm_api.hip compiled host-only with
// -fsanitize=address,undefined and this file, which stands in for everything
// below the host layer:
//   * the HIP runtime calls nm_api.hip makes ("device" memory is host memory),
//   * the kernel launchers (variant table, prune / table-build / fill kernels).
// The stand-ins check what the host layer hands them: launch_conv verifies the
// geometry in ConvParams against its own arithmetic and that every pointer
// it would pass to a kernel is one the fake allocator handed out, large enough.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <string>
#include <vector>

#include "nm_internal.h"

#define CHECK(c)                                                            \
    do {                                                                    \
        if (!(c)) {                                                         \
            fprintf(stderr, "check failed at line %d: %s (last error: %s)\n", __LINE__, #c, nm_last_error()); \
            exit(1);                                                        \
        }                                                                   \
    } while (0)

// ------------------------------------------------------------------ fake HIP
static std::map<char*, size_t> g_allocs;
static bool g_fail_malloc = false;
static int g_launches = 0;

static bool inside(const void* p, size_t need)
{
    const char* c = (const char*)p;
    for (const auto& kv : g_allocs)
        if (c >= kv.first && c + need <= kv.first + kv.second) return true;
    return false;
}

extern "C" {
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int)
{
    memset(p, 0, sizeof(*p));
    snprintf(p->name, sizeof(p->name), "Fake GPU for host tests");
    snprintf(p->gcnArchName, sizeof(p->gcnArchName), "gfx950:sramecc+:xnack-");
    p->multiProcessorCount = 256;
    return hipSuccess;
}
const char* hipGetErrorString(hipError_t) { return "fake HIP error"; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipFuncSetAttribute(const void*, hipFuncAttribute, int) { return hipSuccess; }
hipError_t hipMalloc(void** p, size_t n)
{
    if (g_fail_malloc) { *p = nullptr; return hipErrorOutOfMemory; }
    char* c = (char*)malloc(n ? n : 1);
    g_allocs[c] = n;
    *p = c;
    return hipSuccess;
}
hipError_t hipFree(void* p)
{
    if (!p) return hipSuccess;
    auto it = g_allocs.find((char*)p);
    if (it == g_allocs.end()) { fprintf(stderr, "hipFree of a pointer that was never allocated\n"); exit(1); }
    g_allocs.erase(it);
    free(p);
    return hipSuccess;
}
hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) { memcpy(d, s, n); return hipSuccess; }
hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) { memset(d, v, n); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
static bool g_capturing = false;
hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus* st)
{
    *st = g_capturing ? hipStreamCaptureStatusActive : hipStreamCaptureStatusNone;
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t* e) { *e = (hipEvent_t)malloc(1); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { free(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
// "time" = launches since the last query, so that variants differ deterministically
static int g_timer_variant = 0;
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t)
{
    *ms = 0.01f * (float)(1 + (g_timer_variant * 7919) % 101);
    return hipSuccess;
}
}

// ------------------------------------------------------- fake kernel layer
namespace nm {

static const VariantDesc kFake[] = {
    // name, BP, NBLK, WP, NJ, CK, SPC, vec, kind, share, ksplit, areg
    {"F_NB4_WP1_NJ1_CK32_SPC2", 64, 4, 1, 1, 32, 2, 1, 0, 1, 1, 0},
    {"F_NB4_WP1_NJ1_CK32_SPC4", 64, 4, 1, 1, 32, 4, 1, 0, 1, 1, 0},
    {"F_NB4_WP1_NJ1_CK32_SPC8", 64, 4, 1, 1, 32, 8, 1, 0, 1, 1, 0},
    {"F_NB8_WP1_NJ2_CK64_SPC4", 128, 8, 1, 2, 64, 4, 1, 0, 1, 1, 0},
    {"F_NB8_WP1_NJ2_CK64_SPC8", 128, 8, 1, 2, 64, 8, 1, 0, 1, 1, 0},
    {"F_NB8_WP1_NJ2_CK64_SPC2", 128, 8, 1, 2, 64, 2, 1, 0, 1, 1, 0},
    {"F_SCALAR_CK32_SPC8", 256, 4, 4, 4, 32, 8, 0, 0, 1, 1, 0},
    {"F_VAR_NB4_CK32_SPC8", 64, 4, 1, 1, 32, 8, 1, 5, 1, 1, 0},
    {"F_B16_NB4_CK64_SPC1", 64, 4, 1, 1, 64, 1, 1, 1, 1, 1, 0},
    {"F_B16_NB4_CK64_SPC2", 64, 4, 1, 1, 64, 2, 1, 1, 1, 1, 0},
    {"F_SP1_NB4_NJ2_CK64", 64, 4, 1, 2, 64, 1, 1, 2, 1, 1, 0},
    {"F_SP0_NB4_NJ2_CK128", 64, 4, 1, 2, 128, 2, 1, 3, 1, 1, 0},
    {"F_SPR1_NB4_NJ2_CK64", 64, 4, 1, 2, 64, 1, 1, 2, 1, 1, 1},
    {"F_RUN_NB4_KS3", 64, 4, 1, 1, 192, 3, 1, 4, 1, 1, 0},
    {"F_RUN_NB4_KS1", 64, 4, 1, 1, 64, 1, 1, 4, 1, 1, 0},
    {"F_F8_NB4_WP1_NJ4", 64, 4, 1, 4, 64, 1, 1, 6, 1, 1, 0},
    {"F_F8S_NB4_WP1_NJ2_CK64", 64, 4, 1, 2, 64, 1, 1, 7, 1, 1, 0},
    {"F_F8R_NB4_WP1_NJ2_CK128", 64, 4, 1, 2, 128, 2, 1, 7, 1, 1, 1},
    // K-split forms of the fp32 kernel
    {"F_NB4_WP1_NJ1_CK32_SPC4_S2", 64, 4, 1, 1, 32, 4, 1, 0, 1, 2, 0},
    {"F_NB4_WP1_NJ1_CK32_SPC4_S4", 64, 4, 1, 1, 32, 4, 1, 0, 1, 4, 0},
    {"F_NB4_WP1_NJ1_CK32_SPC2_S16", 64, 4, 1, 1, 32, 2, 1, 0, 1, 16, 0},
    {"F_SCALAR_CK32_SPC8_S2", 256, 4, 4, 4, 32, 8, 0, 0, 1, 2, 0},
};
int variant_count() { return (int)(sizeof(kFake) / sizeof(kFake[0])); }
const VariantDesc& variant_desc(int v) { return kFake[v]; }

int launch_conv(int v, nm_dtype_t xdt, nm_dtype_t ydt, const ConvParams& p, hipStream_t)
{
    CHECK(v >= 0 && v < variant_count());
    const VariantDesc& d = kFake[v];
    g_timer_variant = v;
    ++g_launches;
    const size_t es = xdt == NM_F32 ? 4 : (xdt == NM_BF16 ? 2 : 1), yes = ydt == NM_F32 ? 4 : 2;
    CHECK(xdt == ydt || (xdt == NM_F8E4M3 && ydt == NM_BF16));
    const bool f8 = d.kind == 6 || d.kind == 7;
    CHECK(f8 == (xdt == NM_F8E4M3));
    CHECK(p.oscale > 0.f && (f8 || p.oscale == 1.f));
    if (f8) {   // whole chunks per tap, and the table holds every 64-channel k-step of every row block
        CHECK(p.Cin % d.CK == 0 && p.nchunks == p.Kh * p.Kw * (p.Cin / d.CK));
        CHECK(p.wfrag_bytes == (size_t)p.n_rowblocks * (p.K / 64) * 1024);
    }
    // the geometry the kernels rely on
    const long eh = (long)p.H + 2L * p.ph - (long)p.dh * (p.Kh - 1) - 1, ew = (long)p.W + 2L * p.pw - (long)p.dw * (p.Kw - 1) - 1;
    CHECK(eh >= 0 && ew >= 0 && p.Ho == eh / p.sh + 1 && p.Wo == ew / p.sw + 1);
    CHECK(p.P == p.B * p.Ho * p.Wo && p.K == p.Kh * p.Kw * p.Cin);
    CHECK(p.n_ptiles == (p.P + d.BP - 1) / d.BP && p.n_wg == p.n_ptiles * p.n_cblocks * p.ksplit);
    CHECK(p.ksplit == (d.ksplit > 1 ? d.ksplit : 1));
    if (p.ksplit > 1) {   // every split owns chunks, together they cover the K axis, and the partial sums have a home
        CHECK(p.cps >= 1 && (p.ksplit - 1) * p.cps < p.nchunks && p.ksplit * p.cps >= p.nchunks);
        CHECK(inside(p.partial, (size_t)p.ksplit * p.P * p.Cout * 4));
    }
    CHECK(p.n_cblocks * (4 / d.WP) * d.NJ >= p.n_rowblocks && (p.n_cblocks - 1) * (4 / d.WP) * d.NJ < p.n_rowblocks);
    CHECK(p.wg_per_xcd * 8 >= p.n_wg);
    CHECK((size_t)p.x_elems * es == p.x_bytes && p.x_bytes < 0x80000000u);
    // multiply-shift division is exact on every value the kernels feed it
    const unsigned howo = (unsigned)(p.Ho * p.Wo);
    for (unsigned x : {0u, 1u, howo - 1, howo, howo + 1, (unsigned)p.P - 1, (unsigned)p.P + 1023u, 0x7ffffffeu}) {
        const unsigned q = (unsigned)(((unsigned long long)(2ull * x) * p.howo_mul) >> 32) >> p.howo_shift;
        CHECK(q == x / howo);
        const unsigned q2 = (unsigned)(((unsigned long long)(2ull * x) * p.wo_mul) >> 32) >> p.wo_shift;
        CHECK(q2 == x / (unsigned)p.Wo);
    }
    // every pointer is an allocation of the right size
    CHECK(inside(p.x, p.x_bytes) && inside(p.y, (size_t)p.P * p.Cout * yes));
    CHECK(!p.bias || inside(p.bias, (size_t)p.Cout * 4));
    CHECK(!p.res || inside(p.res, (size_t)p.P * p.Cout * yes));
    CHECK(inside(p.wfrag, p.wfrag_bytes));
    CHECK(p.rows_bytes == 0 || inside(p.rows, p.rows_bytes));
    if (!d.vec) CHECK(p.ktab && inside(p.ktab, (size_t)p.nchunks * d.CK * 4));
    return NM_OK;
}

// "prune": keep the first n columns of every group (ascending, valid), except that column
// tile 0 of handles with m >= 32 keeps the LAST n, so that kept sets crowd into some chunks
int run_prune(const float*, nm_packed* wp, hipStream_t)
{
    CHECK(inside(wp->d_idx, (size_t)wp->n_tiles * wp->kprime * 4));
    CHECK(inside(wp->d_vals, (size_t)wp->n_tiles * wp->kprime * wp->tile * 4));
    for (int j = 0; j < wp->n_tiles; ++j)
        for (int g = 0; g < wp->G; ++g)
            for (int i = 0; i < wp->n; ++i)
                wp->d_idx[((size_t)j * wp->G + g) * wp->n + i] =
                    g * wp->m + ((j == 0 && wp->m >= 32) ? wp->m - wp->n + i : i);
    return NM_OK;
}
int run_build_prepack(nm_packed* wp, Prepack& pp, hipStream_t)
{
    CHECK(inside(pp.d_wfrag, pp.wfrag_bytes));
    CHECK(pp.rows_bytes == 0 || inside(pp.d_rows, pp.rows_bytes));
    memset(pp.d_wfrag, 0, pp.wfrag_bytes);   // touches every byte the kernel would fill
    (void)wp;
    return NM_OK;
}
int run_quantize_e4m3(nm_packed* wp, hipStream_t)
{
    CHECK(wp->scale > 0.f && inside(wp->d_vals, (size_t)wp->n_tiles * wp->kprime * wp->tile * 4));
    int e = 0;
    CHECK(frexpf(wp->scale, &e) == 0.5f);   // a power of two
    return NM_OK;
}
int run_build_mask(const nm_packed* wp, uint8_t* d_mask, hipStream_t)
{
    CHECK(inside(d_mask, (size_t)wp->cout * wp->K));
    memset(d_mask, 0, (size_t)wp->cout * wp->K);
    return NM_OK;
}
int run_fill_random(void* d, size_t n, nm_dtype_t dt, uint32_t, hipStream_t)
{
    CHECK(inside(d, n * (dt == NM_F32 ? 4 : (dt == NM_BF16 ? 2 : 1))));
    return NM_OK;
}
int run_maxpool(const void*, nm_dtype_t, int, int, int, int, int, int, int, int, int, void*, hipStream_t) { return NM_OK; }
int run_avgpool(const void*, nm_dtype_t, int, int, int, void*, hipStream_t) { return NM_OK; }
int run_im2col(const void*, nm_dtype_t, int, int, int, int, int, int, int, int, int, int, int, int, int, int, void*,
               hipStream_t) { return NM_OK; }
static char* fake = nullptr;
int static_scratch(int, float** out)
{
    if (!fake) {   // this "device's" copy of the static scratch array; never freed
        fake = (char*)malloc(kStaticScratchBytes);
        g_allocs[fake] = kStaticScratchBytes;
    }
    *out = (float*)fake;
    return NM_OK;
}
int run_splitk_reduce(const ConvParams& p, nm_dtype_t, hipStream_t)
{
    CHECK(p.ksplit > 1 && inside(p.partial, (size_t)p.ksplit * p.P * p.Cout * 4));
    return NM_OK;
}
int run_stream_floor(const void* x, size_t xb, void* y, size_t yb, hipStream_t)
{
    CHECK(inside(x, xb) && inside(y, yb));
    return NM_OK;
}
}  // namespace nm

// ------------------------------------------------------------------- driver
static void* dev_alloc(size_t n)
{
    void* p = nullptr;
    CHECK(hipMalloc(&p, n) == hipSuccess);
    return p;
}

static void conv_case(int b, int h, int w, int cin, int cout, int kh, int kw, int n, int m, int tile, nm_dtype_t dt,
                      int sh, int sw, int ph, int pw, int dh, int dw)
{
    std::vector<float> wt((size_t)cout * kh * kw * cin, 0.5f);
    nm_packed_t* wp = nullptr;
    CHECK(nm_prune(wt.data(), cout, kh, kw, cin, n, m, tile, dt, &wp) == NM_OK && wp);
    int nt, g, nn, kp;
    CHECK(nm_packed_dims(wp, &nt, &g, &nn, &kp) == NM_OK && nt == (cout + tile - 1) / tile && kp == g * n);
    std::vector<int32_t> idx((size_t)nt * kp);
    std::vector<float> vals((size_t)nt * kp * tile);
    std::vector<uint8_t> mask((size_t)cout * kh * kw * cin);
    CHECK(nm_packed_indices(wp, idx.data()) == NM_OK);
    CHECK(nm_packed_values(wp, vals.data()) == NM_OK);
    CHECK(nm_packed_mask(wp, mask.data()) == NM_OK);
    const nm_dtype_t ydt = dt == NM_F8E4M3 ? NM_BF16 : dt;
    const size_t es = dt == NM_F32 ? 4 : (dt == NM_BF16 ? 2 : 1), yes = ydt == NM_F32 ? 4 : 2;
    const long eh = (long)h + 2L * ph - (long)dh * (kh - 1) - 1, ew = (long)w + 2L * pw - (long)dw * (kw - 1) - 1;
    const int ho = (int)(eh / sh) + 1, wo = (int)(ew / sw) + 1;
    void* x = dev_alloc((size_t)b * h * w * cin * es);
    void* y = dev_alloc((size_t)b * ho * wo * cout * yes);
    void* r = dev_alloc((size_t)b * ho * wo * cout * yes);
    float* bias = (float*)dev_alloc((size_t)cout * 4);
    const int before = g_launches;
    CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_OK);
    CHECK(g_launches == before + 1 && nm_last_variant() >= 0);
    CHECK(nm_conv2d_res(x, dt, b, h, w, cin, wp, nullptr, r, sh, sw, ph, pw, dh, dw, 0, y, ydt, nullptr) == NM_OK);
    CHECK(nm_conv2d_res(x, dt, b, h, w, cin, wp, nullptr, y, sh, sw, ph, pw, dh, dw, 0, y, ydt, nullptr) == NM_ERR_ARG);
    int v = -1;
    float ms = 0.f;
    CHECK(nm_autotune(dt, b, h, w, cin, wp, 1, sh, sw, ph, pw, dh, dw, 1, ydt, nullptr, &v, &ms) == NM_OK);
    CHECK(v >= 0 && ms > 0.f && nm_variant_legal(v, wp, dt, ydt) == 1);
    CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_OK);
    CHECK(nm_last_variant() == v);
    // every legal variant forced in turn, an illegal one refused
    for (int u = 0; u < nm_variant_count(); ++u) {
        CHECK(nm_force_variant(u) == NM_OK);
        const int legal = nm_variant_legal(u, wp, dt, ydt);
        const int rc = nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr);
        CHECK(legal ? (rc == NM_OK || rc == NM_ERR_UNSUPPORTED) : rc == NM_ERR_UNSUPPORTED);
    }
    CHECK(nm_force_variant(-1) == NM_OK);
    // K-split variants: through the growable workspace, through the static scratch, and under capture
    for (int u = 0; u < nm_variant_count(); ++u) {
        const char* nme = nm_variant_name(u);
        if (!strstr(nme, "_S") || nm_variant_legal(u, wp, dt, ydt) != 1) continue;
        CHECK(nm_force_variant(u) == NM_OK);
        CHECK(nm_conv2d_static(x, dt, b, h, w, cin, wp, bias, r, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_OK);
        CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_OK);
        g_capturing = true;   // large enough already: no allocation, so capture is fine
        CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_OK);
        g_capturing = false;
    }
    CHECK(nm_force_variant(-1) == NM_OK);
    // argument and shape errors
    CHECK(nm_conv2d(x, dt, b, h, w, cin + 1, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_ERR_ARG);
    CHECK(nm_conv2d((char*)x + 2, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_ERR_ARG);
    CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, 0, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_ERR_ARG);
    CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, h + 2 * ph + 1, dw, 1, y, ydt, nullptr) ==
          (kh > 1 ? NM_ERR_SHAPE : NM_OK));
    CHECK(nm_conv2d(x, dt, b, h, w, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt == NM_F32 ? NM_BF16 : NM_F32, nullptr) ==
          NM_ERR_UNSUPPORTED);
    CHECK(nm_conv2d(x, dt, 1 << 20, 4096, 4096, cin, wp, bias, sh, sw, ph, pw, dh, dw, 1, y, ydt, nullptr) == NM_ERR_SHAPE);
    CHECK(hipFree(x) == hipSuccess && hipFree(y) == hipSuccess && hipFree(r) == hipSuccess && hipFree(bias) == hipSuccess);
    CHECK(nm_packed_free(wp) == NM_OK);
}

// a K split whose partial sums outgrow the static scratch, and one that would have to allocate under capture
static void split_limits()
{
    const int cout = 64, cin = 64;
    std::vector<float> wt((size_t)cout * 9 * cin, 0.5f);
    nm_packed_t* wp = nullptr;
    CHECK(nm_prune(wt.data(), cout, 3, 3, cin, 2, 4, 16, NM_F32, &wp) == NM_OK);
    int forced = -1;
    for (int u = 0; u < nm_variant_count(); ++u)
        if (strstr(nm_variant_name(u), "_S4") && nm_variant_legal(u, wp, NM_F32, NM_F32) == 1) forced = u;
    CHECK(forced >= 0 && nm_force_variant(forced) == NM_OK);
    const int b = 8, h = 96, w = 96;   // 4 splits x 73728 pixels x 64 channels x 4 bytes = 75 MB
    void* x = dev_alloc((size_t)b * h * w * cin * 4);
    void* y = dev_alloc((size_t)b * h * w * cout * 4);
    CHECK(nm_conv2d_static(x, NM_F32, b, h, w, cin, wp, nullptr, nullptr, 1, 1, 1, 1, 1, 1, 0, y, NM_F32, nullptr) == NM_ERR_SHAPE);
    CHECK(strstr(nm_last_error(), "static buffer"));
    g_capturing = true;
    CHECK(nm_conv2d(x, NM_F32, b, h, w, cin, wp, nullptr, 1, 1, 1, 1, 1, 1, 0, y, NM_F32, nullptr) == NM_ERR_ALLOC);
    g_capturing = false;
    CHECK(nm_conv2d(x, NM_F32, b, h, w, cin, wp, nullptr, 1, 1, 1, 1, 1, 1, 0, y, NM_F32, nullptr) == NM_OK);
    CHECK(nm_force_variant(-1) == NM_OK);
    CHECK(hipFree(x) == hipSuccess && hipFree(y) == hipSuccess && nm_packed_free(wp) == NM_OK);
}

int main(int argc, char** argv)
{
    const std::string tmp = argc > 1 ? argv[1] : "/tmp";
    CHECK(nm_variant_count() > 0 && nm_variant_name(-1) == nullptr && nm_variant_name(nm_variant_count()) == nullptr);
    CHECK(nm_last_variant() == -1);

    // ---- nm_prune argument checks
    nm_packed_t* wp = nullptr;
    float w4[16] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16};
    CHECK(nm_prune(nullptr, 1, 1, 1, 16, 2, 4, 16, NM_F32, &wp) == NM_ERR_ARG);
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 4, 16, NM_F32, nullptr) == NM_ERR_ARG);
    CHECK(nm_prune(w4, 0, 1, 1, 16, 2, 4, 16, NM_F32, &wp) == NM_ERR_ARG && !wp);
    CHECK(nm_prune(w4, 1, 1, 1, 16, 5, 4, 16, NM_F32, &wp) == NM_ERR_ARG);
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 5, 16, NM_F32, &wp) == NM_ERR_ARG);     // K % m
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 4, 0, NM_F32, &wp) == NM_ERR_ARG);
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 4, 16, (nm_dtype_t)7, &wp) == NM_ERR_ARG);
    w4[7] = INFINITY;
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 4, 16, NM_F32, &wp) == NM_ERR_ARG && strstr(nm_last_error(), "finite"));
    w4[7] = NAN;
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 4, 16, NM_F32, &wp) == NM_ERR_ARG);
    w4[7] = 8;
    g_fail_malloc = true;      // an allocation failure half way frees everything it had
    CHECK(nm_prune(w4, 1, 1, 1, 16, 2, 4, 16, NM_F32, &wp) == NM_ERR_ALLOC && !wp && g_allocs.empty());
    g_fail_malloc = false;
    CHECK(nm_packed_dims(nullptr, nullptr, nullptr, nullptr, nullptr) == NM_ERR_ARG);
    CHECK(nm_packed_indices(nullptr, nullptr) == NM_ERR_ARG && nm_packed_values(nullptr, nullptr) == NM_ERR_ARG);
    CHECK(nm_packed_mask(nullptr, nullptr) == NM_ERR_ARG && nm_packed_free(nullptr) == NM_OK);
    CHECK(nm_force_variant(-2) == NM_ERR_ARG && nm_force_variant(nm_variant_count()) == NM_ERR_ARG);
    CHECK(nm_conv2d(nullptr, NM_F32, 1, 1, 1, 1, nullptr, nullptr, 1, 1, 0, 0, 1, 1, 0, nullptr, NM_F32, nullptr) == NM_ERR_ARG);
    CHECK(nm_autotune(NM_F32, 1, 1, 1, 1, nullptr, 0, 1, 1, 0, 0, 1, 1, 0, NM_F32, nullptr, nullptr, nullptr) == NM_ERR_ARG);

    {
        void* a = dev_alloc(100);
        void* b = dev_alloc(64);
        CHECK(nm_stream_floor(a, 100, b, 64, nullptr) == NM_OK);
        CHECK(nm_stream_floor(nullptr, 100, b, 64, nullptr) == NM_ERR_ARG);
        CHECK(nm_stream_floor((char*)a + 4, 96, b, 64, nullptr) == NM_ERR_ARG);
        CHECK(hipFree(a) == hipSuccess && hipFree(b) == hipSuccess);
    }

    // ---- planning, launching, tuning over a grid of layers (ragged tiles, strides, dilation,
    // few input channels, groups wider than a chunk, T = 8 / 32, both tensor types)
    CHECK(nm_cache_clear() == NM_OK);
    conv_case(2, 9, 7, 16, 20, 3, 3, 2, 4, 16, NM_F32, 1, 1, 1, 1, 1, 1);
    conv_case(1, 12, 12, 3, 24, 7, 7, 1, 1, 16, NM_F32, 2, 2, 3, 3, 1, 1);     // element-wise staging
    conv_case(1, 12, 12, 3, 24, 7, 7, 1, 1, 16, NM_BF16, 2, 2, 3, 3, 1, 1);    // kernel-row runs
    conv_case(3, 8, 8, 64, 40, 1, 1, 2, 4, 8, NM_BF16, 2, 2, 0, 0, 1, 1);
    conv_case(1, 6, 10, 64, 64, 3, 3, 32, 64, 32, NM_F32, 1, 2, 2, 1, 2, 1);   // one group per tap
    conv_case(1, 5, 5, 128, 16, 1, 1, 4, 8, 16, NM_BF16, 1, 1, 0, 0, 1, 1);    // dense instruction only
    conv_case(1, 1, 1, 8, 5, 1, 1, 1, 2, 5, NM_F32, 1, 1, 0, 0, 1, 1);
    conv_case(2, 7, 6, 128, 40, 3, 3, 2, 4, 16, NM_F8E4M3, 2, 1, 1, 1, 1, 1);    // fp8 in, bf16 out
    {   // E4M3 weights that the fp8 kernel cannot take, and fp8 tensors on weights of another type
        std::vector<float> wt(16 * 48, 0.25f);
        nm_packed_t* h8 = nullptr;
        CHECK(nm_prune(wt.data(), 16, 1, 1, 48, 2, 4, 16, NM_F8E4M3, &h8) == NM_ERR_UNSUPPORTED && !h8);
        CHECK(nm_prune(wt.data(), 12, 1, 1, 64, 2, 4, 16, NM_F8E4M3, &h8) == NM_ERR_UNSUPPORTED && !h8);
        std::vector<float> w64(16 * 64, 0.25f);
        CHECK(nm_prune(w64.data(), 16, 1, 1, 64, 2, 4, 16, NM_F32, &h8) == NM_OK);
        void* xb = dev_alloc(64), *yb = dev_alloc(64);
        CHECK(nm_conv2d(xb, NM_F8E4M3, 1, 1, 1, 64, h8, nullptr, 1, 1, 0, 0, 1, 1, 0, yb, NM_BF16, nullptr) == NM_ERR_UNSUPPORTED);
        float sc = 0.f;
        CHECK(nm_packed_scale(h8, &sc) == NM_OK && sc == 1.f && nm_packed_scale(nullptr, &sc) == NM_ERR_ARG);
        CHECK(hipFree(xb) == hipSuccess && hipFree(yb) == hipSuccess && nm_packed_free(h8) == NM_OK);
    }
    split_limits();
    // nothing leaked on the "device": what is left is the K-split workspace and the static scratch
    CHECK(g_allocs.size() <= 2);
    const int n_entries = nm_cache_size();
    CHECK(n_entries == 8);

    // ---- cache file round trip and hostile files
    const std::string path = tmp + "/nm_cache_san.txt";
    CHECK(nm_cache_save(path.c_str()) == NM_OK);
    CHECK(nm_cache_clear() == NM_OK && nm_cache_size() == 0);
    CHECK(nm_cache_load(path.c_str()) == NM_OK && nm_cache_size() == n_entries);
    CHECK(nm_cache_load((tmp + "/does_not_exist.txt").c_str()) == NM_ERR_IO);
    CHECK(nm_cache_save((tmp + "/no_such_dir/x.txt").c_str()) == NM_ERR_IO);
    CHECK(nm_cache_save(nullptr) == NM_ERR_ARG && nm_cache_load(nullptr) == NM_ERR_ARG);
    const char* hostile[] = {
        "", "nmconv-cache", "nmconv-cache 1 5\n", "garbage garbage\n1 2 3\n",
        "nmconv-cache 2 14 24 dev\n1 2 3\n",                                  // truncated entry
        "nmconv-cache 2 14 24 dev\n0 0 1 1 1 1 1 1 1 1 1 0 0 1 1 1 1 1 0 0 0 0 0 0 NO_SUCH_VARIANT 0.5\n",
        "nmconv-cache 2 14 24 dev\n0 0 1 1 1 1 1 1 1 1 1 0 0 1 1 1 1 1 0 0 0 0 0 0 "
        "AAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAA 1.0\n",
        "nmconv-cache 2 14 24 "
        "DDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDDD\n",
        "nmconv-cache 2 14 24 dev\n99999999999999999999 1 2\n",
    };
    for (const char* text : hostile) {
        const std::string hp = tmp + "/nm_cache_hostile.txt";
        FILE* f = fopen(hp.c_str(), "w");
        CHECK(f);
        fputs(text, f);
        fclose(f);
        const int before = nm_cache_size();
        const int rc = nm_cache_load(hp.c_str());
        CHECK(rc == NM_OK || rc == NM_ERR_IO);
        CHECK(nm_cache_size() == before);          // nothing it holds names a real variant of a real shape
    }
    CHECK(nm_cache_clear() == NM_OK);
    CHECK(nm_workspace_free() == NM_OK);
    g_allocs.erase(nm::fake);
    free(nm::fake);
    CHECK(g_allocs.empty());
    puts("host-layer sanitizer run: ok");
    return 0;
}
