// C ABI of libnmconv: argument checking, the packed-weights handle, variant
// choice, the tuning cache and the profiler-driven tuner.  All arithmetic of
// the method runs in the kernels; this file only plans and launches.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>

#include "nm_internal.h"

namespace nm {

static thread_local char g_err[512] = "";
static thread_local int g_last_variant = -1;

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int allow_lds(const void* fn, size_t bytes, unsigned long long* done)
{
    if (bytes <= 64 * 1024) return NM_OK;
    int dev = 0;
    NM_HIP_CHECK(hipGetDevice(&dev));
    const unsigned long long bit = 1ull << (dev & 63);
    static std::mutex mu;
    std::lock_guard<std::mutex> lk(mu);
    if (*done & bit) return NM_OK;
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) {
        set_error("hipFuncSetAttribute(LDS %zu) failed: %s", bytes, hipGetErrorString(e));
        return NM_ERR_HIP;
    }
    *done |= bit;
    return NM_OK;
}

namespace {

inline size_t elem_size(nm_dtype_t dt) { return dt == NM_F32 ? 4 : (dt == NM_BF16 ? 2 : 1); }
// the pairs the kernels exist for: fp32 -> fp32, bf16 -> bf16, E4M3 -> bf16
inline bool dtype_pair_ok(nm_dtype_t xdt, nm_dtype_t ydt)
{
    return (xdt == NM_F32 && ydt == NM_F32) || (xdt == NM_BF16 && ydt == NM_BF16) ||
           (xdt == NM_F8E4M3 && ydt == NM_BF16);
}

constexpr int kMaxLdsBytes = 160 * 1024;
constexpr int kNumCU = 256;

constexpr int kKeyInts = 24;
struct ShapeKey {
    int v[kKeyInts];
    bool operator<(const ShapeKey& o) const { return memcmp(v, o.v, sizeof(v)) < 0; }
};
struct CacheVal {
    int variant;
    float ms;
};

std::mutex g_mu;
std::map<ShapeKey, CacheVal> g_cache;
int g_forced = -1;

// 31-bit FNV-1a
unsigned fnv(unsigned h, const void* data, size_t n)
{
    const unsigned char* b = (const unsigned char*)data;
    for (size_t i = 0; i < n; ++i) h = (h ^ b[i]) * 16777619u;
    return h;
}

// Identity of a device for the tuning cache: a timing taken on one kind of GPU says
// nothing about another.  Architecture string and CU count, hashed; kept per ordinal.
struct DeviceId {
    int hash = 0;
    char name[128] = "";
};
const DeviceId* device_id(int dev)
{
    static std::mutex mu;
    static std::map<int, DeviceId> ids;
    std::lock_guard<std::mutex> lk(mu);
    auto it = ids.find(dev);
    if (it != ids.end()) return &it->second;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return nullptr;
    DeviceId id;
    // (the marketing name is left out: it comes from a system file that may be missing, and then
    //  differs from one process to the next)
    snprintf(id.name, sizeof(id.name), "%s|%dCU", prop.gcnArchName, prop.multiProcessorCount);
    for (char* c = id.name; *c; ++c)
        if (*c == ' ' || *c == '\n') *c = '_';   // one token in the cache file
    id.hash = (int)(fnv(2166136261u, id.name, strlen(id.name)) & 0x7fffffffu);
    return &ids.emplace(dev, id).first->second;
}

// Which variants may run a layer depends on its weights, not only on its shape: the
// k-steps per chunk its kept sets need (groups wider than a chunk spread unevenly) and
// which operand tables were built.  Two layers of one shape that differ there must not
// share a cache entry.
int prepack_signature(const nm_packed* wp)
{
    unsigned h = 2166136261u;
    for (const Prepack& pp : wp->prepacks) {
        const int t[5] = {pp.kind, pp.geom.CK, pp.geom.vec, pp.SPC, pp.par};
        h = fnv(h, t, sizeof(t));
    }
    return (int)(h & 0x7fffffffu);
}

ShapeKey make_key(nm_dtype_t xdt, nm_dtype_t ydt, int b, int h, int w, const nm_packed* wp,
                  int sh, int sw, int ph, int pw, int dh, int dw, int has_bias, int relu)
{
    ShapeKey k;
    const DeviceId* id = device_id(wp->device);
    const int vals[kKeyInts] = {(int)xdt, (int)ydt, b, h, w, wp->cin, wp->cout, wp->kh, wp->kw,
                                sh, sw, ph, pw, dh, dw, wp->n, wp->m, wp->tile, (int)wp->value_dtype,
                                has_bias ? 1 : 0, relu ? 1 : 0, id ? id->hash : 0, wp->sig, 0};
    memcpy(k.v, vals, sizeof(vals));
    return k;
}

// LDS footprint of variant d on the layer wp (the ring of the gather-free bf16
// kernel is only as deep as the layer's K loop is long).
size_t lds_bytes(const VariantDesc& d, const nm_packed* wp)
{
    // the epilogue's output tile [BP][channels of the workgroup] plus 16 bytes per pixel
    const size_t otile = (size_t)d.BP * ((size_t)(4 / d.WP) * d.NJ * 16 * (d.kind == 0 || d.kind == 5 ? 4 : 2) + 16);
    if (d.kind == 6)   // only the wavefront-private output tiles [16 NBLK][16 NJ] bf16 with 16 bytes of padding per row
        return (size_t)4 * 16 * d.NBLK * (d.NJ * 32 + 16);
    if (d.kind == 7) {   // up to three stages of the strip [BP][CK] bytes plus each wave's operands (1 KB per k-step and row block)
        const int nchunks = wp->kh * wp->kw * ((wp->cin + d.CK - 1) / d.CK);
        const size_t ops = d.areg ? 0 : (size_t)4 * d.NJ * (d.CK / 64) * 1024;
        return std::max(otile, (size_t)std::min(3, nchunks) * ((size_t)d.BP * d.CK + ops));
    }
    if (d.kind == 4)   // the strip [BP][64 SPC] bf16 plus the dense weights of the workgroup's row blocks
        return std::max(otile, (size_t)d.BP * d.SPC * 128 + (size_t)(4 / d.WP) * d.NJ * d.SPC * 2048);
    if (d.kind >= 2 && d.kind <= 4) {   // up to three stages of the strip [BP][CK] bf16 plus each wave's operands
        const int nchunks = wp->kh * wp->kw * ((wp->cin + d.CK - 1) / d.CK);
        const size_t ops = d.areg ? 0 : (size_t)4 * d.NJ * (d.CK / 64) * (d.kind == 2 ? 1024 + 256 : 2048);
        return std::max(otile, (size_t)std::min(3, nchunks) * ((size_t)d.BP * d.CK * 2 + ops));
    }
    if (d.kind == 1) {
        const int opr = d.CK / 8, pstep = 256 / opr, nit = (d.BP * opr + 255) / 256;
        const int rows = nit * pstep > d.BP ? nit * pstep : d.BP;
        return std::max(otile, (size_t)2 * rows * (d.CK * 2 + 4));
    }
    return std::max(otile, (size_t)2 * d.CK * strip_stride(d.BP, d.CK, d.vec != 0) * sizeof(float));
}

// The part of the convolution arguments that decides whether the kernel-row-run
// kernel applies and which of its two operand tables it needs.
struct RunArgs {
    int w, sw, pw, dw;
};

// k-steps the kernel-row-run kernel needs for this layer when runs start `par` elements early
int run_ksteps(const nm_packed* wp, int par)
{
    const int gr = (par + wp->kw * wp->cin + 7) / 8;
    return (wp->kh * gr + 7) / 8;
}

const Prepack* find_prepack(const nm_packed* wp, const VariantDesc& d, int par = -1)
{
    for (const Prepack& pp : wp->prepacks)
        if (pp.kind == d.kind && pp.geom.CK == d.CK && pp.geom.vec == d.vec && pp.SPC == d.SPC &&
            (d.vec || pp.d_ktab) && (d.kind != 4 || par < 0 || pp.par == par))
            return &pp;
    return nullptr;
}

// kinds 6 (register-streaming) and 7 (LDS-staged) are the fp8 kernels; they share one operand table layout
inline bool is_f8_kind(int kind) { return kind == 6 || kind == 7; }

// With `ra` the answer is for that convolution; without, "for some convolution".
bool variant_legal(int v, const nm_packed* wp, nm_dtype_t xdt, const RunArgs* ra = nullptr)
{
    if (v < 0 || v >= variant_count()) return false;
    const VariantDesc& d = variant_desc(v);
    if (lds_bytes(d, wp) > (size_t)kMaxLdsBytes) return false;
    if (d.kind == 5 && xdt != NM_F32) return false;   // instantiated for fp32 tensors only
    // fp8: E4M3 tensors with an E4M3 handle run the fp8 kernels and nothing else does
    if (is_f8_kind(d.kind) != (xdt == NM_F8E4M3) || is_f8_kind(d.kind) != (wp->value_dtype == NM_F8E4M3)) return false;
    if (d.kind >= 1 && d.kind <= 4) {
        // bf16 matrix cores: bf16 tensors, weights already rounded to bf16, and a
        // shared operand only for column tiles made of exactly two row blocks
        if (xdt != NM_BF16 || wp->value_dtype != NM_BF16) return false;
        if (d.share != 1 && d.share != wp->rbpt) return false;
    }
    if (d.ksplit > 1) {
        // every split must own at least one chunk of the K axis
        const Prepack* pp = find_prepack(wp, d);
        if (!pp) return false;
        const int cps = (pp->geom.nchunks + d.ksplit - 1) / d.ksplit;
        if ((d.ksplit - 1) * cps >= pp->geom.nchunks) return false;
    }
    if (d.kind == 4 && ra) {
        // a kernel row must be one contiguous, 4-byte aligned run of every pixel
        if (ra->dw != 1 || (ra->sw * wp->cin) % 2 != 0 || (ra->w * wp->cin) % 2 != 0) return false;
        return find_prepack(wp, d, (ra->pw * wp->cin) % 2) != nullptr;
    }
    return find_prepack(wp, d) != nullptr;
}

// Largest number of kept columns any (tile, chunk) pair holds.
int max_kept_per_chunk(const nm_packed* wp, const ChunkGeom& g)
{
    std::vector<int> cnt(g.nchunks);
    int best = 0;
    for (int j = 0; j < wp->n_tiles; ++j) {
        std::fill(cnt.begin(), cnt.end(), 0);
        for (int kk = 0; kk < wp->kprime; ++kk) {
            const int k = wp->h_idx[(size_t)j * wp->kprime + kk];
            int c;
            if (g.vec) {
                const int tap = k / wp->cin, ci = k - tap * wp->cin;
                c = tap * g.ncpt + ci / g.CK;
            } else {
                c = k / g.CK;
            }
            best = std::max(best, ++cnt[c]);
        }
    }
    return best;
}

struct Geometry {
    int Ho, Wo, P;
};

int conv_geometry(int b, int h, int w, const nm_packed* wp, int sh, int sw, int ph, int pw, int dh,
                  int dw, size_t es, Geometry* g)
{
    if (b < 1 || h < 1 || w < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1) {
        set_error("bad convolution arguments (sizes, stride, dilation must be >= 1, padding >= 0)");
        return NM_ERR_ARG;
    }
    const long eh = (long)h + 2L * ph - (long)dh * (wp->kh - 1) - 1;
    const long ew = (long)w + 2L * pw - (long)dw * (wp->kw - 1) - 1;
    if (eh < 0 || ew < 0) {
        set_error("output would be empty: input %dx%d, kernel %dx%d, pad %d,%d, dilation %d,%d", h, w,
                  wp->kh, wp->kw, ph, pw, dh, dw);
        return NM_ERR_SHAPE;
    }
    g->Ho = (int)(eh / sh) + 1;
    g->Wo = (int)(ew / sw) + 1;
    const long long P = (long long)b * g->Ho * g->Wo;
    const long long xin = (long long)b * h * w * wp->cin;
    const long long yout = P * wp->cout;
    if (P > 0x7fffffffLL - 1024 || xin > 0x7fffffffLL || yout > 0x7fffffffLL) {
        set_error("tensor too large: more than 2^31 - 1 elements");
        return NM_ERR_SHAPE;
    }
    if (xin * (long long)es >= 0x80000000LL) {
        set_error("input tensor too large: the kernels address x through a 2 GiB buffer window");
        return NM_ERR_SHAPE;
    }
    g->P = (int)P;
    return NM_OK;
}

// x / d for x < 2^31 as umulhi(2 x, mul) >> shift: shift = ceil(log2 d) and
// mul = floor(2^(31 + shift) / d) + 1, which fits 32 bits and is exact on that range.
void magic_div(unsigned d, unsigned* mul, unsigned* shift)
{
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    *mul = (unsigned)(((1ull << (31 + s)) / d) + 1);
    *shift = s;
}

void fill_params(ConvParams& p, const VariantDesc& d, const Prepack& pp, const nm_packed* wp,
                 const void* x, void* y, const float* bias, int b, int h, int w, const Geometry& g,
                 int sh, int sw, int ph, int pw, int dh, int dw, int relu, size_t es)
{
    p.x = x; p.y = y; p.bias = bias; p.res = nullptr;
    p.wfrag = pp.d_wfrag; p.rows = pp.d_rows; p.ktab = pp.d_ktab;
    p.wfrag_bytes = (unsigned)pp.wfrag_bytes; p.rows_bytes = (unsigned)pp.rows_bytes;
    p.B = b; p.H = h; p.W = w; p.Cin = wp->cin; p.Cout = wp->cout; p.Kh = wp->kh; p.Kw = wp->kw;
    p.Ho = g.Ho; p.Wo = g.Wo;
    p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.dh = dh; p.dw = dw;
    p.relu = relu ? 1 : 0;
    p.P = g.P; p.K = wp->K;
    p.nchunks = pp.geom.nchunks; p.ncpt = pp.geom.ncpt;
    p.tile = wp->tile; p.rbpt = wp->rbpt; p.n_rowblocks = wp->n_rowblocks;
    const int rb_per_wg = (4 / d.WP) * d.NJ;
    p.n_ptiles = (g.P + d.BP - 1) / d.BP;
    p.n_cblocks = (wp->n_rowblocks + rb_per_wg - 1) / rb_per_wg;
    p.oscale = 1.0f / wp->scale;
    p.ksplit = d.ksplit > 1 ? d.ksplit : 1;
    p.cps = (pp.geom.nchunks + p.ksplit - 1) / p.ksplit;
    p.partial = nullptr;   // the caller points it at a workspace of split_bytes()
    p.n_wg = p.n_ptiles * p.n_cblocks * p.ksplit;
    p.wg_per_xcd = (p.n_wg + 7) / 8;
    magic_div((unsigned)(g.Ho * g.Wo), &p.howo_mul, &p.howo_shift);
    magic_div((unsigned)g.Wo, &p.wo_mul, &p.wo_shift);
    p.x_elems = (unsigned)((size_t)b * h * w * wp->cin);
    p.x_bytes = (unsigned)((size_t)b * h * w * wp->cin * es);
    p.run_d = pp.par;
    p.run_gr = (pp.par + wp->kw * wp->cin + 7) / 8;
    magic_div((unsigned)p.run_gr, &p.gr_mul, &p.gr_shift);
    magic_div((unsigned)wp->cin, &p.cin_mul, &p.cin_shift);
}

// Deterministic default when the shape has not been tuned: a small model of
// "rounds of workgroups x work per workgroup", preferring tiles that fill the
// 256 CUs and reuse the staged strip across many row blocks.
//
// For the gather-free bf16 and the staged fp8 kernels the model is replaced by a rule read off
// tuned ResNet stacks (the model's picks ran x1.46 behind the tuned ones there): a tile of 128
// pixels x 128 channels (64 pixels where that leaves under half the CUs a workgroup, 64 channels
// where the layer has no more), all four wavefronts along the channels; producer wavefronts and
// register-held weights unless the launch is many rounds of workgroups on a 1x1 layer; 128-channel
// chunks on deep, small layers, 64 otherwise.  Variants are ranked by their distance from that.
int heuristic_variant(const nm_packed* wp, int P, nm_dtype_t xdt, const RunArgs* ra)
{
    {
        const long wg128 = (long)((P + 127) / 128) * ((wp->n_rowblocks + 7) / 8);
        const int bp_t = wg128 >= kNumCU / 2 ? 128 : 64;
        const int wgc_t = wp->n_rowblocks >= 8 ? 128 : 64;
        const long n_wg_t = (long)((P + bp_t - 1) / bp_t) * ((wp->n_rowblocks * 16 + wgc_t - 1) / wgc_t);
        const bool plain_t = wp->kh * wp->kw == 1 && n_wg_t >= 4L * kNumCU;
        const int ck_t = (wp->cin >= 256 && n_wg_t <= 2L * kNumCU) ? 128 : 64;
        auto lg = [](double a, double b) { return fabs(log2(a / b)); };
        int pick = -1;
        double pick_score = 0;
        for (int v = 0; v < variant_count(); ++v) {
            const VariantDesc& d = variant_desc(v);
            if (d.kind != 2 && d.kind != 3 && d.kind != 7) continue;
            if (!variant_legal(v, wp, xdt, ra)) continue;
            const int wgc = (4 / d.WP) * d.NJ * 16;
            double score = 4.0 * lg(d.BP, bp_t) + 4.0 * lg(wgc, wgc_t) + 1.0 * lg(d.CK, ck_t) + (d.WP != 1 ? 1.5 : 0.0);
            score += d.kind == 3 ? 6.0 : 0.0;                       // the sparse instruction where its operand exists
            score += plain_t ? (d.spec ? 2.0 : 0.0) : (d.areg ? 0.0 : d.spec ? 1.0 : 3.0);
            if (pick < 0 || score < pick_score - 1e-9) {
                pick = v;
                pick_score = score;
            }
        }
        if (pick >= 0) return pick;
    }
    int best = -1;
    double best_cost = 0;
    for (int v = 0; v < variant_count(); ++v) {
        if (!variant_legal(v, wp, xdt, ra)) continue;
        const VariantDesc& d = variant_desc(v);
        if (d.ksplit > 1) continue;   // a K split needs a workspace: only where the tuner has shown that it pays
        const int rb_per_wg = (4 / d.WP) * d.NJ;
        const long n_pt = (P + d.BP - 1) / d.BP;
        const long n_cb = (wp->n_rowblocks + rb_per_wg - 1) / rb_per_wg;
        const long n_wg = n_pt * n_cb;
        int occ = (int)std::min<size_t>(2, kMaxLdsBytes / lds_bytes(d, wp));
        if (occ < 1) occ = 1;
        const long rounds = (n_wg + (long)kNumCU * occ - 1) / ((long)kNumCU * occ);
        const double mfma = (double)d.BP * rb_per_wg;            // per chunk step, relative
        const double stage = (double)d.BP * 2.0;                 // staging cost per chunk, relative
        // the bf16 matrix-core kernel contracts several times faster where it applies
        const double speed[8] = {1.0, 0.3, 0.1, 0.2, 0.1, 0.7, 0.12, 0.1};   // relative cost of a unit of contraction
        const double cost = (double)rounds * occ * (mfma + stage) * speed[d.kind];
        if (best < 0 || cost < best_cost * 0.999) {
            best = v;
            best_cost = cost;
        }
    }
    return best;
}

// ---- workspace for the partial sums of K-split variants -----------------------------------
// One grow-only device buffer per device, shared by every call on that device (calls that
// overlap on different streams and both run a K-split variant would race on it: such variants
// are chosen only by the tuner or the test hook, and a serving loop that overlaps convolutions
// should not tune with them).  Growing it allocates, which a stream under capture cannot do.
size_t split_bytes(const VariantDesc& d, const Geometry& g, const nm_packed* wp)
{
    return d.ksplit > 1 ? (size_t)d.ksplit * (size_t)g.P * (size_t)wp->cout * sizeof(float) : 0;
}

struct Workspace {
    float* ptr = nullptr;
    size_t bytes = 0;
};
std::mutex g_ws_mu;
std::map<int, Workspace> g_ws;

// rc NM_OK and *out = a buffer of at least `bytes`, or an error; with may_alloc false the
// buffer must already be large enough
int get_workspace(int dev, size_t bytes, bool may_alloc, float** out)
{
    std::lock_guard<std::mutex> lk(g_ws_mu);
    Workspace& w = g_ws[dev];
    if (w.bytes < bytes) {
        if (!may_alloc) {
            set_error("the K-split workspace holds %zu bytes, this call needs %zu and may not allocate", w.bytes, bytes);
            return NM_ERR_ALLOC;
        }
        (void)hipFree(w.ptr);   // waits for the kernels still using it
        w.ptr = nullptr;
        w.bytes = 0;
        const size_t want = (bytes + ((size_t)1 << 20) - 1) & ~(((size_t)1 << 20) - 1);
        const hipError_t e = hipMalloc(reinterpret_cast<void**>(&w.ptr), want);
        if (e != hipSuccess) {
            w.ptr = nullptr;
            set_error("hipMalloc(%zu) for the K-split workspace failed: %s", want, hipGetErrorString(e));
            return NM_ERR_ALLOC;
        }
        w.bytes = want;
    }
    *out = w.ptr;
    return NM_OK;
}

int check_conv_args(const void* x, nm_dtype_t xdt, int cin, const nm_packed* wp, void* y,
                    nm_dtype_t ydt)
{
    if (!wp || !x || !y) {
        set_error("null pointer argument");
        return NM_ERR_ARG;
    }
    if (cin != wp->cin) {
        set_error("cin %d does not match the packed weights (%d)", cin, wp->cin);
        return NM_ERR_ARG;
    }
    if ((xdt != NM_F32 && xdt != NM_BF16 && xdt != NM_F8E4M3) || (ydt != NM_F32 && ydt != NM_BF16 && ydt != NM_F8E4M3)) {
        set_error("unknown dtype");
        return NM_ERR_ARG;
    }
    if (!dtype_pair_ok(xdt, ydt)) {
        set_error("unsupported dtype pair: fp32 -> fp32, bf16 -> bf16 or E4M3 -> bf16");
        return NM_ERR_UNSUPPORTED;
    }
    if ((xdt == NM_F8E4M3) != (wp->value_dtype == NM_F8E4M3)) {
        set_error("E4M3 activations need weights packed as E4M3 (and the other way round)");
        return NM_ERR_UNSUPPORTED;
    }
    if (((uintptr_t)x % 16) || ((uintptr_t)y % 16)) {
        set_error("x and y must be 16-byte aligned");
        return NM_ERR_ARG;
    }
    int dev = -1;
    NM_HIP_CHECK(hipGetDevice(&dev));
    if (dev != wp->device) {
        set_error("packed weights live on device %d, current device is %d", wp->device, dev);
        return NM_ERR_ARG;
    }
    return NM_OK;
}

void free_packed(nm_packed* wp)
{
    if (!wp) return;
    (void)hipFree(wp->d_idx);
    (void)hipFree(wp->d_vals);
    for (Prepack& pp : wp->prepacks) {
        (void)hipFree(pp.d_rows);
        (void)hipFree(pp.d_wfrag);
        (void)hipFree(pp.d_ktab);
    }
    delete wp;
}

}  // namespace
}  // namespace nm

using namespace nm;

extern "C" {

const char* nm_last_error(void) { return g_err; }

int nm_variant_count(void) { return variant_count(); }

const char* nm_variant_name(int variant)
{
    if (variant < 0 || variant >= variant_count()) return nullptr;
    return variant_desc(variant).name;
}

int nm_prune(const float* w, int cout, int kh, int kw, int cin, int n, int m, int tile,
             nm_dtype_t value_dtype, nm_packed_t** out)
{
    if (!w || !out) {
        set_error("null pointer argument");
        return NM_ERR_ARG;
    }
    *out = nullptr;
    if (cout < 1 || kh < 1 || kw < 1 || cin < 1 || n < 1 || m < 1 || tile < 1 || n > m) {
        set_error("bad sizes: cout %d kh %d kw %d cin %d n %d m %d tile %d", cout, kh, kw, cin, n, m, tile);
        return NM_ERR_ARG;
    }
    if (value_dtype != NM_F32 && value_dtype != NM_BF16 && value_dtype != NM_F8E4M3) {
        set_error("unknown value dtype");
        return NM_ERR_ARG;
    }
    if (value_dtype == NM_F8E4M3 && (cin % 64 != 0 || tile % 16 != 0 || cout % 8 != 0)) {
        set_error("E4M3 weights need cin %% 64 == 0, tile %% 16 == 0 and cout %% 8 == 0 (cin %d, tile %d, cout %d)",
                  cin, tile, cout);
        return NM_ERR_UNSUPPORTED;
    }
    const long long K = (long long)kh * kw * cin;
    if (K % m != 0) {
        set_error("K = %lld is not a multiple of m = %d", K, m);
        return NM_ERR_ARG;
    }
    if (m > 16384) {
        set_error("m = %d exceeds the supported group size 16384", m);
        return NM_ERR_ARG;
    }
    if (K * cout > 0x7fffffffLL) {
        set_error("weight tensor too large");
        return NM_ERR_ARG;
    }
    const size_t nw = (size_t)cout * K;
    for (size_t i = 0; i < nw; ++i)
        if (!isfinite(w[i])) {
            set_error("weight %zu is not finite", i);
            return NM_ERR_ARG;
        }

    nm_packed* wp = new (std::nothrow) nm_packed();
    if (!wp) {
        set_error("out of host memory");
        return NM_ERR_ALLOC;
    }
    wp->cout = cout; wp->kh = kh; wp->kw = kw; wp->cin = cin; wp->K = (int)K;
    wp->n = n; wp->m = m; wp->tile = tile;
    wp->G = (int)(K / m); wp->kprime = wp->G * n; wp->n_tiles = (cout + tile - 1) / tile;
    wp->rbpt = (tile + 15) / 16; wp->n_rowblocks = wp->n_tiles * wp->rbpt;
    wp->value_dtype = value_dtype;

    float* d_w = nullptr;
    int rc = NM_OK;
    hipStream_t s = nullptr;
    auto fail = [&](int code) {
        (void)hipFree(d_w);
        free_packed(wp);
        return code;
    };
#define NM_TRY_HIP(expr, code)                                                             \
    do {                                                                                   \
        hipError_t e__ = (expr);                                                           \
        if (e__ != hipSuccess) {                                                           \
            set_error("%s failed: %s", #expr, hipGetErrorString(e__));                     \
            return fail(code);                                                             \
        }                                                                                  \
    } while (0)

    NM_TRY_HIP(hipGetDevice(&wp->device), NM_ERR_HIP);
    NM_TRY_HIP(hipMalloc(&d_w, nw * sizeof(float)), NM_ERR_ALLOC);
    NM_TRY_HIP(hipMalloc(&wp->d_idx, (size_t)wp->n_tiles * wp->kprime * sizeof(int32_t)), NM_ERR_ALLOC);
    NM_TRY_HIP(hipMalloc(&wp->d_vals, (size_t)wp->n_tiles * wp->kprime * tile * sizeof(float)), NM_ERR_ALLOC);
    NM_TRY_HIP(hipMemcpyAsync(d_w, w, nw * sizeof(float), hipMemcpyHostToDevice, s), NM_ERR_HIP);
    rc = run_prune(d_w, wp, s);
    if (rc != NM_OK) return fail(rc);
    wp->h_idx.resize((size_t)wp->n_tiles * wp->kprime);
    NM_TRY_HIP(hipMemcpyAsync(wp->h_idx.data(), wp->d_idx, wp->h_idx.size() * sizeof(int32_t),
                              hipMemcpyDeviceToHost, s), NM_ERR_HIP);
    NM_TRY_HIP(hipStreamSynchronize(s), NM_ERR_HIP);

    if (value_dtype == NM_F8E4M3) {
        // one power-of-two scale per layer: the largest 2^e that keeps every kept weight within
        // the format (|w| 2^e <= 448); the kept values become the E4M3 numbers they are stored as
        float most = 0.f;
        for (int j = 0; j < wp->n_tiles; ++j)
            for (int kk = 0; kk < wp->kprime; ++kk) {
                const size_t k = (size_t)wp->h_idx[(size_t)j * wp->kprime + kk];
                const int r1 = std::min(cout, (j + 1) * tile);
                for (int r = j * tile; r < r1; ++r) most = std::max(most, fabsf(w[(size_t)r * K + k]));
            }
        float scale = 1.f;
        if (most > 0.f) {
            int e = 0;
            (void)frexpf(448.0f / most, &e);       // 448 / most = f 2^e with 0.5 <= f < 1
            scale = ldexpf(1.0f, e - 1);
            while (most * scale > 448.0f) scale *= 0.5f;   // the quotient above is rounded
        }
        wp->scale = scale;
        rc = run_quantize_e4m3(wp, s);
        if (rc != NM_OK) return fail(rc);
    }

    // Operand tables for every chunk geometry a kernel variant may ask for.
    const bool vec_ok = cin % 4 == 0;
    for (int v = 0; v < variant_count(); ++v) {
        const VariantDesc& d = variant_desc(v);
        if (is_f8_kind(d.kind) != (value_dtype == NM_F8E4M3)) continue;   // E4M3 handles feed the fp8 kernels only
        if (is_f8_kind(d.kind)) {
            // one table layout for both kernels (64-channel k-steps in K order); an entry per
            // chunk size, because the chunk geometry travels with the table
            if (cin % d.CK != 0 || find_prepack(wp, d)) continue;
            Prepack pp;
            pp.kind = d.kind;
            pp.geom = make_chunk_geom(cin, wp->K, d.CK, 1);
            pp.SPC = d.SPC;
            pp.rows_bytes = 0;
            pp.wfrag_bytes = (size_t)wp->n_rowblocks * (wp->K / 64) * 64 * 16;
            if (pp.wfrag_bytes >= 0x80000000ull) continue;
            wp->prepacks.push_back(pp);
            Prepack& ref = wp->prepacks.back();
            NM_TRY_HIP(hipMalloc(reinterpret_cast<void**>(&ref.d_wfrag), ref.wfrag_bytes), NM_ERR_ALLOC);
            rc = run_build_prepack(wp, ref, s);
            if (rc != NM_OK) return fail(rc);
            continue;
        }
        if (d.kind == 4) {
            // kernel-row runs: only where channel runs are too short for the other bf16 kernels
            if (value_dtype != NM_BF16 || cin % 8 == 0) continue;
            for (int par = 0; par < 2; ++par) {
                if (run_ksteps(wp, par) != d.SPC || find_prepack(wp, d, par)) continue;
                Prepack pp;
                pp.kind = 4;
                pp.geom.vec = 1; pp.geom.CK = d.CK; pp.geom.ncpt = 1; pp.geom.nchunks = 1;
                pp.SPC = d.SPC;
                pp.par = par;
                pp.rows_bytes = 0;
                pp.wfrag_bytes = (size_t)wp->n_rowblocks * pp.SPC * 2 * 64 * 8 * sizeof(uint16_t);
                wp->prepacks.push_back(pp);
                Prepack& ref = wp->prepacks.back();
                NM_TRY_HIP(hipMalloc(reinterpret_cast<void**>(&ref.d_wfrag), ref.wfrag_bytes), NM_ERR_ALLOC);
                rc = run_build_prepack(wp, ref, s);
                if (rc != NM_OK) return fail(rc);
            }
            continue;
        }
        if (d.kind == 5) {
            if (!vec_ok || value_dtype != NM_F32) continue;
        } else if (d.kind >= 2) {
            // gather-free bf16 kernel: whole 64-channel k-steps of one tap per chunk; the
            // sparse operand holds at most 2 kept columns per aligned group of 4
            if (value_dtype != NM_BF16 || cin % d.CK != 0) continue;
            if (d.kind == 2 && !(n <= 2 && m % 4 == 0)) continue;
        } else if (d.kind == 1) {
            if (value_dtype != NM_BF16 || cin % 8 != 0) continue;
        } else if ((d.vec != 0) != vec_ok) {
            continue;
        }
        if (find_prepack(wp, d)) continue;
        const ChunkGeom g = make_chunk_geom(cin, wp->K, d.CK, d.vec);
        if (d.kind < 2) {
            const int per_step = d.kind == 1 ? 32 : 4;   // kept columns per k-step
            const int need = (max_kept_per_chunk(wp, g) + per_step - 1) / per_step;
            // smallest instantiated SPC >= need for this (kind, CK, mode)
            int pick = 0;
            for (int u = 0; u < variant_count(); ++u) {
                const VariantDesc& e = variant_desc(u);
                if (e.kind == d.kind && e.CK == d.CK && e.vec == d.vec && e.SPC >= need &&
                    (pick == 0 || e.SPC < pick))
                    pick = e.SPC;
            }
            if (pick == 0 || pick != d.SPC) continue;
        } else if (d.kind == 5) {
            // worth its table only where the kept columns are spread unevenly over the
            // chunks: otherwise the fixed-step form does the same work
            const int most = max_kept_per_chunk(wp, g);
            if ((long)most * g.nchunks * 10 <= (long)wp->kprime * 11) continue;
        }
        Prepack pp;
        pp.kind = d.kind;
        pp.geom = g;
        pp.SPC = d.SPC;
        size_t rows_bytes, wf_bytes;
        if (d.kind >= 2 && d.kind <= 4) {
            rows_bytes = (size_t)wp->n_tiles * g.nchunks * 4 * pp.SPC * sizeof(uint32_t);
            wf_bytes = (size_t)wp->n_rowblocks * g.nchunks * pp.SPC * (d.kind == 2 ? 1 : 2) * 64 * 8 *
                       sizeof(uint16_t);
        } else if (d.kind == 1) {
            rows_bytes = (size_t)wp->n_tiles * g.nchunks * pp.SPC * 4 * 8 * sizeof(uint32_t);
            wf_bytes = (size_t)wp->n_rowblocks * g.nchunks * pp.SPC * 64 * 8 * sizeof(uint16_t);
        } else {
            rows_bytes = (size_t)wp->n_tiles * g.nchunks * 4 * pp.SPC * sizeof(uint32_t);
            wf_bytes = (size_t)wp->n_rowblocks * g.nchunks * 64 * pp.SPC * sizeof(float);
        }
        if (wf_bytes >= 0x80000000ull || rows_bytes >= 0x80000000ull) continue;   // 2 GiB buffer windows
        pp.rows_bytes = rows_bytes;
        pp.wfrag_bytes = wf_bytes;
        NM_TRY_HIP(hipMalloc(&pp.d_rows, rows_bytes), NM_ERR_ALLOC);
        wp->prepacks.push_back(pp);   // owned by the handle from here on
        Prepack& ref = wp->prepacks.back();
        NM_TRY_HIP(hipMalloc(reinterpret_cast<void**>(&ref.d_wfrag), wf_bytes), NM_ERR_ALLOC);
        NM_TRY_HIP(hipMemsetAsync(ref.d_rows, 0, rows_bytes, s), NM_ERR_HIP);
        NM_TRY_HIP(hipMemsetAsync(ref.d_wfrag, 0, wf_bytes, s), NM_ERR_HIP);
        rc = run_build_prepack(wp, ref, s);
        if (rc != NM_OK) return fail(rc);
        if (!g.vec) {
            // decode table of the flat k axis (layout only: which tap and channel row k is)
            if (kh > 255 || kw > 255 || cin > 65535) continue;
            std::vector<uint32_t> kt((size_t)g.nchunks * g.CK, 0xffffffffu);
            for (int k = 0; k < wp->K; ++k) {
                const int tap = k / cin, ci = k - tap * cin;
                kt[k] = (uint32_t)(tap / kw) | ((uint32_t)(tap % kw) << 8) | ((uint32_t)ci << 16);
            }
            NM_TRY_HIP(hipMalloc(&ref.d_ktab, kt.size() * sizeof(uint32_t)), NM_ERR_ALLOC);
            NM_TRY_HIP(hipMemcpy(ref.d_ktab, kt.data(), kt.size() * sizeof(uint32_t), hipMemcpyHostToDevice),
                       NM_ERR_HIP);
        }
    }
#undef NM_TRY_HIP
    (void)hipFree(d_w);
    if (wp->prepacks.empty()) {
        set_error("no kernel variant can run this layer (cin %d, n:m %d:%d, tile %d)", cin, n, m, tile);
        free_packed(wp);
        return NM_ERR_UNSUPPORTED;
    }
    wp->sig = prepack_signature(wp);
    *out = wp;
    return NM_OK;
}

int nm_packed_free(nm_packed_t* wp)
{
    free_packed(wp);
    return NM_OK;
}

int nm_packed_dims(const nm_packed_t* wp, int* n_tiles, int* groups, int* n, int* kprime)
{
    if (!wp) {
        set_error("null handle");
        return NM_ERR_ARG;
    }
    if (n_tiles) *n_tiles = wp->n_tiles;
    if (groups) *groups = wp->G;
    if (n) *n = wp->n;
    if (kprime) *kprime = wp->kprime;
    return NM_OK;
}

int nm_packed_indices(const nm_packed_t* wp, int32_t* idx_host)
{
    if (!wp || !idx_host) {
        set_error("null pointer argument");
        return NM_ERR_ARG;
    }
    NM_HIP_CHECK(hipMemcpy(idx_host, wp->d_idx, (size_t)wp->n_tiles * wp->kprime * sizeof(int32_t),
                           hipMemcpyDeviceToHost));
    return NM_OK;
}

int nm_packed_values(const nm_packed_t* wp, float* vals_host)
{
    if (!wp || !vals_host) {
        set_error("null pointer argument");
        return NM_ERR_ARG;
    }
    NM_HIP_CHECK(hipMemcpy(vals_host, wp->d_vals,
                           (size_t)wp->n_tiles * wp->kprime * wp->tile * sizeof(float),
                           hipMemcpyDeviceToHost));
    return NM_OK;
}

int nm_packed_mask(const nm_packed_t* wp, uint8_t* mask_host)
{
    if (!wp || !mask_host) {
        set_error("null pointer argument");
        return NM_ERR_ARG;
    }
    uint8_t* d_mask = nullptr;
    const size_t bytes = (size_t)wp->cout * wp->K;
    hipError_t e = hipMalloc(&d_mask, bytes);
    if (e != hipSuccess) {
        set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
        return NM_ERR_ALLOC;
    }
    int rc = run_build_mask(wp, d_mask, nullptr);
    if (rc == NM_OK) {
        e = hipMemcpy(mask_host, d_mask, bytes, hipMemcpyDeviceToHost);
        if (e != hipSuccess) {
            set_error("hipMemcpy failed: %s", hipGetErrorString(e));
            rc = NM_ERR_HIP;
        }
    }
    (void)hipFree(d_mask);
    return rc;
}

int nm_packed_scale(const nm_packed_t* wp, float* scale)
{
    if (!wp || !scale) {
        set_error("null pointer argument");
        return NM_ERR_ARG;
    }
    *scale = wp->scale;
    return NM_OK;
}

int nm_force_variant(int v)
{
    if (v < -1 || v >= variant_count()) {
        set_error("variant %d out of range", v);
        return NM_ERR_ARG;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    g_forced = v;
    return NM_OK;
}

int nm_last_variant(void) { return g_last_variant; }

int nm_variant_legal(int variant, const nm_packed_t* wp, nm_dtype_t xdt, nm_dtype_t ydt)
{
    if (!wp || variant < 0 || variant >= variant_count()) {
        set_error("bad arguments");
        return NM_ERR_ARG;
    }
    if (!dtype_pair_ok(xdt, ydt)) return 0;
    return variant_legal(variant, wp, xdt) ? 1 : 0;
}

static int conv2d_impl(const void* x, nm_dtype_t xdt, int b, int h, int w, int cin, const nm_packed_t* wp,
                       const float* bias, const void* res, int sh, int sw, int ph, int pw, int dh, int dw,
                       int relu, void* y, nm_dtype_t ydt, void* stream, bool static_only = false)
{
    int rc = check_conv_args(x, xdt, cin, wp, y, ydt);
    if (rc != NM_OK) return rc;
    if (res && ((uintptr_t)res % 16)) {
        set_error("residual must be 16-byte aligned");
        return NM_ERR_ARG;
    }
    Geometry g;
    rc = conv_geometry(b, h, w, wp, sh, sw, ph, pw, dh, dw, elem_size(xdt), &g);
    if (rc != NM_OK) return rc;
    if (res) {
        const size_t ybytes = (size_t)g.P * wp->cout * elem_size(ydt);
        const uintptr_t r0 = (uintptr_t)res, y0 = (uintptr_t)y;
        if (r0 < y0 + ybytes && y0 < r0 + ybytes) {
            set_error("residual must not overlap y");
            return NM_ERR_ARG;
        }
    }

    int v = -1;
    bool forced = false;
    {
        const ShapeKey key = make_key(xdt, ydt, b, h, w, wp, sh, sw, ph, pw, dh, dw, bias != nullptr, relu);
        std::lock_guard<std::mutex> lk(g_mu);
        if (g_forced >= 0) {
            v = g_forced;
            forced = true;
        } else {
            auto it = g_cache.find(key);
            if (it != g_cache.end()) v = it->second.variant;
        }
    }
    const RunArgs ra = {w, sw, pw, dw};
    if (v >= 0 && !variant_legal(v, wp, xdt, &ra)) {
        if (forced) {
            set_error("variant %d (%s) cannot run this layer", v, nm_variant_name(v));
            return NM_ERR_UNSUPPORTED;
        }
        v = -1;   // stale cache entry: fall back to the default
    }
    if (v < 0) v = heuristic_variant(wp, g.P, xdt, &ra);
    if (v < 0) {
        set_error("no kernel variant can run this layer");
        return NM_ERR_UNSUPPORTED;
    }
    const VariantDesc& d = variant_desc(v);
    ConvParams p;
    fill_params(p, d, *find_prepack(wp, d, (pw * wp->cin) % 2), wp, x, y, bias, b, h, w, g, sh, sw, ph, pw,
                dh, dw, relu, elem_size(xdt));
    p.res = res;
    if (d.ksplit > 1) {
        const size_t need = split_bytes(d, g, wp);
        if (static_only) {
            if (need > kStaticScratchBytes) {
                set_error("variant %s needs %zu bytes of scratch for its partial sums; the static buffer holds %u",
                          d.name, need, (unsigned)kStaticScratchBytes);
                return NM_ERR_SHAPE;
            }
            rc = static_scratch(wp->device, &p.partial);
        } else {
            // growing the workspace allocates, which a stream under capture must not do
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            (void)hipStreamIsCapturing((hipStream_t)stream, &cs);
            rc = get_workspace(wp->device, need, cs == hipStreamCaptureStatusNone, &p.partial);
        }
        if (rc != NM_OK) return rc;
    }
    rc = launch_conv(v, xdt, ydt, p, (hipStream_t)stream);
    if (rc == NM_OK && d.ksplit > 1) rc = run_splitk_reduce(p, ydt, (hipStream_t)stream);
    if (rc == NM_OK) g_last_variant = v;
    return rc;
}

int nm_conv2d(const void* x, nm_dtype_t xdt, int b, int h, int w, int cin, const nm_packed_t* wp,
              const float* bias, int sh, int sw, int ph, int pw, int dh, int dw, int relu, void* y,
              nm_dtype_t ydt, void* stream)
{
    return conv2d_impl(x, xdt, b, h, w, cin, wp, bias, nullptr, sh, sw, ph, pw, dh, dw, relu, y, ydt, stream);
}

int nm_conv2d_res(const void* x, nm_dtype_t xdt, int b, int h, int w, int cin, const nm_packed_t* wp,
                  const float* bias, const void* res, int sh, int sw, int ph, int pw, int dh, int dw,
                  int relu, void* y, nm_dtype_t ydt, void* stream)
{
    return conv2d_impl(x, xdt, b, h, w, cin, wp, bias, res, sh, sw, ph, pw, dh, dw, relu, y, ydt, stream);
}

int nm_conv2d_static(const void* x, nm_dtype_t xdt, int b, int h, int w, int cin, const nm_packed_t* wp,
                     const float* bias, const void* res, int sh, int sw, int ph, int pw, int dh, int dw,
                     int relu, void* y, nm_dtype_t ydt, void* stream)
{
    return conv2d_impl(x, xdt, b, h, w, cin, wp, bias, res, sh, sw, ph, pw, dh, dw, relu, y, ydt, stream, true);
}

int nm_maxpool2d(const void* x, nm_dtype_t dt, int b, int h, int w, int c, int k, int stride, int pad,
                 void* y, void* stream)
{
    if (!x || !y || b < 1 || h < 1 || w < 1 || c < 1 || k < 1 || stride < 1 || pad < 0 || pad >= k ||
        (dt != NM_F32 && dt != NM_BF16)) {
        set_error("bad max-pooling arguments");
        return NM_ERR_ARG;
    }
    if (h + 2 * pad < k || w + 2 * pad < k) {
        set_error("output would be empty: input %dx%d, window %d, pad %d", h, w, k, pad);
        return NM_ERR_SHAPE;
    }
    const int ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    if (((uintptr_t)x % 16) || ((uintptr_t)y % 16)) {
        set_error("x and y must be 16-byte aligned");
        return NM_ERR_ARG;
    }
    return run_maxpool(x, dt, b, h, w, c, k, stride, pad, ho, wo, y, (hipStream_t)stream);
}

int nm_im2col(const void* x, nm_dtype_t dt, int b, int h, int w, int cin, int kh, int kw, int sh, int sw,
              int ph, int pw, int dh, int dw, void* a_out, void* stream)
{
    if (!x || !a_out || b < 1 || h < 1 || w < 1 || cin < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 ||
        pw < 0 || dh < 1 || dw < 1 || (dt != NM_F32 && dt != NM_BF16)) {
        set_error("bad im2col arguments");
        return NM_ERR_ARG;
    }
    if (((uintptr_t)x % 16) || ((uintptr_t)a_out % 16)) {
        set_error("x and a must be 16-byte aligned");
        return NM_ERR_ARG;
    }
    const long eh = (long)h + 2L * ph - (long)dh * (kh - 1) - 1, ew = (long)w + 2L * pw - (long)dw * (kw - 1) - 1;
    if (eh < 0 || ew < 0) {
        set_error("output would be empty");
        return NM_ERR_SHAPE;
    }
    const int ho = (int)(eh / sh) + 1, wo = (int)(ew / sw) + 1;
    if ((long long)b * ho * wo * kh * kw * cin > 0x7fffffffLL * 4) {
        set_error("im2col matrix too large");
        return NM_ERR_SHAPE;
    }
    return run_im2col(x, dt, b, h, w, cin, kh, kw, sh, sw, ph, pw, dh, dw, ho, wo, a_out, (hipStream_t)stream);
}

int nm_stream_floor(const void* x, size_t x_bytes, void* y, size_t y_bytes, void* stream)
{
    if (!x || !y || ((uintptr_t)x % 16) || ((uintptr_t)y % 16)) {
        set_error("x and y must be non-null and 16-byte aligned");
        return NM_ERR_ARG;
    }
    return run_stream_floor(x, x_bytes, y, y_bytes, (hipStream_t)stream);
}

int nm_avgpool_global(const void* x, nm_dtype_t dt, int b, int h, int w, int c, void* y, void* stream)
{
    if (!x || !y || b < 1 || h < 1 || w < 1 || c < 1 || (dt != NM_F32 && dt != NM_BF16)) {
        set_error("bad average-pooling arguments");
        return NM_ERR_ARG;
    }
    if (b > 65535) {
        set_error("batch %d exceeds 65535", b);
        return NM_ERR_ARG;
    }
    return run_avgpool(x, dt, b, h * w, c, y, (hipStream_t)stream);
}

int nm_autotune(nm_dtype_t xdt, int b, int h, int w, int cin, const nm_packed_t* wp, int has_bias,
                int sh, int sw, int ph, int pw, int dh, int dw, int relu, nm_dtype_t ydt,
                void* stream, int* chosen, float* best_ms)
{
    if (!wp) {
        set_error("null handle");
        return NM_ERR_ARG;
    }
    if (cin != wp->cin) {
        set_error("cin %d does not match the packed weights (%d)", cin, wp->cin);
        return NM_ERR_ARG;
    }
    if (!dtype_pair_ok(xdt, ydt) || (xdt == NM_F8E4M3) != (wp->value_dtype == NM_F8E4M3)) {
        set_error("unsupported dtype pair: fp32 -> fp32, bf16 -> bf16 or E4M3 -> bf16 (E4M3 with E4M3 weights)");
        return NM_ERR_UNSUPPORTED;
    }
    Geometry g;
    int rc = conv_geometry(b, h, w, wp, sh, sw, ph, pw, dh, dw, elem_size(xdt), &g);
    if (rc != NM_OK) return rc;
    const ShapeKey key = make_key(xdt, ydt, b, h, w, wp, sh, sw, ph, pw, dh, dw, has_bias, relu);
    const RunArgs ra = {w, sw, pw, dw};
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_cache.find(key);
        if (it != g_cache.end() && variant_legal(it->second.variant, wp, xdt, &ra)) {
            if (chosen) *chosen = it->second.variant;
            if (best_ms) *best_ms = it->second.ms;
            return NM_OK;
        }
    }
    hipStream_t s = (hipStream_t)stream;
    const size_t es = elem_size(xdt), yes = elem_size(ydt);
    const size_t xn = (size_t)b * h * w * cin, yn = (size_t)g.P * wp->cout;
    // Cold-cache protocol: in a network every layer finds the 256 MB last-level
    // cache full of other layers' data, so the candidates are timed on a ring
    // of input/output sets (about 768 MB in total) and no launch reuses the
    // set of a recent one.
    const size_t xbytes = (xn * es + 255) & ~(size_t)255, ybytes = (yn * yes + 255) & ~(size_t)255;
    const size_t pool = (size_t)768 << 20;
    int nbuf = (int)std::min<size_t>(64, std::max<size_t>(1, pool / (xbytes + ybytes)));
    char* dpool = nullptr;
    float* dbias = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(dpool); (void)hipFree(dbias);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    };
#define NM_TRY(expr, code)                                                       \
    do {                                                                         \
        hipError_t e__ = (expr);                                                 \
        if (e__ != hipSuccess) {                                                 \
            set_error("%s failed: %s", #expr, hipGetErrorString(e__));           \
            cleanup();                                                           \
            return code;                                                         \
        }                                                                        \
    } while (0)
    NM_TRY(hipMalloc(&dpool, (xbytes + ybytes) * nbuf), NM_ERR_ALLOC);
    if (has_bias) {
        NM_TRY(hipMalloc(&dbias, wp->cout * sizeof(float)), NM_ERR_ALLOC);
        rc = run_fill_random(dbias, wp->cout, NM_F32, 7u, s);
        if (rc != NM_OK) { cleanup(); return rc; }
    }
    for (int i = 0; i < nbuf; ++i) {
        rc = run_fill_random(dpool + (xbytes + ybytes) * i, xn, xdt, 1u + i, s);
        if (rc != NM_OK) { cleanup(); return rc; }
    }
    NM_TRY(hipEventCreate(&e0), NM_ERR_HIP);
    NM_TRY(hipEventCreate(&e1), NM_ERR_HIP);

    int best_v = -1;
    float best = 0.f;
    int turn = 0;
    int rc_t = NM_OK;
    // one timed group of `reps` launches of variant v on fresh tensor sets: ms per launch, < 0 on error
    auto time_group = [&](int v, int reps) -> float {
        const VariantDesc& d = variant_desc(v);
        const Prepack* pp = find_prepack(wp, d, (pw * wp->cin) % 2);
        ConvParams p;
        float* partial = nullptr;
        if (d.ksplit > 1) {   // sized here, once: nm_conv2d then finds the workspace large enough
            rc_t = get_workspace(wp->device, split_bytes(d, g, wp), true, &partial);
            if (rc_t != NM_OK) return -1.f;
        }
        if (hipEventRecord(e0, s) != hipSuccess) { rc_t = NM_ERR_HIP; return -1.f; }
        for (int i = 0; i < reps; ++i) {
            char* set = dpool + (xbytes + ybytes) * (turn++ % nbuf);
            fill_params(p, d, *pp, wp, set, set + xbytes, dbias, b, h, w, g, sh, sw, ph, pw, dh, dw, relu, es);
            p.partial = partial;
            rc_t = launch_conv(v, xdt, ydt, p, s);
            if (rc_t == NM_OK && d.ksplit > 1) rc_t = run_splitk_reduce(p, ydt, s);
            if (rc_t != NM_OK) return -1.f;
        }
        float ms = 0.f;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            set_error("timing a tuning candidate failed");
            rc_t = NM_ERR_HIP;
            return -1.f;
        }
        return ms / reps;
    };
    // First pass: every legal variant, one warm-up launch (code object, attributes) and the
    // median of three groups.  Second pass: the five fastest (up to ten if that close) again, interleaved so that clock
    // and cache drift hit them alike, median of seven groups -- single passes were seen to
    // pick variants a few percent off the best from run to run.
    std::vector<std::pair<float, int>> first;
    for (int v = 0; v < variant_count(); ++v) {
        if (!variant_legal(v, wp, xdt, &ra)) continue;
        {   // a K split is worth its second kernel only where the output tiles are one short, ragged round (at most two per CU)
            const VariantDesc& d = variant_desc(v);
            const long tiles = (long)((g.P + d.BP - 1) / d.BP) *
                               ((wp->n_rowblocks + (4 / d.WP) * d.NJ - 1) / ((4 / d.WP) * d.NJ));
            if (d.ksplit > 1 && (tiles > 2 * kNumCU || tiles * d.ksplit > 8 * kNumCU)) continue;
        }
        if (time_group(v, 1) < 0.f) { cleanup(); return rc_t; }
        float t[3];
        for (int r = 0; r < 3; ++r)
            if ((t[r] = time_group(v, 3)) < 0.f) { cleanup(); return rc_t; }
        std::sort(t, t + 3);
        first.push_back(std::make_pair(t[1], v));
    }
    std::sort(first.begin(), first.end());
    if (getenv("NM_TUNE_VERBOSE")) {   // the whole field, fastest first: what the choice was made from
        fprintf(stderr, "nm_autotune %dx%dx%d -> %d, %dx%d, b %d, %d:%d T%d: %zu candidates\n", h, w, cin, wp->cout,
                wp->kh, wp->kw, b, wp->n, wp->m, wp->tile, first.size());
        for (const auto& c : first) fprintf(stderr, "  %9.2f us  %s\n", c.first * 1e3f, variant_desc(c.second).name);
    }
    // finalists: the five fastest, and whatever else came within 5 % of the fastest (at most ten)
    int finalists = (int)std::min<size_t>(5, first.size());
    while (finalists < (int)std::min<size_t>(10, first.size()) && first[finalists].first <= first[0].first * 1.05f)
        ++finalists;
    std::vector<std::vector<float>> again(finalists);
    for (int r = 0; r < 7 && finalists > 1; ++r)
        for (int c = 0; c < finalists; ++c) {
            const float t = time_group(first[c].second, 4);
            if (t < 0.f) { cleanup(); return rc_t; }
            again[c].push_back(t);
        }
    for (int c = 0; c < finalists; ++c) {
        float t = first[c].first;
        if (!again[c].empty()) {
            std::sort(again[c].begin(), again[c].end());
            t = again[c][again[c].size() / 2];
        }
        if (best_v < 0 || t < best) {
            best_v = first[c].second;
            best = t;
        }
    }
#undef NM_TRY
    cleanup();
    if (best_v < 0) {
        set_error("no kernel variant can run this layer");
        return NM_ERR_UNSUPPORTED;
    }
    {
        std::lock_guard<std::mutex> lk(g_mu);
        g_cache[key] = CacheVal{best_v, best};
    }
    if (chosen) *chosen = best_v;
    if (best_ms) *best_ms = best;
    return NM_OK;
}

int nm_autotune_tile(const float* w, int cout, int kh, int kw, int cin, int n, int m,
                     const int* tiles, int n_candidates, nm_dtype_t value_dtype,
                     nm_dtype_t xdt, int b, int h, int wd, int has_bias,
                     int sh, int sw, int ph, int pw, int dh, int dw, int relu, nm_dtype_t ydt,
                     void* stream, nm_packed_t** out, int* best_tile, float* ms_per_candidate)
{
    if (!out || !tiles || n_candidates < 1) {
        set_error("null output or empty candidate list");
        return NM_ERR_ARG;
    }
    *out = nullptr;
    nm_packed_t* best = nullptr;
    float best_ms = 0.f;
    for (int i = 0; i < n_candidates; ++i) {
        nm_packed_t* wp = nullptr;
        int rc = nm_prune(w, cout, kh, kw, cin, n, m, tiles[i], value_dtype, &wp);
        float ms = 0.f;
        if (rc == NM_OK)
            rc = nm_autotune(xdt, b, h, wd, cin, wp, has_bias, sh, sw, ph, pw, dh, dw, relu, ydt, stream,
                             nullptr, &ms);
        if (rc != NM_OK) {   // the message of the failing call stands
            free_packed(wp);
            free_packed(best);
            return rc;
        }
        if (ms_per_candidate) ms_per_candidate[i] = ms;
        if (!best || ms < best_ms) {
            free_packed(best);
            best = wp;
            best_ms = ms;
            if (best_tile) *best_tile = tiles[i];
        } else {
            free_packed(wp);
        }
    }
    *out = best;
    return NM_OK;
}

int nm_workspace_free(void)
{
    std::lock_guard<std::mutex> lk(g_ws_mu);
    for (auto& kv : g_ws) {
        (void)hipFree(kv.second.ptr);   // waits for the kernels still using it
        kv.second = Workspace();
    }
    return NM_OK;
}

int nm_cache_clear(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_cache.clear();
    return NM_OK;
}

int nm_cache_size(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    return (int)g_cache.size();
}

// File format: first line "nmconv-cache 2 <variant count> <key integers per line>
// <device of the writer>", then one line per entry: the key integers (shape,
// dtypes, N:M, tile, bias / activation flags, device identity, operand-table
// signature), the variant's name, its time in ms.  Variants are stored by name so
// that a cache written by a build with a different variant table cannot select
// the wrong kernel; entries tuned on another kind of device stay in the file but
// never match a key made on this one.
int nm_cache_save(const char* path)
{
    if (!path) {
        set_error("null path");
        return NM_ERR_ARG;
    }
    FILE* f = fopen(path, "w");
    if (!f) {
        set_error("cannot open %s for writing", path);
        return NM_ERR_IO;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    int dev = 0;
    const DeviceId* id = hipGetDevice(&dev) == hipSuccess ? device_id(dev) : nullptr;
    fprintf(f, "nmconv-cache 2 %d %d %s\n", variant_count(), kKeyInts, id ? id->name : "unknown");
    for (const auto& kv : g_cache) {
        for (int i = 0; i < kKeyInts; ++i) fprintf(f, "%d ", kv.first.v[i]);
        fprintf(f, "%s %.6f\n", variant_desc(kv.second.variant).name, kv.second.ms);
    }
    const bool ok = fclose(f) == 0;
    if (!ok) {
        set_error("write to %s failed", path);
        return NM_ERR_IO;
    }
    return NM_OK;
}

int nm_cache_load(const char* path)
{
    if (!path) {
        set_error("null path");
        return NM_ERR_ARG;
    }
    FILE* f = fopen(path, "r");
    if (!f) {
        set_error("cannot open %s", path);
        return NM_ERR_IO;
    }
    int ver = 0, cnt = 0, nkey = 0;
    char devname[128];
    if (fscanf(f, "nmconv-cache %d %d %d %127s", &ver, &cnt, &nkey, devname) != 4 || ver != 2 ||
        nkey != kKeyInts) {
        fclose(f);
        set_error("%s is not an nmconv cache file of this format", path);
        return NM_ERR_IO;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    while (true) {
        ShapeKey k;
        bool ok = true;
        for (int i = 0; i < kKeyInts && ok; ++i) ok = fscanf(f, "%d", &k.v[i]) == 1;
        char name[128];
        float ms = 0.f;
        if (!ok || fscanf(f, "%127s %f", name, &ms) != 2) break;
        for (int v = 0; v < variant_count(); ++v)
            if (strcmp(name, variant_desc(v).name) == 0) {
                g_cache[k] = CacheVal{v, ms};
                break;
            }
    }
    fclose(f);
    return NM_OK;
}

}  // extern "C"
