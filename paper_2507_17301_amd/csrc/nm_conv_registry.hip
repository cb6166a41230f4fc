// Table of kernel variants: description + launcher per dtype pair.
#include <deque>
#include <string>

#include "nm_launch_decl.h"
#include "nm_variants.h"

namespace nm {
namespace {
typedef int (*LaunchFn)(const ConvParams&, hipStream_t);
struct Entry {
    VariantDesc d;
    LaunchFn ff;   // fp32 in, fp32 out (fp32 MFMA kernel only)
    LaunchFn bb;   // bf16 in, bf16 out
};

#define NM_ENTRY(NB, WP, NJ, CK, SPC, VEC)                                                     \
    {{"NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK "_SPC" #SPC "_V" #VEC, 16 * NB * WP, NB, WP, NJ, CK, SPC, VEC, 0, 1, 1, 0}, \
     &launch_t<NB, WP, NJ, CK, SPC, (VEC) != 0 ? 1 : 0, float, float>,                                 \
     &launch_t<NB, WP, NJ, CK, SPC, (VEC) != 0 ? 1 : 0, bf16_t, bf16_t>},
#define NM_SHAPE_ENTRIES(NB, WP, NJ) NM_VEC_CHUNKS(NM_ENTRY, NB, WP, NJ)

#define NM_ENTRY16(NB, WP, NJ, SH, CK, SPC)                                                     \
    {{"B16_NB" #NB "_WP" #WP "_NJ" #NJ "_SH" #SH "_CK" #CK "_SPC" #SPC, 16 * NB * WP, NB, WP, NJ, CK, SPC, 1, 1, SH, 1, 0}, \
     nullptr, &launch16_t<NB, WP, NJ, CK, SPC, SH>},
#define NM_SHAPE_ENTRIES16(NB, WP, NJ, SH) NM16_CHUNKS(NM_ENTRY16, NB, WP, NJ, SH)

// kind 2: sparse matrix instruction, kind 3: dense instruction on zero-filled weights
#define NM_ENTRYSP(NB, WP, NJ, CK, SP)                                                          \
    {{"SP" #SP "_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK, 16 * NB * WP, NB, WP, NJ, CK, CK / 64, 1, (SP) ? 2 : 3, 1, 1, 0}, \
     nullptr, &launch_sp16_t<NB, WP, NJ, CK, (SP) != 0, false>},
#define NM_SHAPE_ENTRIESSP(NB, WP, NJ) NMSP_CHUNKS(NM_ENTRYSP, NB, WP, NJ)
// the same with producer wavefronts (same operand tables, same LDS footprint)
#define NM_ENTRYSPW(NB, WP, NJ, CK, SP)                                                         \
    {{"SPW" #SP "_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK, 16 * NB * WP, NB, WP, NJ, CK, CK / 64, 1, (SP) ? 2 : 3, 1, 1, 0, 1}, \
     nullptr, &launch_sp16_t<NB, WP, NJ, CK, (SP) != 0, true>},
#define NM_SHAPE_ENTRIESSPW(NB, WP, NJ) NMSPW_CHUNKS(NM_ENTRYSPW, NB, WP, NJ)

// producer wavefronts and register operands
#define NM_ENTRYSPR(NB, WP, NJ, CK, SP)                                                         \
    {{"SPR" #SP "_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK, 16 * NB * WP, NB, WP, NJ, CK, CK / 64, 1, (SP) ? 2 : 3, 1, 1, 1, 1}, \
     nullptr, &launch_sp16_t<NB, WP, NJ, CK, (SP) != 0, true, true>},
#define NM_SHAPE_ENTRIESSPR(NB, WP, NJ) NMSPR_CHUNKS(NM_ENTRYSPR, NB, WP, NJ)

// kind 4: contiguous kernel-row runs
#define NM_ENTRYRUN(NB, WP, NJ, KS)                                                             \
    {{"RUN_NB" #NB "_WP" #WP "_NJ" #NJ "_KS" #KS, 16 * NB * WP, NB, WP, NJ, 64 * KS, KS, 1, 4, 1, 1, 0}, \
     nullptr, &launch_run16_t<NB, WP, NJ, KS>},
#define NM_SHAPE_ENTRIESRUN(NB, WP, NJ) NMRUN_CHUNKS(NM_ENTRYRUN, NB, WP, NJ)

// kind 5: fp32 MFMA kernel, per-(tile, chunk) number of k-steps (fp32 tensors only)
#define NM_ENTRYVAR(NB, WP, NJ, CK, SPC)                                                        \
    {{"VAR_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK "_SPC" #SPC, 16 * NB * WP, NB, WP, NJ, CK, SPC, 1, 5, 1, 1, 0}, \
     &launch_t<NB, WP, NJ, CK, SPC, 2, float, float>, nullptr},
#define NM_SHAPE_ENTRIESVAR(NB, WP, NJ) NMVAR_CHUNKS(NM_ENTRYVAR, NB, WP, NJ)

// kind 6: fp8 E4M3 in, bf16 out (the launcher sits in the bf16-output slot; x is E4M3)
#define NM_ENTRYF8(NB, WP, NJ)                                                                  \
    {{"F8_NB" #NB "_WP" #WP "_NJ" #NJ, 16 * NB * WP, NB, WP, NJ, 64, 1, 1, 6, 1, 1, 0}, nullptr, &launch_f8_t<NB, WP, NJ>},

// kind 7: fp8 E4M3 in, bf16 out through the LDS-staged kernel: plain, with producer wavefronts,
// with producer wavefronts and register-held weights
#define NM_ENTRYF8S(NB, WP, NJ, CK)                                                                       \
    {{"F8S_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK, 16 * NB * WP, NB, WP, NJ, CK, CK / 64, 1, 7, 1, 1, 0}, \
     nullptr, &launch_sp16_t<NB, WP, NJ, CK, false, false, false, true>},                                 \
    {{"F8W_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK, 16 * NB * WP, NB, WP, NJ, CK, CK / 64, 1, 7, 1, 1, 0, 1}, \
     nullptr, &launch_sp16_t<NB, WP, NJ, CK, false, true, false, true>},                                  \
    {{"F8R_NB" #NB "_WP" #WP "_NJ" #NJ "_CK" #CK, 16 * NB * WP, NB, WP, NJ, CK, CK / 64, 1, 7, 1, 1, 1, 1}, \
     nullptr, &launch_sp16_t<NB, WP, NJ, CK, false, true, true, true>},
#define NM_SHAPE_ENTRIESF8S(NB, WP, NJ) NMF8S_CHUNKS(NM_ENTRYF8S, NB, WP, NJ)

const Entry kEntries[] = {NM_SHAPES(NM_SHAPE_ENTRIES) NM_SCALAR_VARIANTS(NM_ENTRY)
                          NM16_SHAPES(NM_SHAPE_ENTRIES16) NMSP_SHAPES(NM_SHAPE_ENTRIESSP) NMSPW_SHAPES(NM_SHAPE_ENTRIESSPW) NMSPR_SHAPES(NM_SHAPE_ENTRIESSPR)
                          NMRUN_SHAPES(NM_SHAPE_ENTRIESRUN) NMVAR_SHAPES(NM_SHAPE_ENTRIESVAR)
                          NMF8_SHAPES(NM_ENTRYF8) NMF8S_SHAPES(NM_SHAPE_ENTRIESF8S)};
constexpr int kCount = (int)(sizeof(kEntries) / sizeof(kEntries[0]));

// The fp32 MFMA kernel also runs with its K axis split over several workgroups per output
// tile (for layers with too few output tiles to fill the chip).  Those forms are variants of
// their own -- ids kCount and up, the base variant's name with "_S<splits>" appended -- so that
// the tuner, the cache and the test hook treat them like any other.
constexpr int kSplits[] = {2, 4, 8, 16};
struct Table {
    std::vector<VariantDesc> desc;
    std::vector<int> base;
    std::deque<std::string> names;
};
Table build_table()
{
    Table t;
    for (int i = 0; i < kCount; ++i) {
        t.desc.push_back(kEntries[i].d);
        t.base.push_back(i);
    }
    for (int s : kSplits)
        for (int i = 0; i < kCount; ++i) {
            if (kEntries[i].d.kind != 0 && kEntries[i].d.kind != 5) continue;
            VariantDesc d = kEntries[i].d;
            t.names.push_back(std::string(d.name) + "_S" + std::to_string(s));
            d.name = t.names.back().c_str();
            d.ksplit = s;
            t.desc.push_back(d);
            t.base.push_back(i);
        }
    return t;
}
const Table& table()
{
    static const Table t = build_table();
    return t;
}
}  // namespace

int variant_count() { return (int)table().desc.size(); }
const VariantDesc& variant_desc(int v) { return table().desc[v]; }

int launch_conv(int v, nm_dtype_t xdt, nm_dtype_t ydt, const ConvParams& p, hipStream_t s)
{
    if (v < 0 || v >= variant_count()) {
        set_error("variant %d out of range", v);
        return NM_ERR_UNSUPPORTED;
    }
    const Entry& e = kEntries[table().base[v]];
    const bool f8 = e.d.kind == 6 || e.d.kind == 7;
    if (xdt == NM_F32 && ydt == NM_F32 && e.ff && !f8) return e.ff(p, s);
    if (xdt == NM_BF16 && ydt == NM_BF16 && e.bb && !f8) return e.bb(p, s);
    if (xdt == NM_F8E4M3 && ydt == NM_BF16 && e.bb && f8) return e.bb(p, s);
    set_error("unsupported dtype pair: fp32 -> fp32, bf16 -> bf16 or E4M3 -> bf16");
    return NM_ERR_UNSUPPORTED;
}
}  // namespace nm
