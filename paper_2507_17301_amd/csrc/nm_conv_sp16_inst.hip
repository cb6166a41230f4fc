// Explicit instantiations of the gather-free bf16 kernel.  Compiled once per
// shape (-DNM_INST_NBLK=.. -DNM_INST_WP=.. -DNM_INST_NJ=..); with -DNM_INST_SPW the
// form with producer wavefronts, with -DNM_INST_SPR that form with register operands, with
// -DNM_INST_F8S the three forms for E4M3 tensors.
#include "nm_conv_sp16_kernel.h"
#include "nm_variants.h"

namespace nm {
#if defined(NM_INST_F8S)
#define NM_INSTSP(NB, WP, NJ, CK)                                                                          \
    template int launch_sp16_t<NB, WP, NJ, CK, false, false, false, true>(const ConvParams&, hipStream_t); \
    template int launch_sp16_t<NB, WP, NJ, CK, false, true, false, true>(const ConvParams&, hipStream_t);  \
    template int launch_sp16_t<NB, WP, NJ, CK, false, true, true, true>(const ConvParams&, hipStream_t);
NMF8S_CHUNKS(NM_INSTSP, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
#elif defined(NM_INST_SPR)
#define NM_INSTSP(NB, WP, NJ, CK, SP) \
    template int launch_sp16_t<NB, WP, NJ, CK, (SP) != 0, true, true>(const ConvParams&, hipStream_t);
NMSPR_CHUNKS(NM_INSTSP, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
#elif defined(NM_INST_SPW)
#define NM_INSTSP(NB, WP, NJ, CK, SP) \
    template int launch_sp16_t<NB, WP, NJ, CK, (SP) != 0, true>(const ConvParams&, hipStream_t);
NMSPW_CHUNKS(NM_INSTSP, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
#else
#define NM_INSTSP(NB, WP, NJ, CK, SP) \
    template int launch_sp16_t<NB, WP, NJ, CK, (SP) != 0, false>(const ConvParams&, hipStream_t);
NMSP_CHUNKS(NM_INSTSP, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
#endif
}  // namespace nm
