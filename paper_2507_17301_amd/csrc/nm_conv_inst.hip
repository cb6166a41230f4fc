// Explicit instantiations of the convolution kernel.  Compiled once per shape
// (-DNM_INST_NBLK=.. -DNM_INST_WP=.. -DNM_INST_NJ=..), with -DNM_INST_VAR for the
// shapes of the variable-step form, and once with -DNM_INST_SCALAR for the
// element-wise staging variants.
#include "nm_conv_kernel.h"
#include "nm_variants.h"

namespace nm {
#define NM_INST(NB, WP, NJ, CK, SPC, VEC)                                                        \
    template int launch_t<NB, WP, NJ, CK, SPC, (VEC) != 0 ? 1 : 0, float, float>(const ConvParams&, hipStream_t); \
    template int launch_t<NB, WP, NJ, CK, SPC, (VEC) != 0 ? 1 : 0, bf16_t, bf16_t>(const ConvParams&, hipStream_t);

#define NM_INST_VARSTEP(NB, WP, NJ, CK, SPC) \
    template int launch_t<NB, WP, NJ, CK, SPC, 2, float, float>(const ConvParams&, hipStream_t);

#if defined(NM_INST_SCALAR)
NM_SCALAR_VARIANTS(NM_INST)
#elif defined(NM_INST_VAR)
NMVAR_CHUNKS(NM_INST_VARSTEP, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
#else
NM_VEC_CHUNKS(NM_INST, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
#endif
}  // namespace nm
