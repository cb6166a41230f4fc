// Explicit instantiations of the bf16 matrix-core kernel.  Compiled once per
// shape (-DNM_INST_NBLK=.. -DNM_INST_WP=.. -DNM_INST_NJ=.. -DNM_INST_SHARE=..).
#include "nm_conv_bf16_kernel.h"
#include "nm_variants.h"

namespace nm {
#define NM_INST16(NB, WP, NJ, SH, CK, SPC) \
    template int launch16_t<NB, WP, NJ, CK, SPC, SH>(const ConvParams&, hipStream_t);
NM16_CHUNKS(NM_INST16, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ, NM_INST_SHARE)
}  // namespace nm
