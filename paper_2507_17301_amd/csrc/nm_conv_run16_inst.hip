// Explicit instantiations of the kernel-row-run bf16 kernel.  Compiled once per
// shape (-DNM_INST_NBLK=.. -DNM_INST_WP=.. -DNM_INST_NJ=..).
#include "nm_conv_run16_kernel.h"
#include "nm_variants.h"

namespace nm {
#define NM_INSTRUN(NB, WP, NJ, KS) template int launch_run16_t<NB, WP, NJ, KS>(const ConvParams&, hipStream_t);
NMRUN_CHUNKS(NM_INSTRUN, NM_INST_NBLK, NM_INST_WP, NM_INST_NJ)
}  // namespace nm
