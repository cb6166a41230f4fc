// Explicit instantiations of the fp8 kernel.  Compiled once per shape
// (-DNM_INST_NBLK=.. -DNM_INST_WP=.. -DNM_INST_NJ=..).
#include "nm_conv_f8_kernel.h"

namespace nm {
template int launch_f8_t<NM_INST_NBLK, NM_INST_WP, NM_INST_NJ>(const ConvParams&, hipStream_t);
}  // namespace nm
