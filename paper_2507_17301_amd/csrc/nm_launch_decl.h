// Declaration of the per-variant launchers (defined by explicit instantiation
// in nm_conv_inst.hip, referenced by the registry).
#pragma once
#include "nm_internal.h"

namespace nm {
struct bf16_t { unsigned short v; };

template <int NBLK, int WP, int NJ, int CK, int SPC, int MODE, typename TIN, typename TOUT>
int launch_t(const ConvParams& p, hipStream_t s);
template <int NBLK, int WP, int NJ, int CK, int SPC, int SHARE>
int launch16_t(const ConvParams& p, hipStream_t s);
template <int NBLK, int WP, int NJ, int CK, bool SPARSE, bool SPEC, bool AREG = false, bool F8 = false>
int launch_sp16_t(const ConvParams& p, hipStream_t s);
template <int NBLK, int WP, int NJ, int KS>
int launch_run16_t(const ConvParams& p, hipStream_t s);
template <int NBLK, int WP, int NJ>
int launch_f8_t(const ConvParams& p, hipStream_t s);
}  // namespace nm
