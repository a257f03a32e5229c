// One (filter taps, channel count) family of the wide LDS-resident kernel; compiled once per family
// with -DRMSMP_WIDE_TAPS=.. -DRMSMP_WIDE_CPT=.. so that the families build in parallel.
// -DRMSMP_WIDE_DEEP=1 builds the family's variant for 1x1 layers / GEMMs whose channels are staged
// in several parts of 32*CPT (a separate variant: the loop over the parts costs registers).
#include "patch_wide.h"

#ifndef RMSMP_WIDE_DEEP
#define RMSMP_WIDE_DEEP 0
#endif
#if RMSMP_WIDE_DEEP
#define RMSMP_WIDE_CAT2(a, b, c) launch_wide_deep_##b
#else
#define RMSMP_WIDE_CAT2(a, b, c) launch_wide_##a##_##b
#endif
#define RMSMP_WIDE_CAT(a, b) RMSMP_WIDE_CAT2(a, b, 0)

namespace rmsmp {

int RMSMP_WIDE_CAT(RMSMP_WIDE_TAPS, RMSMP_WIDE_CPT)(const WidePlan& p, hipStream_t s) {
  return launch_wide_tc<RMSMP_WIDE_TAPS, RMSMP_WIDE_CPT, RMSMP_WIDE_DEEP != 0>(p, s);
}

}  // namespace rmsmp
