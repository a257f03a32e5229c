// One (filter taps, channel count) family of the wide LDS-resident kernel; compiled once per family
// with -DRMSMP_WIDE_TAPS=.. -DRMSMP_WIDE_CPT=.. so that the families build in parallel.
#include "patch_wide.h"

#define RMSMP_WIDE_CAT2(a, b, c) launch_wide_##a##_##b
#define RMSMP_WIDE_CAT(a, b) RMSMP_WIDE_CAT2(a, b, 0)

namespace rmsmp {

int RMSMP_WIDE_CAT(RMSMP_WIDE_TAPS, RMSMP_WIDE_CPT)(const WidePlan& p, hipStream_t s) {
  return launch_wide_tc<RMSMP_WIDE_TAPS, RMSMP_WIDE_CPT>(p, s);
}

}  // namespace rmsmp
