// The two-layer launch of the wide LDS-resident kernel (a 3x3 layer and a 1x1 layer on the same
// input) for one channel count; compiled once per count with -DRMSMP_WIDE_CPT=.. so that the
// counts build in parallel.
#include "patch_wide.h"

#define RMSMP_PAIR_CAT2(a) launch_wide_pair_##a
#define RMSMP_PAIR_CAT(a) RMSMP_PAIR_CAT2(a)

namespace rmsmp {

int RMSMP_PAIR_CAT(RMSMP_WIDE_CPT)(const WidePlan& pa, const WidePlan& pb, hipStream_t s) {
  return launch_wide_pair_t<RMSMP_WIDE_CPT>(pa, pb, s);
}

}  // namespace rmsmp
