// Instantiations of the specialised group-by scans for calls in which a grouping attribute has more than 255
// values (its code table has 16-bit entries): accumulators in LDS, in memory through atomics, in memory through buckets.
#include "groupby_fast.h"

namespace lq {

// Each returns -1 when there is no instantiation for this mix of dimensions.
int launch_fast_wide(const FastArgs& a, const FastLaunch& L, int mode) {
  if (mode == 0) return launch_fast<0, true>(a, L);
  if (mode == 1) return launch_fast<1, true>(a, L);
  return launch_fast<2, true>(a, L);
}

}  // namespace lq
