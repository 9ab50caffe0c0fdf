// Instantiations of the specialised group-by scan with the accumulators in memory (more than 8,192 of them:
// the multi-column group-by of Section 2.4.2), through device-wide atomics or through buckets.
#include "groupby_fast.h"

namespace lq {

// Each returns -1 when there is no instantiation for this mix of dimensions.
int launch_fast_many(const FastArgs& a, const FastLaunch& L) { return launch_fast<1>(a, L); }
int launch_fast_bucket(const FastArgs& a, const FastLaunch& L) { return launch_fast<2>(a, L); }

}  // namespace lq
