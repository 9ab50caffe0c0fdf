// Instantiations of the specialised group-by scan with the accumulators in memory (more than 8,192 of them:
// the multi-column group-by of Section 2.4.2).
#include "groupby_fast.h"

namespace lq {

// Returns -1 when there is no instantiation for this mix of dimensions.
int launch_fast_many(const FastArgs& a, const FastLaunch& L) { return launch_fast<true>(a, L); }

}  // namespace lq
