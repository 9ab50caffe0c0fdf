// Instantiations of the row-batch join stage for 32 and 64 lanes per fact row (hidden widths 128 and 256).
#include "fused_rowbatch_wide.h"

namespace lq {

// Shape checks are done by the caller (try_rowbatch_wide).
int try_rowbatch_wide_32_64_lanes(const PredictArgs& a, hipStream_t s) {
  return a.wout[0] == 128 ? pick_k<32, true>(a, s) : pick_k<64, true>(a, s);
}

}  // namespace lq
