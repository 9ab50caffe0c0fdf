// Instantiations of the row-batch join stage for fp32 with 32 and 64 lanes per fact row (hidden widths
// 68 to 256).
#include "fused_rowbatch_wide.h"

namespace lq {

// Shape checks are done by the caller (try_rowbatch_wide).
int try_rowbatch_wide_f32_32_64_lanes(const PredictArgs& a, hipStream_t s) {
  return a.wout[0] <= 128 ? pick_k<float, 32, 16>(a, s) : pick_k<float, 64, 16>(a, s);
}

}  // namespace lq
