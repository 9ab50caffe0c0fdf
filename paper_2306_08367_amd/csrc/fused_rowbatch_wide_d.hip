// Instantiations of the row-batch join stage for fp32 stars with 5 to 8 dimension tables.
#include "fused_rowbatch_wide.h"

namespace lq {

// Element types, n, the layer count and the alignment are checked by the caller (try_rowbatch_wide).
int try_rowbatch_wide_f32_many_dims(const PredictArgs& a, hipStream_t s) {
  const int l1 = a.wout[0];
  if (l1 <= 32) return pick_k_many<8>(a, s);
  if (l1 <= 64) return pick_k_many<16>(a, s);
  if (l1 <= 128) return pick_k_many<32>(a, s);
  return pick_k_many<64>(a, s);
}

}  // namespace lq
