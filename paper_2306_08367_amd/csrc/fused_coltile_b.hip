// Instantiations of the column-tiled join stage for bf16 models, tables and outputs (eight columns per
// lane, fp32 arithmetic), as a linear operator or with a second layer of up to sixteen outputs (more than four
// outputs: at most four fact columns).
#include "fused_coltile.h"

namespace lq {

// Element types, widths and alignment are checked by the caller (try_fused_coltile).
int try_fused_coltile_bf16(const PredictArgs& a, hipStream_t s) {
  return ct_pick_k<bf16_t, 16>(a, s);
}

}  // namespace lq
