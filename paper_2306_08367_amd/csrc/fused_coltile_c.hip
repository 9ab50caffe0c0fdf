// Instantiations of the column-tiled join stage for fp32 stars with 5 to 8 dimension tables.
#include "fused_coltile.h"

namespace lq {

// Element types, widths and alignment are checked by the caller (try_fused_coltile).
int try_fused_coltile_f32_many_dims(const PredictArgs& a, hipStream_t s) {
  switch (a.K) {
    case 5: return ct_pick_many_dims<5>(a, s);
    case 6: return ct_pick_many_dims<6>(a, s);
    case 7: return ct_pick_many_dims<7>(a, s);
    case 8: return ct_pick_many_dims<8>(a, s);
    default: return -1;
  }
}

}  // namespace lq
