// Instantiations of the column-tiled join stage for fp32 stars with 1 to 4 dimension tables and the
// dispatcher of the whole family (first-layer widths above 256 fp32 / 512 bf16 columns).
#include "fused_coltile.h"

namespace lq {

int try_fused_coltile_bf16(const PredictArgs& a, hipStream_t s);            // fused_coltile_b.hip
int try_fused_coltile_f32_many_dims(const PredictArgs& a, hipStream_t s);   // fused_coltile_c.hip

// Returns -1 when the shape is not one this kernel family covers.
int try_fused_coltile(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype == LQ_BF16) {
    if (a.wout[0] <= 512 || !ct_shape_ok(a, 8)) return -1;
    return try_fused_coltile_bf16(a, s);
  }
  if (a.x_dtype != LQ_F32 || a.wout[0] <= 256 || !ct_shape_ok(a, 4)) return -1;
  if (a.K > 4) return try_fused_coltile_f32_many_dims(a, s);
  return ct_pick_k<float, 16>(a, s);
}

}  // namespace lq
