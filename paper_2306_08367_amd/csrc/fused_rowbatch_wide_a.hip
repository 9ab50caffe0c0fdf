// Instantiations of the row-batch join stage for fp32 with 8 and 16 lanes per fact row (hidden widths
// up to 64) and the dispatcher of the whole family.
#include "fused_rowbatch_wide.h"

namespace lq {

int try_rowbatch_wide_f32_32_64_lanes(const PredictArgs& a, hipStream_t s);   // fused_rowbatch_wide_b.hip
int try_rowbatch_wide_bf16(const PredictArgs& a, hipStream_t s);              // fused_rowbatch_wide_c.hip
int try_rowbatch_wide_f32_many_dims(const PredictArgs& a, hipStream_t s);     // fused_rowbatch_wide_d.hip

// Returns -1 when the shape is not one this kernel family covers.
int try_rowbatch_wide(const PredictArgs& a, hipStream_t s) {
  if (a.n_layers > 2 || a.n < 256) return -1;
  if (a.x_dtype == LQ_BF16 && a.p_dtype == LQ_BF16 && a.y_dtype == LQ_BF16) return try_rowbatch_wide_bf16(a, s);
  if (a.x_dtype != LQ_F32 || a.p_dtype != LQ_F32 || a.y_dtype != LQ_F32) return -1;
  for (int k = 0; k < a.K; ++k) {
    if (!aligned(a.P[k], 16) || a.ldp[k] % 4) return -1;
    if (a.prows[k] * a.ldp[k] * 4 > 0xffffffffLL) return -1;     // the kernels keep byte offsets into a table in 32 bits
  }
  // (any hidden width: the last 16-byte piece of a row may end in the padding of the row stride, which is a multiple
  // of four floats; a linear model's Y may have any alignment)
  const int l1 = a.wout[0];
  if (l1 > 256 || l1 < 12) return -1;                   // (below 12: one row per 1..3 lanes, the lane-group kernel)
  if (a.K > 4) return try_rowbatch_wide_f32_many_dims(a, s);
  if (l1 <= 32) return pick_k<float, 8, 16>(a, s);      // lanes beyond l_1 / 4 idle
  if (l1 <= 64) return pick_k<float, 16, 16>(a, s);     // (64 with 0 / 4 / 8 aligned fact columns and 1 / 2 / 4 outputs: the unrolled kernel, tried first)
  return try_rowbatch_wide_f32_32_64_lanes(a, s);
}

}  // namespace lq
