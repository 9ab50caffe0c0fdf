// Instantiations of the row-batch join stage for bf16 models, tables and outputs (hidden widths 64 to
// 512, eight columns per lane, fp32 arithmetic), as a linear operator or with a second layer of up to
// four outputs; wider second layers go to the matrix-core kernel.
#include "fused_rowbatch_wide.h"

namespace lq {

// n and the layer count are checked by the caller (try_rowbatch_wide).
int try_rowbatch_wide_bf16(const PredictArgs& a, hipStream_t s) {
  if (a.K == 4 && a.c_f > 4) return -1;      // (would not fit the register file without spilling)
  for (int k = 0; k < a.K; ++k) {
    if (!aligned(a.P[k], 16) || a.ldp[k] % 8) return -1;
    if (a.prows[k] * a.ldp[k] * 2 > 0xffffffffLL) return -1;     // the kernels keep byte offsets into a table in 32 bits
  }
  // (any hidden width: the last 16-byte piece of a row may end in the padding of the row stride, which is a multiple
  // of eight values; a linear model's Y may have any alignment)
  const int l1 = a.wout[0];
  if (l1 > 512 || l1 < 16) return -1;
  if (l1 <= 64) return pick_k<bf16_t, 8, 4>(a, s);      // lanes beyond l_1 / 8 idle
  if (l1 <= 128) return pick_k<bf16_t, 16, 4>(a, s);
  if (l1 <= 256) return pick_k<bf16_t, 32, 4>(a, s);
  return pick_k<bf16_t, 64, 4>(a, s);
}

}  // namespace lq
