// Instantiations of the matrix-core kernel for deeper fp32 models with three layers (fused_deep.h).
#include "fused_deep.h"

namespace lq {

int launch_deep_3(const PredictArgs& a, const DeepLds& L, size_t lds, int64_t blocks, int vec_y, int T1, int PARTS, int TH,
                  hipStream_t s) {
  return launch_deep_nl<3>(a, L, lds, blocks, vec_y, T1, PARTS, TH, s);
}

}  // namespace lq
