// Dispatcher of the matrix-core kernel for deeper fp32 models (see fused_deep.h) and its two-layer
// instantiations; the three-layer and four-or-more-layer ones are compiled in fused_deep_b.hip and
// fused_deep_c.hip so that the three sources build in parallel.
#include "fused_deep.h"

namespace lq {

int launch_deep_3(const PredictArgs& a, const DeepLds& L, size_t lds, int64_t blocks, int vec_y, int T1, int PARTS, int TH,
                  hipStream_t s);
int launch_deep_4(const PredictArgs& a, const DeepLds& L, size_t lds, int64_t blocks, int vec_y, int T1, int PARTS, int TH,
                  hipStream_t s);

// Returns -1 when the shape is not one this kernel covers.
int try_fused_deep(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype != LQ_F32 || a.p_dtype != LQ_F32 || a.y_dtype != LQ_F32) return -1;
  const int NL = a.n_layers;
  if (NL < 2 || NL > LQ_MAX_LAYERS) return -1;
  const int l1 = a.wout[0];
  if (l1 < 1 || l1 > 256) return -1;        // (any width: a row's last 16-byte piece may end in the padding of the row stride)
  if (a.c_f > 64 || a.K < 1 || a.K > LQ_MAX_DIMS) return -1;
  for (int k = 0; k < a.K; ++k) {
    if (!aligned(a.P[k], 16) || a.ldp[k] % 4) return -1;
    if (a.prows[k] * (a.ldp[k] / 4) > 0xffffffffLL) return -1;     // the kernel counts 16-byte pieces of a table in 32 bits
  }
  // 16-unit tiles of the hidden layer, padded to a power of two; above 128 in two column parts
  const int PARTS = l1 > 128 ? 2 : 1;
  const int T1 = l1 <= 32 ? 2 : (l1 <= 64 ? 4 : 8);
  const int TALL = T1 * PARTS;
  int wide = 0;                                       // widest later layer that has to fit TH tiles
  const int l_out = a.wout[NL - 1];
  for (int j = 1; j < NL; ++j)
    if (j < NL - 1 || NL == 2 || l_out > 16) wide = std::max(wide, a.wout[j]);   // (an output layer of <= 16 is its own tile)
  // One to four outputs: the row-batch kernels are at least as fast while the fact table brings few columns of its
  // own; with more of them x W_f is better off on the matrix cores (measured per 4e6 rows on a three-table star,
  // row-batch -> this kernel: 64->1 with 12 fact columns 0.36 -> 0.28 ms, 64->4 0.55 -> 0.27, 128->4 0.90 -> 0.52,
  // 64->1 with 20 (beyond the row-batch kernels' 16) 1.10 -> 0.34; 32->1 with 8: 0.12 against 0.14, stays there).
  if (NL == 2 && l_out <= 4 && !(a.c_f > 8 || (a.c_f > 4 && l1 >= 64))) return -1;
  if (wide > 256 || (wide > 128 && l1 > 64)) return -1;     // (later layers of 129..256 units next to first layers of up to 64)
  const int TH = wide <= 16 ? 1 : (wide <= 32 ? 2 : (wide <= 64 ? 4 : (wide <= 128 ? 8 : 16)));

  DeepLds L{};
  L.kc = (a.c_f + 3) / 4;
  int off = 0;
  L.wf = off; off += TALL * L.kc * 64;
  L.b1 = off; off += 16 * TALL;
  for (int j = 1; j < NL; ++j) {
    const int tin = j == 1 ? TALL : TH;
    const int tout = (j == NL - 1 && NL > 2 && l_out <= 16) ? 1 : TH;
    L.w[j - 1] = off; off += tout * tin * 256;
    L.b[j - 1] = off; off += 16 * tout;
  }
  L.wvec = off; off += 16 * TH;
  L.total = off;
  off += DEEP_WAVES * 16 * (16 * T1 + 4);         // one 16-row tile per wavefront
  const size_t lds = static_cast<size_t>(off) * 4;
  if (lds > 150 * 1024) return -1;
  const int vec_y = (l_out % 4 == 0 && a.ldy % 4 == 0 && aligned(a.Y, 16)) ? 1 : 0;

  const int64_t n_steps = (a.n + 15) / 16;
  const int64_t blocks = (n_steps + DEEP_WAVES - 1) / DEEP_WAVES;    // the launcher caps them at one resident set
  if (blocks <= 0 || a.probe) return LQ_OK;
  if (NL == 2) return launch_deep_nl<2>(a, L, lds, blocks, vec_y, T1, PARTS, TH, s);
  if (NL == 3) return launch_deep_3(a, L, lds, blocks, vec_y, T1, PARTS, TH, s);
  return launch_deep_4(a, L, lds, blocks, vec_y, T1, PARTS, TH, s);
}

}  // namespace lq
