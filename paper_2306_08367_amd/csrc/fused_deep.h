// Join-computation stage (last line of Eq. 1) followed by a deeper or wider fp32 MLP (a second
// layer of 5..128 outputs, or three or more layers with later hidden widths up to 128), with every layer after the gather on the matrix
// cores and all activations in registers.
//
// A wavefront owns 16 fact rows per step.  In the matrix layers lane l works for row l % 16 and, of
// every 16 hidden units, for the four units 4 (l / 16) .. + 3.  That is the operand layout of the
// 16x16x4 fp32 matrix instruction when the product is taken transposed, H_(j+1)^T = W_j^T H_j^T:
// the activations are the B operand (k = l / 16, column = row l % 16), the weights the A operand,
// and the result (output unit 4 (l / 16) + v, row l % 16) is again in this layout, so layers chain
// with no exchange between lanes.  The fact-table term x W_f is one more product of the same form.
// The weights are staged once per workgroup in LDS, already in operand order and zero-padded to
// multiples of 16 (16x16 tiles, one 16-byte read per lane and four products).
//
// The gathers use the row-contiguous layout of the row-batch kernels (l_1 / 4 neighbouring lanes read
// one projected row as a run of 16-byte pieces: measured about twice as fast as gathering straight
// into the operand layout, which reads 64-byte pieces of 16 rows); the sum over the dimensions moves
// to the operand layout through a 16-row LDS tile private to the wavefront.
//
// Software pipeline per wavefront: while step s is on the matrix cores the gathers of step s + 1 and
// the keys and fact columns of step s + 2 are in flight.
#ifndef LQ_FUSED_DEEP_H_
#define LQ_FUSED_DEEP_H_

#include "lq_common.h"

namespace lq {

// Offsets (in floats) of the staged model inside the dynamic LDS block.
struct DeepLds {
  int wf, b1;              // [T1][KC][64] and [16 T1]
  int w[LQ_MAX_LAYERS - 1], b[LQ_MAX_LAYERS - 1];   // layer j + 1: [TOUT][TIN][64][4] and [16 TOUT]
  int wvec;                // last layer as a plain vector (used when it has one output)
  int kc;                  // ceil(c_f / 4)
  int total;
};

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int DEEP_THREADS = 256;
constexpr int DEEP_WAVES = DEEP_THREADS / 64;


// out^T += W^T h^T for TIN input tiles (tiles kt0 .. kt0 + TIN - 1 of a layer of TIN_ALL input
// tiles); w points into LDS.  The 16x16 weight tiles are taken in the order (kt, ot), IL output tiles
// at a time whose products alternate (consecutive matrix instructions then write different
// accumulators), and are requested one group ahead of the products that use them, so that the matrix
// cores wait neither for LDS nor for the previous product of the same accumulator.
template <int TIN, int TOUT, int TIN_ALL>
__device__ __forceinline__ void dense_accumulate(const v4f (&h)[TIN], const float* w, int kt0, int lane, v4f (&out)[TOUT]) {
  constexpr int IL = TOUT % 2 == 0 ? 2 : 1;
  constexpr int NG = TIN * TOUT / IL;                                   // groups of IL tiles
  const v4f* wl = reinterpret_cast<const v4f*>(w) + kt0 * 64 + lane;   // tile (ot, kt) at wl[(ot TIN_ALL + kt) 64]
  v4f wv[2][IL];
#pragma unroll
  for (int i = 0; i < IL; ++i) wv[0][i] = wl[(i * TIN_ALL + 0) * 64];
#pragma unroll
  for (int gi = 0; gi < NG; ++gi) {
    const int kt = gi / (TOUT / IL), ot0 = (gi % (TOUT / IL)) * IL;
    if (gi + 1 < NG) {
      const int kn = (gi + 1) / (TOUT / IL), on = ((gi + 1) % (TOUT / IL)) * IL;
#pragma unroll
      for (int i = 0; i < IL; ++i) wv[(gi + 1) & 1][i] = wl[((on + i) * TIN_ALL + kn) * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int i = 0; i < IL; ++i)
        out[ot0 + i] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[gi & 1][i][v], h[kt][v], out[ot0 + i], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int TOUT>
__device__ __forceinline__ void load_bias(const float* bias, int lane, v4f (&out)[TOUT]) {
#pragma unroll
  for (int ot = 0; ot < TOUT; ++ot) out[ot] = *reinterpret_cast<const v4f*>(bias + 16 * ot + 4 * (lane >> 4));
}

// out^T = W^T h^T + b for one whole layer.
template <int TIN, int TOUT>
__device__ __forceinline__ void dense_layer(const v4f (&h)[TIN], const float* w, const float* bias, int lane,
                                            v4f (&out)[TOUT]) {
  load_bias<TOUT>(bias, lane, out);
  dense_accumulate<TIN, TOUT, TIN>(h, w, 0, lane, out);
}

template <int T>
__device__ __forceinline__ void relu(v4f (&h)[T]) {
#pragma unroll
  for (int t = 0; t < T; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v) h[t][v] = __builtin_amdgcn_fmed3f(h[t][v], 0.f, __builtin_inff());   // one instruction; NaN -> 0 like fmaxf
}

// Rows of Y for the 16 rows of a step; lane holds output units 16 ot + 4 (l / 16) + v of row l % 16.
template <int T>
__device__ __forceinline__ void store_rows(const PredictArgs& a, const v4f (&y)[T], int64_t row, bool valid, int q4,
                                           int l_out, bool vec_y) {
  if (!valid) return;
  float* dst = static_cast<float*>(a.Y) + row * a.ldy;
#pragma unroll
  for (int ot = 0; ot < T; ++ot) {
    const int c = 16 * ot + 4 * q4;
    if (vec_y) {
      if (c < l_out) *reinterpret_cast<v4f*>(dst + c) = y[ot];
    } else {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (c + v < l_out) dst[c + v] = y[ot][v];
    }
  }
}

// Stages the model in LDS in operand order (THREADS threads of the workgroup call this; the caller
// synchronises afterwards).  TALL: 16-unit tiles of the first hidden layer, TH: of the later ones.
template <int THREADS, int NL>
__device__ __forceinline__ void stage_model(const PredictArgs& a, const DeepLds& L, float* lds, int tid, int TALL, int TH) {
  const int l1 = a.wout[0];
  for (int i = tid; i < TALL * L.kc * 64; i += THREADS) {
    const int ln = i & 63, tk = i >> 6, t = tk / L.kc, kc = tk - t * L.kc;
    const int q = 4 * kc + (ln >> 4), c = 16 * t + (ln & 15);
    lds[L.wf + i] = (q < a.c_f && c < l1) ? static_cast<const float*>(a.W[0])[static_cast<int64_t>(q) * a.ldw[0] + c] : 0.f;
  }
  for (int i = tid; i < 16 * TALL; i += THREADS)
    lds[L.b1 + i] = (i < l1 && a.bias[0]) ? static_cast<const float*>(a.bias[0])[i] : 0.f;
  const int nl = NL == 4 ? a.n_layers : NL;
  for (int layer = 1; layer < nl; ++layer) {
    const int tin = layer == 1 ? TALL : TH;
    const int tout = (layer == nl - 1 && NL > 2 && a.wout[nl - 1] <= 16) ? 1 : TH;   // a narrow output layer is one tile
    const int win = a.win[layer], wout = a.wout[layer];
    const float* W = static_cast<const float*>(a.W[layer]);
    const int64_t ldw = a.ldw[layer];
    for (int i = tid; i < tout * tin * 256; i += THREADS) {
      const int v = i & 3, ln = (i >> 2) & 63, tile = i >> 8, ot = tile / tin, kt = tile - ot * tin;
      const int f = 16 * kt + 4 * (ln >> 4) + v, c = 16 * ot + (ln & 15);
      lds[L.w[layer - 1] + i] = (f < win && c < wout) ? W[static_cast<int64_t>(f) * ldw + c] : 0.f;
    }
    for (int i = tid; i < 16 * tout; i += THREADS)
      lds[L.b[layer - 1] + i] = (i < wout && a.bias[layer]) ? static_cast<const float*>(a.bias[layer])[i] : 0.f;
  }
  if (NL > 2) {
    const int win = a.win[nl - 1];
    for (int i = tid; i < 16 * TH; i += THREADS)
      lds[L.wvec + i] = i < win ? static_cast<const float*>(a.W[nl - 1])[static_cast<int64_t>(i) * a.ldw[nl - 1]] : 0.f;
  }
}

// Everything after the second layer for the 16 rows of a step (lane l: row `row`, units 4 (l / 16) .. + 3
// of every 16), and the store of Y.  h2 holds the second layer's sums with its bias, before the ReLU.
template <int TH, int NL>
__device__ __forceinline__ void later_layers(const PredictArgs& a, const DeepLds& L, const float* lds, v4f (&h2)[TH],
                                             int64_t row, int lane, int nl, int l_out, int vec_y) {
  const int q4 = lane >> 4;
  const bool valid = row < a.n;
  if constexpr (NL == 2) {
    store_rows<TH>(a, h2, row, valid, q4, l_out, vec_y != 0);
  } else {
    relu<TH>(h2);
    if constexpr (NL == 4) {
      for (int layer = 2; layer < nl - 1; ++layer) {     // the hidden layers between the second and the last
        v4f h3[TH];
        dense_layer<TH, TH>(h2, lds + L.w[layer - 1], lds + L.b[layer - 1], lane, h3);
        relu<TH>(h3);
#pragma unroll
        for (int t = 0; t < TH; ++t) h2[t] = h3[t];
      }
    }
    if (l_out == 1) {
      // one output: a dot product per row, summed over the four lanes of the row
      float y = 0.f;
#pragma unroll
      for (int t = 0; t < TH; ++t) {
        const v4f w = *reinterpret_cast<const v4f*>(lds + L.wvec + 16 * t + 4 * q4);
#pragma unroll
        for (int v = 0; v < 4; ++v) y = fmaf(h2[t][v], w[v], y);
      }
      y += __shfl_xor(y, 16);
      y += __shfl_xor(y, 32);
      y += lds[L.b[nl - 2]];
      if (valid && q4 == 0) static_cast<float*>(a.Y)[row * a.ldy] = y;
    } else if (l_out <= 16) {
      v4f y[1];
      dense_layer<TH, 1>(h2, lds + L.w[nl - 2], lds + L.b[nl - 2], lane, y);
      store_rows<1>(a, y, row, valid, q4, l_out, vec_y != 0);
    } else {
      v4f y[TH];
      dense_layer<TH, TH>(h2, lds + L.w[nl - 2], lds + L.b[nl - 2], lane, y);
      store_rows<TH>(a, y, row, valid, q4, l_out, vec_y != 0);
    }
  }
}

// Asking for two wavefronts per SIMD caps the kernel at 256 registers, all of them ordinary ones: the
// accumulators of the matrix instructions then need no copies before the vector instructions that
// follow them (bias, ReLU, the sum over the row).  The instantiations with the most gathers in flight or
// the widest later layers need more and keep the default.
template <int T1, int TH, int KMAX> struct DeepRegs {
  static constexpr int MIN_WAVES = (T1 * KMAX <= 24 && TH <= 4) ? 2 : 1;
};

// T1, PARTS: l_1 <= 16 T1 PARTS (a multiple of 4); the hidden layer is gathered and fed to the second
// layer in PARTS column parts of 16 T1 units, so that at most 4 T1 registers per table are in flight.  TH: later hidden layers (and, with two layers, the output) are at most 16 TH wide.
// NL: number of layers, 2, 3, or 4 for "four or more" (the count is then read at run time).
// KMAX: number of dimension tables whose gathers are all in flight at once (1..4).  EXTRA: there are
// more than KMAX = 4 tables; the further ones are gathered inside the step, after the prefetch of the
// next step has been requested.
template <int T1, int PARTS, int TH, int NL, int KMAX, bool EXTRA>
__global__ __launch_bounds__(DEEP_THREADS, (DeepRegs<T1, TH, KMAX>::MIN_WAVES)) void fused_deep_kernel(PredictArgs a, DeepLds L, int vec_y) {
  constexpr int TALL = T1 * PARTS;                // 16-unit tiles of the whole hidden layer
  extern __shared__ __align__(16) float lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, q4 = lane >> 4;
  const int l1 = a.wout[0];

  stage_model<DEEP_THREADS, NL>(a, L, lds, tid, TALL, TH);
  const int nl = NL == 4 ? a.n_layers : NL;
  __syncthreads();

  const int64_t n_steps = (a.n + 15) / 16;
  int64_t step = static_cast<int64_t>(blockIdx.x) * DEEP_WAVES + wave;
  if (step >= n_steps) return;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * DEEP_WAVES;
  const int l_out = a.wout[nl - 1];
  const float* X = static_cast<const float*>(a.X);

  // Software pipeline over the steps of this wavefront: while step s is on the matrix cores, the
  // gathers of step s + 1 and the keys / fact columns of step s + 2 are in flight.
  //
  // Gathers use a row-contiguous layout (LPR = l_1 / 4 neighbouring lanes read one projected row
  // as a run of 16-byte pieces, 64 / LPR rows per instruction); the sum over the dimensions then
  // moves to the operand layout through a 16-row tile in LDS that belongs to this wavefront.
  constexpr int LPR = 4 * T1, RPI = 64 / LPR, LD = 16 * T1 + 4;   // LD staggers rows over the LDS banks
  const int gsub = lane / LPR, gc = lane % LPR;
  float* tile = lds + L.total + wave * 16 * LD;
  for (int i = lane; i < 16 * LD; i += 64) tile[i] = 0.f;
  // A piece of the summed rows goes to the tile; a lane past the end of a row leaves the tile's zero in
  // place (one column part) or writes a zero over what the previous part left there (two parts).
  // (live: the piece starts inside the row.  A hidden width that is not a multiple of four: the row's last piece
  // ends in the padding of the row stride, whose contents are not ours; those elements count as zero.)
  auto store_piece = [&](float* dst, v4f sum, bool live, int col) {
    if (l1 % 4 != 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) sum[v] = col + v < l1 ? sum[v] : 0.f;
    }
    if constexpr (PARTS > 1) {
      *reinterpret_cast<v4f*>(dst) = live ? sum : v4f{0.f, 0.f, 0.f, 0.f};
    } else {
      if (live) *reinterpret_cast<v4f*>(dst) = sum;
    }
  };
  auto clamp_row = [&](int64_t st) { return min<int64_t>(min<int64_t>(st, n_steps - 1) * 16 + r16, a.n - 1); };
  // Keys are kept as the offset of their row in 16-byte pieces, key * (row stride / 4): one 32-bit
  // product per key where it is loaded, instead of a 64-bit one per gathered piece.
  uint32_t ld16[KMAX];
#pragma unroll
  for (int k = 0; k < KMAX; ++k) ld16[k] = static_cast<uint32_t>(a.ldp[k] >> 2);
  uint32_t key0[KMAX];     // rows of this step (only live when later parts still need them: PARTS > 1)
  uint32_t key1[KMAX];     // rows of the step after this one (lane l: row l % 16)
  float xv[4], x1[4];      // fact columns of this step and of the next
  v4f g[KMAX][T1];         // gathered pieces in flight: g[k][u] = row u RPI + gsub, piece gc of one part
  auto gather = [&](const uint32_t (&key)[KMAX], int part) {
    const int col = part * 16 * T1 + 4 * gc;
    // Widths below 16 T1 PARTS: the lanes past the end of a row re-read its first piece (no branch
    // around the loads, which would serialise the broadcast-then-load pairs); what they fetch never
    // reaches the tile, whose columns past the end of a row hold zeros.
    const uint32_t piece = col < l1 ? col >> 2 : 0;
    uint32_t at[KMAX][T1];
#pragma unroll
    for (int k = 0; k < KMAX; ++k)
#pragma unroll
      for (int u = 0; u < T1; ++u) at[k][u] = static_cast<uint32_t>(__shfl(static_cast<int>(key[k]), u * RPI + gsub)) + piece;
#pragma unroll
    for (int k = 0; k < KMAX; ++k)
#pragma unroll
      for (int u = 0; u < T1; ++u)
        g[k][u] = *reinterpret_cast<const v4f*>(static_cast<const char*>(a.P[k]) + (static_cast<uint64_t>(at[k][u]) << 4));
  };
  {
    const int64_t row = clamp_row(step), row1 = clamp_row(step + stride);
    uint32_t key[KMAX];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) key[k] = static_cast<uint32_t>(a.fk[k][row]) * ld16[k];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) key1[k] = static_cast<uint32_t>(a.fk[k][row1]) * ld16[k];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
      const int q = 4 * kc + q4;
      xv[kc] = q < a.c_f ? X[row * a.ldx + q] : 0.f;
      x1[kc] = q < a.c_f ? X[row1 * a.ldx + q] : 0.f;
    }
    gather(key, 0);
#pragma unroll
    for (int k = 0; k < KMAX; ++k) key0[k] = key[k];
  }

  for (;;) {
    // The staged model is read from LDS where it is used: without this the loads are hoisted out of
    // the loop and the weights take every register there is.
    asm volatile("" ::: "memory");
    const bool more = step + stride < n_steps;
    // keys and fact columns two steps ahead (rows past the end are clamped: harmless reloads)
    const int64_t row2 = clamp_row(step + 2 * stride);
    uint32_t key2[KMAX];
    float x2[4];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) key2[k] = static_cast<uint32_t>(a.fk[k][row2]) * ld16[k];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
      const int q = 4 * kc + q4;
      x2[kc] = q < a.c_f ? X[row2 * a.ldx + q] : 0.f;
    }

    // ---- layers 1 and 2, one column part of the hidden layer at a time
    constexpr int T2 = TH;                 // output tiles of the second layer (NL == 2: of the model)
    v4f h2[T2];
#pragma unroll
    for (int part = 0; part < PARTS; ++part) {
      // sum of the gathered rows -> LDS tile; then the next gathers are requested (the next part of
      // this step, or the first part of the next step) and are in flight during the matrix work
      if constexpr (!EXTRA) {
#pragma unroll
        for (int u = 0; u < T1; ++u) {
          v4f sum = g[0][u];
#pragma unroll
          for (int k = 1; k < KMAX; ++k)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[v] += g[k][u][v];
          store_piece(tile + (u * RPI + gsub) * LD + 4 * gc, sum, part * 16 * T1 + 4 * gc < l1, part * 16 * T1 + 4 * gc);
        }
        if (part + 1 < PARTS) gather(key0, part + 1); else gather(key1, 0);
      } else {
        v4f sum[T1];
#pragma unroll
        for (int u = 0; u < T1; ++u) {
          sum[u] = g[0][u];
#pragma unroll
          for (int k = 1; k < KMAX; ++k)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[u][v] += g[k][u][v];
        }
        if (part + 1 < PARTS) gather(key0, part + 1); else gather(key1, 0);
        const int col = part * 16 * T1 + 4 * gc;
        const int64_t myrow = clamp_row(step);
        for (int k = KMAX; k < a.K; ++k) {                   // tables 5..8: key, then gather, inside the step
          const uint32_t kk = static_cast<uint32_t>(a.fk[k][myrow]) * static_cast<uint32_t>(a.ldp[k] >> 2);
          v4f e[T1];
#pragma unroll
          for (int u = 0; u < T1; ++u) {
            const uint32_t at = static_cast<uint32_t>(__shfl(static_cast<int>(kk), u * RPI + gsub)) + (col < l1 ? col >> 2 : 0);
            e[u] = *reinterpret_cast<const v4f*>(static_cast<const char*>(a.P[k]) + (static_cast<uint64_t>(at) << 4));
          }
#pragma unroll
          for (int u = 0; u < T1; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[u][v] += e[u][v];
        }
#pragma unroll
        for (int u = 0; u < T1; ++u) store_piece(tile + (u * RPI + gsub) * LD + 4 * gc, sum[u], col < l1, col);
      }

      // z = x W_f + b_1 (matrix cores) + the gathered sum (back from the tile), ReLU
      v4f h1[T1];
#pragma unroll
      for (int t = 0; t < T1; ++t) h1[t] = *reinterpret_cast<const v4f*>(lds + L.b1 + 16 * (part * T1 + t) + 4 * q4);
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
        if (kc < L.kc) {
          float wfv[T1];
#pragma unroll
          for (int t = 0; t < T1; ++t) wfv[t] = lds[L.wf + ((part * T1 + t) * L.kc + kc) * 64 + lane];
#pragma unroll
          for (int t = 0; t < T1; ++t) h1[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wfv[t], xv[kc], h1[t], 0, 0, 0);
        }
      for (int kc = 4; kc < L.kc; ++kc) {                 // fact columns 17..64: read where they are used
        const int q = 4 * kc + q4;
        const float xq = q < a.c_f ? X[clamp_row(step) * a.ldx + q] : 0.f;
        float wfv[T1];
#pragma unroll
        for (int t = 0; t < T1; ++t) wfv[t] = lds[L.wf + ((part * T1 + t) * L.kc + kc) * 64 + lane];
#pragma unroll
        for (int t = 0; t < T1; ++t) h1[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wfv[t], xq, h1[t], 0, 0, 0);
      }
#pragma unroll
      for (int t = 0; t < T1; ++t) {
        const v4f z = *reinterpret_cast<const v4f*>(tile + r16 * LD + 16 * t + 4 * q4);
#pragma unroll
        for (int v = 0; v < 4; ++v) h1[t][v] = fmaxf(h1[t][v] + z[v], 0.f);
      }
      if (part == 0) load_bias<T2>(lds + L.b[0], lane, h2);
      dense_accumulate<T1, T2, TALL>(h1, lds + L.w[0], part * T1, lane, h2);
    }

    later_layers<TH, NL>(a, L, lds, h2, step * 16 + r16, lane, nl, l_out, vec_y);
    if (!more) break;
    step += stride;
    if constexpr (PARTS > 1) {
#pragma unroll
      for (int k = 0; k < KMAX; ++k) key0[k] = key1[k];
    }
#pragma unroll
    for (int k = 0; k < KMAX; ++k) key1[k] = key2[k];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) { xv[kc] = x1[kc]; x1[kc] = x2[kc]; }
  }
}


// Launches the instantiation for NL_ (2, 3, or 4 = four or more layers) on at most `blocks` workgroups: one
// resident set of them (every wavefront runs its software pipeline once, none starts late).
template <int NL_>
int launch_deep_nl(const PredictArgs& a, const DeepLds& L, size_t lds, int64_t blocks, int vec_y, int T1, int PARTS, int TH,
                   hipStream_t s) {
#define LQ_DEEP(T1_, PARTS_, TH_, K_, X_)                                                                   \
  do {                                                                                                      \
    const void* fn = reinterpret_cast<const void*>(&fused_deep_kernel<T1_, PARTS_, TH_, NL_, K_, X_>);      \
    if (lds > 64 * 1024)                                                                                    \
      LQ_HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
    const int64_t resident = static_cast<int64_t>(num_cus()) * resident_per_cu(fn, DEEP_THREADS, lds);     \
    hipLaunchKernelGGL((fused_deep_kernel<T1_, PARTS_, TH_, NL_, K_, X_>),                                  \
                       dim3(static_cast<unsigned>(std::min(blocks, resident))), dim3(DEEP_THREADS), lds, s, a, L, vec_y); \
  } while (0)
#define LQ_DEEP_K(T1_, PARTS_, TH_)                                                                         \
  do {                                                                                                      \
    if (a.K == 1) LQ_DEEP(T1_, PARTS_, TH_, 1, false); else if (a.K == 2) LQ_DEEP(T1_, PARTS_, TH_, 2, false); \
    else if (a.K == 3) LQ_DEEP(T1_, PARTS_, TH_, 3, false); else if (a.K == 4) LQ_DEEP(T1_, PARTS_, TH_, 4, false); \
    else LQ_DEEP(T1_, PARTS_, TH_, 4, true);                                                                \
  } while (0)
#define LQ_DEEP_T1(TH_)                                                                                     \
  do {                                                                                                      \
    if (PARTS == 2) LQ_DEEP_K(8, 2, TH_);                                                                   \
    else if (T1 == 2) LQ_DEEP_K(2, 1, TH_); else if (T1 == 4) LQ_DEEP_K(4, 1, TH_);                         \
    else LQ_DEEP_K(8, 1, TH_);                                                                              \
  } while (0)
  if (TH == 1) LQ_DEEP_T1(1); else if (TH == 2) LQ_DEEP_T1(2); else if (TH == 4) LQ_DEEP_T1(4); else if (TH == 8) LQ_DEEP_T1(8);
  else if (T1 == 2) LQ_DEEP_K(2, 1, 16); else LQ_DEEP_K(4, 1, 16);     // later layers of 129..256 units: first layers up to 64 only
#undef LQ_DEEP_T1
#undef LQ_DEEP_K
#undef LQ_DEEP
  LQ_LAUNCH_CHECK("fused_deep_kernel");
  return LQ_OK;
}

}  // namespace
}  // namespace lq
#endif  // LQ_FUSED_DEEP_H_
