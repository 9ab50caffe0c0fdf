// Join-computation stage (last line of Eq. 1) followed by a deeper or wider bf16 MLP (a second
// layer of 17..256 outputs, or three or more layers with later hidden widths up to 256 and at most
// 16 outputs): hidden width a multiple of 8 up to 256, up to 64 fact-owned columns, every layer
// after the gather on the matrix cores.
//
// A wavefront handles 16 fact rows per pass.  Lane (g = lane / 16, j = lane % 16) works on row j
// and, in each 32-wide block kb of hidden units, owns units 32 kb + 8 g .. + 7: the eight bf16 values
// one lane supplies as the K-slice of the B operand of the 16x16x32 bf16 matrix instruction.  The
// gathered rows are summed in fp32 in place and rectified.  Layers are taken transposed,
// H_(j+1)^T = W_j^T H_j^T: the result of a 16-output tile (register v of lane (g, j) = output 4 g + v
// of row j, fp32) is rectified, and two such tiles side by side are again a B operand (elements 0..3
// from the even tile, 4..7 from the odd one), so layers chain in registers.  The weights are staged
// once per workgroup in LDS in that operand order, zero-padded.
// The instruction takes bf16 operands.  The wide first hidden layer is rounded to bf16 once, as in the
// one-tile bf16 kernel; every activation of the later (narrower) layers is fed as two operands, its
// bf16 rounding and the bf16 rounding of what that left over, which keeps those activations at about
// fp32 precision (their rounding errors would not average out over few units).  Accumulation is fp32.
#include "lq_common.h"

namespace lq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int DBF_THREADS = 256;

// Byte offsets of the staged model inside the dynamic LDS block.
struct DeepBfLds {
  int w[LQ_MAX_LAYERS - 1];       // layer j + 1: [TOUT][chunks of 32 inputs][64 lanes] x 16 bytes
  int b[LQ_MAX_LAYERS - 1];       // fp32 [16 TOUT]
  int wf;                         // rows of W_0 that belong to the fact columns: bf16 [c_f][32 KB], zeros past l_1
  int total;
};

__device__ __forceinline__ void unpack_add(const v4u& w, float (&acc)[8]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    acc[2 * q] += __uint_as_float(w[q] << 16);
    acc[2 * q + 1] += __uint_as_float(w[q] & 0xffff0000u);
  }
}
__device__ __forceinline__ unsigned int pack2(float lo, float hi) { return f32x2_to_bf16x2(lo, hi); }
// ReLU of two activations, each split into a bf16 head and a bf16 tail (x = head + tail up to 2^-17
// relative): feeding both to the matrix cores keeps the activations at about fp32 precision although
// the instruction takes bf16 operands (the weights are bf16 values to begin with, so exact).
struct HeadTail { unsigned int head, tail; };
__device__ __forceinline__ HeadTail split2_relu(float x0, float x1) {
  x0 = fmaxf(x0, 0.f); x1 = fmaxf(x1, 0.f);
  const unsigned int head = pack2(x0, x1);
  return {head, pack2(x0 - __uint_as_float(head << 16), x1 - __uint_as_float(head & 0xffff0000u))};
}

// out^T = W^T h^T + b: CH chunks of 32 inputs (B operands: heads hb and tails hl), TOUT tiles of 16 outputs.
template <int CH, int TOUT, bool TAILS = true>
__device__ __forceinline__ void dense_layer(const v4u (&hb)[CH], const v4u (&hl)[CH], const v4u* w, const float* bias, int lane,
                                            v4f (&out)[TOUT]) {
  const int g = lane >> 4;
#pragma unroll
  for (int ot = 0; ot < TOUT; ++ot) out[ot] = *reinterpret_cast<const v4f*>(bias + 16 * ot + 4 * g);
#pragma unroll
  for (int c = 0; c < CH; ++c)
#pragma unroll
    for (int ot = 0; ot < TOUT; ++ot) {
      const bf16x8 wv = __builtin_bit_cast(bf16x8, w[(ot * CH + c) * 64 + lane]);
      out[ot] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, __builtin_bit_cast(bf16x8, hb[c]), out[ot], 0, 0, 0);
      if constexpr (TAILS) out[ot] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, __builtin_bit_cast(bf16x8, hl[c]), out[ot], 0, 0, 0);
    }
}

// ReLU, split, and put pairs of 16-output tiles side by side as B operands of the next layer.
template <int T>
__device__ __forceinline__ void next_operands(const v4f (&h)[T], v4u (&hb)[(T + 1) / 2], v4u (&hl)[(T + 1) / 2]) {
#pragma unroll
  for (int m = 0; m < (T + 1) / 2; ++m) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int t = 2 * m + (e >> 1);                   // elements 0..3 from the even tile, 4..7 from the odd one
      HeadTail s = {0u, 0u};
      if (t < T) s = split2_relu(h[t][2 * (e & 1)], h[t][2 * (e & 1) + 1]);
      hb[m][e] = s.head;
      hl[m][e] = s.tail;
    }
  }
}

template <int T>
__device__ __forceinline__ void store_rows(const PredictArgs& a, const v4f (&y)[T], int64_t row, bool live, int g, int l_out) {
  if (!live) return;
#pragma unroll
  for (int ot = 0; ot < T; ++ot)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int c = 16 * ot + 4 * g + v;
      if (c < l_out) store_from_f32(a.Y, row * a.ldy + c, a.y_dtype, y[ot][v]);
    }
}

// Stages W (layer index `layer`) as A operands.  first: inputs are the hidden units of layer 1 (lane
// (g, i) of chunk kb holds units 32 kb + 8 g + t); otherwise they are pairs of 16-output tiles (unit
// 32 m + 4 g + e for e < 4, 32 m + 16 + 4 g + e - 4 for e >= 4).
__device__ __forceinline__ void stage_weights(const PredictArgs& a, int layer, bool first, int chunks, int tout, v4u* dst, float* bias_dst) {
  const bf16_t* W = static_cast<const bf16_t*>(a.W[layer]);
  const int64_t ldw = a.ldw[layer];
  const int win = a.win[layer], wout = a.wout[layer];
  for (int i = threadIdx.x; i < tout * chunks * 64; i += DBF_THREADS) {
    const int ln = i & 63, tile = i >> 6, ot = tile / chunks, c = tile - ot * chunks;
    const int g = ln >> 4, col = 16 * ot + (ln & 15);
    unsigned int h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int unit = first ? 32 * c + 8 * g + e : 32 * c + (e < 4 ? 4 * g + e : 16 + 4 * g + e - 4);
      h[e] = (unit < win && col < wout) ? W[static_cast<int64_t>(unit) * ldw + col] : 0u;
    }
    dst[i] = (v4u){h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
  }
  for (int i = threadIdx.x; i < 16 * tout; i += DBF_THREADS)
    bias_dst[i] = (i < wout && a.bias[layer]) ? bf16_to_f32(static_cast<const bf16_t*>(a.bias[layer])[i]) : 0.f;
}

// KB: l_1 <= 32 KB (a multiple of 8; lanes whose units lie past l_1 idle).  TH: later hidden layers (and, with two layers, the output) are at most 16 TH wide.
// NL: number of layers, 2, 3, or 4 for "four or more" (the count is then read at run time).
template <int KB, int TH, int NL>
__global__ __launch_bounds__(DBF_THREADS, (TH <= 8 ? 2 : 1)) void fused_deep_bf16_kernel(PredictArgs a, DeepBfLds L) {
  constexpr int M = (TH + 1) / 2;                       // 32-input chunks of a later hidden layer
  constexpr int TLAST = NL == 2 ? TH : 1;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63, g = lane >> 4, j = lane & 15;

  const int nl = NL == 4 ? a.n_layers : NL;
  stage_weights(a, 1, true, KB, TH, reinterpret_cast<v4u*>(smem + L.w[0]), reinterpret_cast<float*>(smem + L.b[0]));
  for (int layer = 2; layer < nl; ++layer)
    stage_weights(a, layer, false, M, (layer == nl - 1 && a.wout[nl - 1] <= 16) ? 1 : TH, reinterpret_cast<v4u*>(smem + L.w[layer - 1]),
                  reinterpret_cast<float*>(smem + L.b[layer - 1]));
  const int l1 = a.wout[0];
  // (the fact term's weights were read from memory in every pass, through the address path the gathers need:
  // 256 -> 17 with four fact columns 0.41 ms per 1e6 rows against 0.19 without any)
  for (int i = threadIdx.x; i < a.c_f * 32 * KB; i += DBF_THREADS) {
    const int q = i / (32 * KB), u = i - q * (32 * KB);
    reinterpret_cast<bf16_t*>(smem + L.wf)[i] = u < l1 ? static_cast<const bf16_t*>(a.W[0])[static_cast<int64_t>(q) * a.ldw[0] + u] : bf16_t{0};
  }
  __syncthreads();

  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (DBF_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (DBF_THREADS / 64);
  const int64_t npass = (a.n + 15) / 16;
  const int l_out = a.wout[nl - 1];

  // Gathers: the row of table k + 1 is requested before the row of table k is added up, so one row is
  // always in flight (lanes whose units lie past l_1 re-read the first piece of the row and add
  // nothing).  The first table of the next pass is requested before the matrix work of this pass, its
  // keys at the top of this pass.
  int key[LQ_MAX_DIMS];
  v4u w[2][KB];
  auto load_keys = [&](int64_t r, int (&kk)[LQ_MAX_DIMS]) {
#pragma unroll
    for (int k = 0; k < LQ_MAX_DIMS; ++k) kk[k] = k < a.K ? a.fk[k][r] : 0;
  };
  auto request = [&](int k, int f, v4u (&dst)[KB]) {
    const char* p = static_cast<const char*>(a.P[k]) +
                    (static_cast<uint64_t>(static_cast<uint32_t>(f) * static_cast<uint32_t>(a.ldp[k] >> 3)) << 4);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) dst[kb] = *reinterpret_cast<const v4u*>(p + (32 * kb + 8 * g < l1 ? 64 * kb + 16 * g : 0));
  };
  if (wave < npass) {
    load_keys(min<int64_t>(wave * 16 + j, a.n - 1), key);
    request(0, key[0], w[0]);
  }

  for (int64_t pass = wave; pass < npass; pass += nwaves) {
    // The staged model is read from LDS where it is used (otherwise the reads are hoisted out of
    // the loop and the weights take every register there is).
    asm volatile("" ::: "memory");
    const int64_t row = pass * 16 + j;
    const bool live = row < a.n;
    const int64_t rr = live ? row : a.n - 1;
    const bool more = pass + nwaves < npass;
    int keyn[LQ_MAX_DIMS];
    load_keys(min<int64_t>((more ? pass + nwaves : pass) * 16 + j, a.n - 1), keyn);

    // ---- layer 1: z = x W_f + sum_k P_k[fk_k] + b_1 in fp32, lane (g, j) owns units 32 kb + 8 g + t
    float acc[KB][8];
    if (a.bias[0]) {
      const bf16_t* b1 = static_cast<const bf16_t*>(a.bias[0]);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[kb][t] = 32 * kb + 8 * g < l1 ? bf16_to_f32(b1[32 * kb + 8 * g + t]) : 0.f;
    } else {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[kb][t] = 0.f;
    }
    if (a.c_f > 0) {
      const bf16_t* xr = static_cast<const bf16_t*>(a.X) + rr * a.ldx;
      const bf16_t* wf = reinterpret_cast<const bf16_t*>(smem + L.wf) + 8 * g;
      for (int q = 0; q < a.c_f; ++q) {
        const float x = bf16_to_f32(xr[q]);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const v4u t = *reinterpret_cast<const v4u*>(wf + (q * KB + kb) * 32);     // (zeros where the units lie past l_1)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[kb][2 * e] = fmaf(x, __uint_as_float(t[e] << 16), acc[kb][2 * e]);
            acc[kb][2 * e + 1] = fmaf(x, __uint_as_float(t[e] & 0xffff0000u), acc[kb][2 * e + 1]);
          }
        }
      }
    }
#pragma unroll
    for (int k = 0; k < LQ_MAX_DIMS; ++k) {
      if (k >= a.K) break;
      if (k + 1 < a.K) request(k + 1, key[(k + 1) % LQ_MAX_DIMS], w[(k + 1) & 1]);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        if (32 * kb + 8 * g < l1) unpack_add(w[k & 1][kb], acc[kb]);
    }
    if (more) request(0, keyn[0], w[0]);
#pragma unroll
    for (int k = 0; k < LQ_MAX_DIMS; ++k) key[k] = keyn[k];
    // the wide first hidden layer is rounded to bf16 once (rounding errors of many units average out),
    // as in the one-tile bf16 kernel; the few activations of the later layers are fed head and tail
    v4u hb[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
      hb[kb] = (v4u){pack2(fmaxf(acc[kb][0], 0.f), fmaxf(acc[kb][1], 0.f)), pack2(fmaxf(acc[kb][2], 0.f), fmaxf(acc[kb][3], 0.f)),
                     pack2(fmaxf(acc[kb][4], 0.f), fmaxf(acc[kb][5], 0.f)), pack2(fmaxf(acc[kb][6], 0.f), fmaxf(acc[kb][7], 0.f))};

    // ---- later layers
    const v4u* w2 = reinterpret_cast<const v4u*>(smem + L.w[0]);
    const float* b2 = reinterpret_cast<const float*>(smem + L.b[0]);
    if constexpr (NL == 2) {
      v4f y[TLAST];
      dense_layer<KB, TLAST, false>(hb, hb, w2, b2, lane, y);
      store_rows<TLAST>(a, y, row, live, g, l_out);
    } else {
      v4f h2[TH];
      dense_layer<KB, TH, false>(hb, hb, w2, b2, lane, h2);
      v4u hb2[M], hl2[M];
      next_operands<TH>(h2, hb2, hl2);
      if constexpr (NL == 4) {
        for (int layer = 2; layer < nl - 1; ++layer) {     // the hidden layers between the second and the last
          v4f h3[TH];
          dense_layer<M, TH>(hb2, hl2, reinterpret_cast<const v4u*>(smem + L.w[layer - 1]),
                             reinterpret_cast<const float*>(smem + L.b[layer - 1]), lane, h3);
          next_operands<TH>(h3, hb2, hl2);
        }
      }
      const v4u* wlast = reinterpret_cast<const v4u*>(smem + L.w[nl - 2]);
      const float* blast = reinterpret_cast<const float*>(smem + L.b[nl - 2]);
      if (l_out <= 16) {
        v4f y[1];
        dense_layer<M, 1>(hb2, hl2, wlast, blast, lane, y);
        store_rows<1>(a, y, row, live, g, l_out);
      } else {
        v4f y[TH];
        dense_layer<M, TH>(hb2, hl2, wlast, blast, lane, y);
        store_rows<TH>(a, y, row, live, g, l_out);
      }
    }
  }
}

}  // namespace

// Returns -1 when the shape is not one this kernel covers.
int try_fused_deep_bf16(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype != LQ_BF16 || a.p_dtype != LQ_BF16) return -1;
  const int NL = a.n_layers;
  if (NL < 2 || NL > LQ_MAX_LAYERS || a.c_f > 64 || a.K < 1) return -1;
  const int l1 = a.wout[0];
  if (l1 % 8 || l1 > 256) return -1;
  const int KB = l1 <= 32 ? 1 : (l1 <= 64 ? 2 : (l1 <= 128 ? 4 : 8));   // 32-unit blocks, padded to a power of two
  for (int k = 0; k < a.K; ++k) {
    if (!aligned(a.P[k], 16) || a.ldp[k] % 8) return -1;
    if (a.prows[k] * (a.ldp[k] / 8) > 0xffffffffLL) return -1;     // the kernel counts 16-byte pieces of a table in 32 bits
  }
  const int l_out = a.wout[NL - 1];
  // (two layers with up to 16 outputs: the one-tile bf16 kernel, tried before this one, takes first layers of 32, 64, 128
  // and 256 columns without fact columns; other widths that are multiples of 8, and stars with fact columns, end up here)
  int wide = 0;
  for (int j = 1; j < NL; ++j)
    if (j < NL - 1 || NL == 2 || l_out > 16) wide = std::max(wide, a.wout[j]);   // (an output layer of <= 16 is its own tile)
  if (wide > 256) return -1;
  const int TH = wide <= 16 ? 1 : (wide <= 32 ? 2 : (wide <= 64 ? 4 : (wide <= 128 ? 8 : 16)));
  const int M = (TH + 1) / 2;

  DeepBfLds L{};
  int off = 0;
  for (int j = 1; j < NL; ++j) {
    const int chunks = j == 1 ? KB : M;
    const int tout = (j == NL - 1 && NL > 2 && l_out <= 16) ? 1 : TH;
    L.w[j - 1] = off; off += tout * chunks * 64 * 16;
    L.b[j - 1] = off; off += 16 * tout * 4;
  }
  L.wf = off; off += a.c_f * KB * 64;
  L.total = off;
  const size_t lds = static_cast<size_t>(off);
  if (lds > 150 * 1024) return -1;

  const int64_t npass = (a.n + 15) / 16;
  const int64_t blocks = (npass + 3) / 4;             // capped below at one resident set: every wavefront stages once
  if (blocks <= 0 || a.probe) return LQ_OK;
#define LQ_DBF(KB_, TH_, NL_)                                                                           \
  do {                                                                                                  \
    const void* fn = reinterpret_cast<const void*>(&fused_deep_bf16_kernel<KB_, TH_, NL_>);              \
    if (lds > 64 * 1024)                                                                                \
      LQ_HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
    const int64_t resident = static_cast<int64_t>(num_cus()) * resident_per_cu(fn, DBF_THREADS, lds);   \
    hipLaunchKernelGGL((fused_deep_bf16_kernel<KB_, TH_, NL_>), dim3(static_cast<unsigned>(std::min(blocks, resident))), \
                       dim3(DBF_THREADS), lds, s, a, L);                                                \
  } while (0)
#define LQ_DBF_KB(TH_, NL_)                                                                             \
  do {                                                                                                  \
    if (KB == 1) LQ_DBF(1, TH_, NL_); else if (KB == 2) LQ_DBF(2, TH_, NL_);                            \
    else if (KB == 4) LQ_DBF(4, TH_, NL_); else LQ_DBF(8, TH_, NL_);                                    \
  } while (0)
#define LQ_DBF_TH(NL_)                                                                                  \
  do {                                                                                                  \
    if (TH == 1) LQ_DBF_KB(1, NL_); else if (TH == 2) LQ_DBF_KB(2, NL_); else if (TH == 4) LQ_DBF_KB(4, NL_); \
    else if (TH == 8) LQ_DBF_KB(8, NL_); else LQ_DBF_KB(16, NL_);                                       \
  } while (0)
  if (NL == 2) LQ_DBF_TH(2); else if (NL == 3) LQ_DBF_TH(3); else LQ_DBF_TH(4);
#undef LQ_DBF_TH
#undef LQ_DBF_KB
#undef LQ_DBF
  LQ_LAUNCH_CHECK("fused_deep_bf16_kernel");
  return LQ_OK;
}

}  // namespace lq
