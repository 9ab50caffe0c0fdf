// Join-computation stage (last line of Eq. 1) for hidden width 64 in fp32, the shape of the
// paper's "large input, small model" experiments: z_i = x_i W_f + sum_k P_k[fk_k[i], :].
//
// A wavefront owns 64 consecutive fact rows at a time.  The fact columns and the key columns of
// those rows are read ONCE, fully coalesced (lane l holds row l), and then handed around with
// DPP row broadcasts, which cost a VALU slot but no memory-pipe bandwidth: in pass t (0..15) the
// 16 lanes of DPP row s work on fact row 16 s + t, lane c owning hidden columns 4c..4c+3, so a
// projected row of 256 bytes is fetched by one 16-lane group as one contiguous run.  Gathers are
// software-pipelined in groups of four passes (the next group's loads are in flight while the
// current one is consumed, across batches too).  The result of pass t is parked in lane t of each
// DPP row, so a batch ends with one coalesced store (MLP) or per-pass 256-byte row stores
// (linear operator).
#include "lq_common.h"

namespace lq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int RB_THREADS = 256;
constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_MIRROR = 0x140;
constexpr int DPP_ROW_BCAST0 = 0x150;      // row_newbcast:n = 0x150 + n

template <int CTRL> __device__ __forceinline__ float dppf(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL> __device__ __forceinline__ int dppi(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
// Sum over the 16 lanes of a DPP row, result in every lane.
__device__ __forceinline__ float row_allreduce16(float y) {
  y += dppf<DPP_QUAD_XOR1>(y);
  y += dppf<DPP_QUAD_XOR2>(y);
  y += dppf<DPP_ROW_HALF_MIRROR>(y);
  y += dppf<DPP_ROW_MIRROR>(y);
  return y;
}

// Per-batch registers: lane l holds fact row (batch*64 + l).
template <int K, int CFC> struct RowRegs {
  int fk[K > 0 ? K : 1];
  v4f x[CFC > 0 ? CFC : 1];
};
// Gathered rows of one group of 4 passes.
template <int K> struct Gathered { v4f p[4][K > 0 ? K : 1]; };

template <int K, int CFC>
__device__ __forceinline__ void load_rows(const PredictArgs& a, int64_t rr, RowRegs<K, CFC>& r) {
#pragma unroll
  for (int k = 0; k < K; ++k) r.fk[k] = __builtin_nontemporal_load(a.fk[k] + rr);
  const float* xr = static_cast<const float*>(a.X) + rr * a.ldx;
#pragma unroll
  for (int q = 0; q < CFC; ++q) r.x[q] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(xr) + q);
}

// Keys become byte offsets of their rows once per batch (one 32-bit product per key: the host has
// checked that every projected table is smaller than 4 GiB), so that a gather costs a broadcast and one
// add on top of its load instead of a 64-bit multiply-add.
template <int K, int CFC>
__device__ __forceinline__ void keys_to_offsets(const PredictArgs& a, RowRegs<K, CFC>& r) {
#pragma unroll
  for (int k = 0; k < K; ++k)
    r.fk[k] = static_cast<int>(static_cast<uint32_t>(r.fk[k]) * (static_cast<uint32_t>(a.ldp[k]) * 4u));
}

template <int T, int K, int CFC>
__device__ __forceinline__ void issue_pass(const PredictArgs& a, int c, const RowRegs<K, CFC>& r,
                                           v4f (&p)[K > 0 ? K : 1]) {
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const uint32_t at = static_cast<uint32_t>(dppi<DPP_ROW_BCAST0 + T>(r.fk[k])) + 16u * static_cast<uint32_t>(c);
    p[k] = *reinterpret_cast<const v4f*>(static_cast<const char*>(a.P[k]) + at);
  }
}
template <int GRP, int K, int CFC>
__device__ __forceinline__ void issue_group(const PredictArgs& a, int c, const RowRegs<K, CFC>& r,
                                            Gathered<K>& g) {
  issue_pass<GRP * 4 + 0, K, CFC>(a, c, r, g.p[0]);
  issue_pass<GRP * 4 + 1, K, CFC>(a, c, r, g.p[1]);
  issue_pass<GRP * 4 + 2, K, CFC>(a, c, r, g.p[2]);
  issue_pass<GRP * 4 + 3, K, CFC>(a, c, r, g.p[3]);
}

// Constants a lane keeps for the whole kernel.
template <int CFC, int NL, int L2> struct LaneConsts {
  float wf[CFC > 0 ? CFC * 4 : 1][4];   // W_f rows x this lane's 4 columns
  float b1[4];
  float w2[NL == 2 ? 4 : 1][NL == 2 ? L2 : 1];
  float b2[NL == 2 ? L2 : 1];
};

template <int T, int K, int CFC, int NL, int L2>
__device__ __forceinline__ void compute_pass(const PredictArgs& a, int c, int64_t batch_row0, int s,
                                             const RowRegs<K, CFC>& r, const v4f (&p)[K > 0 ? K : 1],
                                             const LaneConsts<CFC, NL, L2>& w, float (&ykeep)[NL == 2 ? L2 : 1]) {
  float z[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) z[v] = w.b1[v];
#pragma unroll
  for (int q = 0; q < CFC; ++q)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xe = dppf<DPP_ROW_BCAST0 + T>(r.x[q][e]);
#pragma unroll
      for (int v = 0; v < 4; ++v) z[v] = fmaf(xe, w.wf[q * 4 + e][v], z[v]);
    }
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int v = 0; v < 4; ++v) z[v] += p[k][v];

  if constexpr (NL == 1) {
    const int64_t row = batch_row0 + 16 * s + T;
    if (row < a.n) {
      v4f o = {z[0], z[1], z[2], z[3]};
      __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(static_cast<float*>(a.Y) + row * a.ldy + 4 * c));
    }
  } else {
    float y[L2];
#pragma unroll
    for (int o = 0; o < L2; ++o) y[o] = 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float h = fmaxf(z[v], 0.f);
#pragma unroll
      for (int o = 0; o < L2; ++o) y[o] = fmaf(h, w.w2[v][o], y[o]);
    }
#pragma unroll
    for (int o = 0; o < L2; ++o) {
      const float t = row_allreduce16(y[o]);
      if (c == T) ykeep[o] = t;
    }
  }
}
template <int GRP, int K, int CFC, int NL, int L2>
__device__ __forceinline__ void compute_group(const PredictArgs& a, int c, int64_t row0, int s,
                                              const RowRegs<K, CFC>& r, const Gathered<K>& g,
                                              const LaneConsts<CFC, NL, L2>& w,
                                              float (&ykeep)[NL == 2 ? L2 : 1]) {
  compute_pass<GRP * 4 + 0, K, CFC, NL, L2>(a, c, row0, s, r, g.p[0], w, ykeep);
  compute_pass<GRP * 4 + 1, K, CFC, NL, L2>(a, c, row0, s, r, g.p[1], w, ykeep);
  compute_pass<GRP * 4 + 2, K, CFC, NL, L2>(a, c, row0, s, r, g.p[2], w, ykeep);
  compute_pass<GRP * 4 + 3, K, CFC, NL, L2>(a, c, row0, s, r, g.p[3], w, ykeep);
}

// K dimensions, CFC float4 chunks of fact columns (c_f = 4 CFC), NL layers (1 or 2), L2 outputs.
template <int K, int CFC, int NL, int L2>
// (Three wavefronts per SIMD leave 170 registers each; with several outputs the per-pass partial sums no
// longer fit and two per SIMD is faster than spilling.)
__global__ __launch_bounds__(RB_THREADS)
__attribute__((amdgpu_waves_per_eu((NL == 2 && L2 > 1) ? 2 : 3, (NL == 2 && L2 > 1) ? 2 : 3)))
void fused_rowbatch64_kernel(PredictArgs a) {
  const int lane = threadIdx.x & 63, c = lane & 15, s = lane >> 4;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (RB_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (RB_THREADS / 64);
  const int64_t nb = (a.n + 63) / 64;
  if (wave >= nb) return;
  const bool y_vec = a.ldy % 4 == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0;

  LaneConsts<CFC, NL, L2> w;
  {
    const float* W0 = static_cast<const float*>(a.W[0]);
#pragma unroll
    for (int q = 0; q < CFC * 4; ++q)
#pragma unroll
      for (int v = 0; v < 4; ++v) w.wf[q][v] = W0[static_cast<int64_t>(q) * a.ldw[0] + 4 * c + v];
#pragma unroll
    for (int v = 0; v < 4; ++v) w.b1[v] = a.bias[0] ? static_cast<const float*>(a.bias[0])[4 * c + v] : 0.f;
    if constexpr (NL == 2) {
      const float* W1 = static_cast<const float*>(a.W[1]);
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int o = 0; o < L2; ++o) w.w2[v][o] = W1[static_cast<int64_t>(4 * c + v) * a.ldw[1] + o];
#pragma unroll
      for (int o = 0; o < L2; ++o) w.b2[o] = a.bias[1] ? static_cast<const float*>(a.bias[1])[o] : 0.f;
    }
  }

  int64_t b = wave;
  int64_t row = b * 64 + lane;
  RowRegs<K, CFC> cur, nxt;
  load_rows<K, CFC>(a, row < a.n ? row : a.n - 1, cur);
  keys_to_offsets<K, CFC>(a, cur);
  Gathered<K> ga, gb;
  issue_group<0, K, CFC>(a, c, cur, ga);
  for (;;) {
    const int64_t bn = b + nwaves;
    const bool more = bn < nb;
    const int64_t rown = bn * 64 + lane;
    load_rows<K, CFC>(a, (more && rown < a.n) ? rown : a.n - 1, nxt);
    float yk[NL == 2 ? L2 : 1];
#pragma unroll
    for (int o = 0; o < (NL == 2 ? L2 : 1); ++o) yk[o] = 0.f;
    const int64_t row0 = b * 64;
    issue_group<1, K, CFC>(a, c, cur, gb);
    compute_group<0, K, CFC, NL, L2>(a, c, row0, s, cur, ga, w, yk);
    issue_group<2, K, CFC>(a, c, cur, ga);
    compute_group<1, K, CFC, NL, L2>(a, c, row0, s, cur, gb, w, yk);
    issue_group<3, K, CFC>(a, c, cur, gb);
    compute_group<2, K, CFC, NL, L2>(a, c, row0, s, cur, ga, w, yk);
    keys_to_offsets<K, CFC>(a, nxt);
    issue_group<0, K, CFC>(a, c, nxt, ga);   // first group of the next batch (a repeat of valid rows at the end)
    compute_group<3, K, CFC, NL, L2>(a, c, row0, s, cur, gb, w, yk);
    if constexpr (NL == 2) {
      if (row < a.n) {
        float* yr = static_cast<float*>(a.Y) + row * a.ldy;
        if (L2 == 4 && y_vec) {            // the row's four outputs as one 16-byte store
          const v4f o4 = {yk[0] + w.b2[0], yk[L2 > 1 ? 1 : 0] + w.b2[L2 > 1 ? 1 : 0],
                          yk[L2 > 2 ? 2 : 0] + w.b2[L2 > 2 ? 2 : 0], yk[L2 > 3 ? 3 : 0] + w.b2[L2 > 3 ? 3 : 0]};
          __builtin_nontemporal_store(o4, reinterpret_cast<v4f*>(yr));
        } else {
#pragma unroll
          for (int o = 0; o < L2; ++o) __builtin_nontemporal_store(yk[o] + w.b2[o], yr + o);
        }
      }
    }
    if (!more) break;
    b = bn;
    row = rown;
    cur = nxt;
  }
}

template <int K, int CFC, int NL, int L2>
int launch_inst(const PredictArgs& a, hipStream_t s) {
  const int64_t nb = (a.n + 63) / 64;
  const int64_t blocks = std::min<int64_t>((nb + 3) / 4, static_cast<int64_t>(num_cus()) * ((NL == 2 && L2 > 1) ? 2 : 3));
  if (a.probe) return LQ_OK;
  hipLaunchKernelGGL((fused_rowbatch64_kernel<K, CFC, NL, L2>), dim3(static_cast<unsigned>(blocks)),
                     dim3(RB_THREADS), 0, s, a);
  LQ_LAUNCH_CHECK("fused_rowbatch64_kernel");
  return LQ_OK;
}

template <int K, int CFC>
int pick_layers(const PredictArgs& a, hipStream_t s) {
  if (a.n_layers == 1) return launch_inst<K, CFC, 1, 1>(a, s);
  switch (a.wout[1]) {
    case 1: return launch_inst<K, CFC, 2, 1>(a, s);
    case 2: return launch_inst<K, CFC, 2, 2>(a, s);
    case 4: return launch_inst<K, CFC, 2, 4>(a, s);
    default: return -1;
  }
}

template <int K>
int pick_cf(const PredictArgs& a, hipStream_t s) {
  switch (a.c_f) {
    case 0: return pick_layers<K, 0>(a, s);
    case 4: return pick_layers<K, 1>(a, s);
    case 8: return pick_layers<K, 2>(a, s);
    default: return -1;
  }
}

}  // namespace

// Returns -1 when the shape is not one this kernel covers.
int try_rowbatch64(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype != LQ_F32 || a.p_dtype != LQ_F32 || a.y_dtype != LQ_F32) return -1;
  if (a.wout[0] != 64 || a.n_layers > 2 || a.K < 1 || a.K > 4) return -1;
  if (a.n < 256) return -1;   // too few 64-row batches to matter; the simpler kernel handles it
  for (int k = 0; k < a.K; ++k) {
    if (!aligned(a.P[k], 16) || a.ldp[k] % 4) return -1;
    if (a.prows[k] * a.ldp[k] * 4 > 0xffffffffLL) return -1;     // the kernel keeps byte offsets into a table in 32 bits
  }
  if (a.c_f > 0 && (!aligned(a.X, 16) || a.ldx % 4)) return -1;
  if (a.n_layers == 1 && (!aligned(a.Y, 16) || a.ldy % 4)) return -1;
  switch (a.K) {
    case 1: return pick_cf<1>(a, s);
    case 2: return pick_cf<2>(a, s);
    case 3: return pick_cf<3>(a, s);
    case 4: return pick_cf<4>(a, s);
    default: return -1;
  }
}

}  // namespace lq
