// Join-computation stage (last line of Eq. 1) for hidden widths 128 and 256 in fp32: the same
// organisation as the width-64 kernel, with 32 or 64 lanes per fact row.
//
// A wavefront owns 64 consecutive fact rows at a time.  Their fact columns and keys are read once,
// coalesced (lane l holds row l).  With LPR = l_1 / 4 lanes per row the wavefront is 64 / LPR lane
// groups; in pass t (0 .. LPR-1) group g works on fact row g LPR + t, lane c of the group owning
// hidden columns 4c..4c+3, so that a projected row (512 or 1024 bytes) is fetched by one group as
// one contiguous run.  The row's key and fact values reach the group through the cross-lane
// network (a lane read for 64 lanes per row, a permute otherwise).  Gathers are software-pipelined
// in groups of four passes, across batches too; the pass loop is a run-time loop, so the code
// stays small for 32 or 64 passes.  A 2-layer model with one output sums over the lanes of a row
// and parks the result of pass t in lane t of the group: one coalesced store per batch.
#include "lq_common.h"

namespace lq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int RBW_THREADS = 256;

template <int CTRL> __device__ __forceinline__ float dppw(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over the LPR (32 or 64) lanes of a group, result in every lane.
template <int LPR> __device__ __forceinline__ float group_sum(float y) {
  y += dppw<0xB1>(y);                  // quad_perm [1,0,3,2]
  y += dppw<0x4E>(y);                  // quad_perm [2,3,0,1]
  y += dppw<0x141>(y);                 // row_half_mirror
  y += dppw<0x140>(y);                 // row_mirror
  y += __shfl_xor(y, 16, 64);
  if (LPR == 64) y += __shfl_xor(y, 32, 64);
  return y;
}
// Value that lane (group base + t) holds, for every lane of the group.
template <int LPR> __device__ __forceinline__ int from_lane(int v, int t, int group_base) {
  if constexpr (LPR == 64) return __builtin_amdgcn_readlane(v, t);
  else return __shfl(v, group_base | t, 64);
}

template <int K, int CFC> struct WRow {
  int fk[K];
  v4f x[CFC > 0 ? CFC : 1];
};
template <int K> struct WGather { v4f p[4][K]; };

template <int K, int CFC>
__device__ __forceinline__ void load_rows(const PredictArgs& a, int64_t rr, WRow<K, CFC>& r) {
#pragma unroll
  for (int k = 0; k < K; ++k) r.fk[k] = __builtin_nontemporal_load(a.fk[k] + rr);
  const float* xr = static_cast<const float*>(a.X) + rr * a.ldx;
#pragma unroll
  for (int q = 0; q < CFC; ++q) r.x[q] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(xr) + q);
}

// Gathers of passes 4 grp .. 4 grp + 3.
template <int LPR, int K, int CFC>
__device__ __forceinline__ void issue_group(const PredictArgs& a, int c, int group_base, int grp,
                                            const WRow<K, CFC>& r, WGather<K>& g) {
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int j = from_lane<LPR>(r.fk[k], 4 * grp + u, group_base);
      g.p[u][k] = *reinterpret_cast<const v4f*>(static_cast<const float*>(a.P[k]) +
                                                static_cast<int64_t>(j) * a.ldp[k] + 4 * c);
    }
}

template <int CFC, int NL> struct WConsts {
  float wf[CFC > 0 ? CFC * 4 : 1][4];   // W_f rows x this lane's 4 columns
  float b1[4];
  float w2[4];
  float b2;
};

template <int LPR, int K, int CFC, int NL>
__device__ __forceinline__ void compute_group(const PredictArgs& a, int c, int group_base, int grp, int64_t row0,
                                              const WRow<K, CFC>& r, const WGather<K>& g,
                                              const WConsts<CFC, NL>& w, float& ykeep) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int t = 4 * grp + u;
    float z[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) z[v] = w.b1[v];
#pragma unroll
    for (int q = 0; q < CFC; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float xe = __int_as_float(from_lane<LPR>(__float_as_int(r.x[q][e]), t, group_base));
#pragma unroll
        for (int v = 0; v < 4; ++v) z[v] = fmaf(xe, w.wf[q * 4 + e][v], z[v]);
      }
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int v = 0; v < 4; ++v) z[v] += g.p[u][k][v];
    if constexpr (NL == 1) {
      const int64_t row = row0 + group_base + t;
      if (row < a.n) {
        const v4f o = {z[0], z[1], z[2], z[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(static_cast<float*>(a.Y) + row * a.ldy + 4 * c));
      }
    } else {
      float y = 0.f;
#pragma unroll
      for (int v = 0; v < 4; ++v) y = fmaf(fmaxf(z[v], 0.f), w.w2[v], y);
      y = group_sum<LPR>(y);
      if (c == t) ykeep = y;
    }
  }
}

// LPR lanes per row (l_1 = 4 LPR), K dimensions, CFC float4 chunks of fact columns, NL layers
// (the second one with a single output).
// Three wavefronts per SIMD leave 170 registers each; the double-buffered gathers of many
// dimensions plus many fact columns need more, and two per SIMD is faster than spilling.
constexpr int waves_per_simd(int K, int CFC) { return 32 * K + 24 * CFC > 100 ? 2 : 3; }

template <int LPR, int K, int CFC, int NL>
__global__ __launch_bounds__(RBW_THREADS)
__attribute__((amdgpu_waves_per_eu(waves_per_simd(K, CFC), waves_per_simd(K, CFC))))
void fused_rowbatch_wide_kernel(PredictArgs a) {
  constexpr int NG = LPR / 4;            // groups of four passes per batch (8 or 16)
  const int lane = threadIdx.x & 63, c = lane & (LPR - 1), group_base = lane & ~(LPR - 1);
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (RBW_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (RBW_THREADS / 64);
  const int64_t nb = (a.n + 63) / 64;
  if (wave >= nb) return;

  WConsts<CFC, NL> w;
  {
    const float* W0 = static_cast<const float*>(a.W[0]);
#pragma unroll
    for (int q = 0; q < CFC * 4; ++q)
#pragma unroll
      for (int v = 0; v < 4; ++v) w.wf[q][v] = W0[static_cast<int64_t>(q) * a.ldw[0] + 4 * c + v];
#pragma unroll
    for (int v = 0; v < 4; ++v) w.b1[v] = a.bias[0] ? static_cast<const float*>(a.bias[0])[4 * c + v] : 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v)
      w.w2[v] = NL == 2 ? static_cast<const float*>(a.W[1])[static_cast<int64_t>(4 * c + v) * a.ldw[1]] : 0.f;
    w.b2 = (NL == 2 && a.bias[1]) ? static_cast<const float*>(a.bias[1])[0] : 0.f;
  }

  int64_t b = wave;
  int64_t row = b * 64 + lane;
  WRow<K, CFC> cur, nxt;
  load_rows<K, CFC>(a, row < a.n ? row : a.n - 1, cur);
  WGather<K> ga, gb;
  issue_group<LPR, K, CFC>(a, c, group_base, 0, cur, ga);
  for (;;) {
    const int64_t bn = b + nwaves;
    const bool more = bn < nb;
    const int64_t rown = bn * 64 + lane;
    load_rows<K, CFC>(a, (more && rown < a.n) ? rown : a.n - 1, nxt);
    float yk = 0.f;
    const int64_t row0 = b * 64;
#pragma unroll 1
    for (int grp = 0; grp < NG; grp += 2) {
      issue_group<LPR, K, CFC>(a, c, group_base, grp + 1, cur, gb);
      compute_group<LPR, K, CFC, NL>(a, c, group_base, grp, row0, cur, ga, w, yk);
      if (grp + 2 < NG) issue_group<LPR, K, CFC>(a, c, group_base, grp + 2, cur, ga);
      else issue_group<LPR, K, CFC>(a, c, group_base, 0, nxt, ga);   // first group of the next batch (valid rows repeated at the end)
      compute_group<LPR, K, CFC, NL>(a, c, group_base, grp + 1, row0, cur, gb, w, yk);
    }
    if constexpr (NL == 2) {
      if (row < a.n) __builtin_nontemporal_store(yk + w.b2, static_cast<float*>(a.Y) + row * a.ldy);
    }
    if (!more) break;
    b = bn;
    row = rown;
    cur = nxt;
  }
}

template <int LPR, int K, int CFC, int NL>
int launch_inst(const PredictArgs& a, hipStream_t s) {
  const int64_t nb = (a.n + 63) / 64;
  const int64_t blocks = std::min<int64_t>((nb + 3) / 4, static_cast<int64_t>(num_cus()) * waves_per_simd(K, CFC));
  hipLaunchKernelGGL((fused_rowbatch_wide_kernel<LPR, K, CFC, NL>), dim3(static_cast<unsigned>(blocks)),
                     dim3(RBW_THREADS), 0, s, a);
  LQ_LAUNCH_CHECK("fused_rowbatch_wide_kernel");
  return LQ_OK;
}

template <int LPR, int K, int CFC>
int pick_layers(const PredictArgs& a, hipStream_t s) {
  return a.n_layers == 1 ? launch_inst<LPR, K, CFC, 1>(a, s) : launch_inst<LPR, K, CFC, 2>(a, s);
}

template <int LPR, int K>
int pick_cf(const PredictArgs& a, hipStream_t s) {
  switch (a.c_f) {
    case 0: return pick_layers<LPR, K, 0>(a, s);
    case 4: return pick_layers<LPR, K, 1>(a, s);
    case 8: return pick_layers<LPR, K, 2>(a, s);
    default: return -1;
  }
}

template <int LPR>
int pick_k(const PredictArgs& a, hipStream_t s) {
  switch (a.K) {
    case 1: return pick_cf<LPR, 1>(a, s);
    case 2: return pick_cf<LPR, 2>(a, s);
    case 3: return pick_cf<LPR, 3>(a, s);
    case 4: return pick_cf<LPR, 4>(a, s);
    default: return -1;
  }
}

}  // namespace

// Returns -1 when the shape is not one this kernel covers.
int try_rowbatch_wide(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype != LQ_F32 || a.p_dtype != LQ_F32 || a.y_dtype != LQ_F32) return -1;
  if (a.wout[0] != 128 && a.wout[0] != 256) return -1;
  if (a.n_layers > 2 || (a.n_layers == 2 && a.wout[1] != 1)) return -1;
  if (a.n < 256) return -1;
  for (int k = 0; k < a.K; ++k)
    if (!aligned(a.P[k], 16) || a.ldp[k] % 4) return -1;
  if (a.c_f > 0 && (!aligned(a.X, 16) || a.ldx % 4)) return -1;
  if (a.n_layers == 1 && (!aligned(a.Y, 16) || a.ldy % 4)) return -1;
  return a.wout[0] == 128 ? pick_k<32>(a, s) : pick_k<64>(a, s);
}

}  // namespace lq
