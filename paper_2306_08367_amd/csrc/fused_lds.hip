// Join-computation stage of Eq. 1 for linear models with 1, 2 or 4 outputs (the regression models of
// Section 3.2): Y = X W_f + sum_k P_k[fk_k] + b with projected tables of a few bytes per row.  The
// gathers of such rows are bound by the request rate of the vector memory path (one request per
// 4..16 bytes), not by bytes, so the tables that fit are kept in LDS: one persistent workgroup per
// compute unit stages them once, then streams over the fact rows; tables that do not fit are
// gathered from memory as before.
#include <algorithm>

#include "lq_common.h"

namespace lq {
namespace {

constexpr int FL_THREADS = 1024;
// rows per thread and step, 64 apart (lanes hold neighbouring rows); fewer for wider rows so that a
// 1,024-thread workgroup stays within 128 registers per lane
constexpr int fl_rows(int L, int KT) { return (L == 1 && KT <= 4) ? 4 : 2; }
constexpr int FL_MAX_CF = 8;            // fact columns (kept in registers)

struct LdsPlan {
  int32_t off[LQ_MAX_DIMS];             // position of table k in LDS in floats, -1 = stays in memory
  int32_t w_off;                        // W_f (c_f x L) followed by the bias (L)
  int32_t vec_x, vec_y;                 // rows of X as 16-byte pieces; rows of Y as one L-float store
};

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

template <int L>
__device__ __forceinline__ void load_row(const float* p, float (&v)[L]) {
  if constexpr (L == 4) {
    const v4f t = *reinterpret_cast<const v4f*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else if constexpr (L == 2) {
    const v2f t = *reinterpret_cast<const v2f*>(p);
    v[0] = t.x; v[1] = t.y;
  } else {
    v[0] = p[0];
  }
}

template <int L, int KT>      // outputs; number of dimensions, 1..4 (1..8 at one output)
__global__ __launch_bounds__(FL_THREADS) void fused_lds_kernel(PredictArgs a, LdsPlan pl) {
  constexpr int R = fl_rows(L, KT);
  extern __shared__ __align__(16) float tab[];
  const int tid = threadIdx.x;
  for (int k = 0; k < KT; ++k)
    if (pl.off[k] >= 0) {
      const float* __restrict__ src = static_cast<const float*>(a.P[k]);
      const int cnt = static_cast<int>(a.prows[k]) * L;            // (rows are contiguous: ldp == L)
      for (int i0 = tid; i0 < cnt; i0 += 4 * FL_THREADS) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i0 + e * FL_THREADS < cnt) v[e] = src[i0 + e * FL_THREADS];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i0 + e * FL_THREADS < cnt) tab[pl.off[k] + i0 + e * FL_THREADS] = v[e];
      }
    }
  if (tid < a.c_f * L) tab[pl.w_off + tid] = static_cast<const float*>(a.W[0])[(tid / L) * a.ldw[0] + tid % L];
  if (tid < L) tab[pl.w_off + a.c_f * L + tid] = a.bias[0] ? static_cast<const float*>(a.bias[0])[tid] : 0.f;
  __syncthreads();
  float wf[FL_MAX_CF][L], bias[L];
#pragma unroll
  for (int c = 0; c < FL_MAX_CF; ++c)
#pragma unroll
    for (int o = 0; o < L; ++o) wf[c][o] = c < a.c_f ? tab[pl.w_off + c * L + o] : 0.f;
#pragma unroll
  for (int o = 0; o < L; ++o) bias[o] = tab[pl.w_off + a.c_f * L + o];

  const int64_t step = static_cast<int64_t>(gridDim.x) * FL_THREADS * R;
  const int in_block = 64 * R * (tid >> 6) + (tid & 63);
  int64_t base = static_cast<int64_t>(blockIdx.x) * FL_THREADS * R + in_block;
  if (base - in_block >= a.n) return;
  const float* __restrict__ X = static_cast<const float*>(a.X);
  float* __restrict__ Y = static_cast<float*>(a.Y);
  int key[KT][R];
  auto load_keys = [&](int64_t b, int (&out)[KT][R]) {
#pragma unroll
    for (int k = 0; k < KT; ++k)
#pragma unroll
      for (int u = 0; u < R; ++u) out[k][u] = a.fk[k][min(b + 64 * u, a.n - 1)];
  };
  load_keys(base, key);
  for (;;) {
    const int64_t nbase = base + step;
    const bool more = nbase - in_block < a.n;            // (uniform over the workgroup)
    int nkey[KT][R];
    load_keys(more ? nbase : base, nkey);                 // keys of the next step are in flight during this one
    v4f xlo[R], xhi[R];
#pragma unroll
    for (int u = 0; u < R; ++u) {
      v4f lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
      if (a.c_f > 0) {
        const float* p = X + min(base + 64 * u, a.n - 1) * a.ldx;
        if (pl.vec_x) {
          lo = *reinterpret_cast<const v4f*>(p);
          if (a.c_f > 4) hi = *reinterpret_cast<const v4f*>(p + 4);
        } else {
          lo.x = p[0];
          if (a.c_f > 1) lo.y = p[1];
          if (a.c_f > 2) lo.z = p[2];
          if (a.c_f > 3) lo.w = p[3];
          if (a.c_f > 4) hi.x = p[4];
          if (a.c_f > 5) hi.y = p[5];
          if (a.c_f > 6) hi.z = p[6];
          if (a.c_f > 7) hi.w = p[7];
        }
      }
      xlo[u] = lo; xhi[u] = hi;
    }
    float acc[R][L];
#pragma unroll
    for (int u = 0; u < R; ++u)
#pragma unroll
      for (int o = 0; o < L; ++o) acc[u][o] = bias[o];
#pragma unroll
    for (int k = 0; k < KT; ++k) {
      if (pl.off[k] >= 0) {                               // (uniform: a table is in LDS for every row or for none)
#pragma unroll
        for (int u = 0; u < R; ++u) {
          float v[L];
          load_row<L>(tab + pl.off[k] + key[k][u] * L, v);
#pragma unroll
          for (int o = 0; o < L; ++o) acc[u][o] += v[o];
        }
      } else {
        const float* __restrict__ g = static_cast<const float*>(a.P[k]);
        float v[R][L];
#pragma unroll
        for (int u = 0; u < R; ++u) load_row<L>(g + static_cast<int64_t>(key[k][u]) * a.ldp[k], v[u]);
#pragma unroll
        for (int u = 0; u < R; ++u)
#pragma unroll
          for (int o = 0; o < L; ++o) acc[u][o] += v[u][o];
      }
    }
    if (a.c_f > 0) {
#pragma unroll
      for (int u = 0; u < R; ++u)
#pragma unroll
        for (int o = 0; o < L; ++o) {
          float t = acc[u][o];
          t += xlo[u].x * wf[0][o]; t += xlo[u].y * wf[1][o]; t += xlo[u].z * wf[2][o]; t += xlo[u].w * wf[3][o];
          t += xhi[u].x * wf[4][o]; t += xhi[u].y * wf[5][o]; t += xhi[u].z * wf[6][o]; t += xhi[u].w * wf[7][o];
          acc[u][o] = t;
        }
    }
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int64_t row = base + 64 * u;
      if (row < a.n) {
        float* y = Y + row * a.ldy;
        if constexpr (L == 4) {
          if (pl.vec_y) __builtin_nontemporal_store(v4f{acc[u][0], acc[u][1], acc[u][2], acc[u][3]}, reinterpret_cast<v4f*>(y));
          else { y[0] = acc[u][0]; y[1] = acc[u][1]; y[2] = acc[u][2]; y[3] = acc[u][3]; }
        } else if constexpr (L == 2) {
          if (pl.vec_y) __builtin_nontemporal_store(v2f{acc[u][0], acc[u][1]}, reinterpret_cast<v2f*>(y));
          else { y[0] = acc[u][0]; y[1] = acc[u][1]; }
        } else {
          __builtin_nontemporal_store(acc[u][0], y);
        }
      }
    }
    if (!more) break;
    base = nbase;
#pragma unroll
    for (int k = 0; k < KT; ++k)
#pragma unroll
      for (int u = 0; u < R; ++u) key[k][u] = nkey[k][u];
  }
}

template <int L>
int launch_l(const PredictArgs& a, const LdsPlan& pl, size_t lds, hipStream_t s) {
  if (a.probe) return (a.K <= 4 || L == 1) ? LQ_OK : -1;
  const dim3 block(FL_THREADS);
#define LQ_FL(KT_)                                                                                      \
  do {                                                                                                  \
    const int64_t need = (a.n + FL_THREADS * fl_rows(L, KT_) - 1) / (FL_THREADS * fl_rows(L, KT_));     \
    const dim3 grid(static_cast<unsigned>(std::min<int64_t>(need, num_cus())));                         \
    if (lds > 64 * 1024)                                                                                \
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_lds_kernel<L, KT_>),          \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
    hipLaunchKernelGGL((fused_lds_kernel<L, KT_>), grid, block, lds, s, a, pl);                         \
  } while (0)
  if (a.K == 1) LQ_FL(1); else if (a.K == 2) LQ_FL(2); else if (a.K == 3) LQ_FL(3); else if (a.K == 4) LQ_FL(4);
  else if constexpr (L == 1) {            // (five to eight tables: one output only, to stay within the registers)
    if (a.K == 5) LQ_FL(5); else if (a.K == 6) LQ_FL(6); else if (a.K == 7) LQ_FL(7); else LQ_FL(8);
  } else {
    return -1;
  }
#undef LQ_FL
  LQ_LAUNCH_CHECK("fused_lds_kernel");
  return LQ_OK;
}

}  // namespace

// -1: the shape is not covered here.
int try_fused_lds(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype != LQ_F32 || a.p_dtype != LQ_F32 || a.y_dtype != LQ_F32) return -1;
  if (a.n_layers != 1 || a.K < 1 || a.K > 8 || a.c_f > FL_MAX_CF || a.n < (1 << 20)) return -1;
  const int L = a.wout[0];
  if (L != 1 && L != 2 && L != 4) return -1;
  if (a.K > 4 && L != 1) return -1;
  if (!aligned(a.Y, 4) || (a.c_f > 0 && !aligned(a.X, 4))) return -1;
  LdsPlan pl{};
  int order[LQ_MAX_DIMS];
  for (int k = 0; k < a.K; ++k) {
    order[k] = k;
    pl.off[k] = -1;
    // rows of a table in memory are read as one L-float piece
    if (!aligned(a.P[k], 4 * L) || a.ldp[k] % L) return -1;
  }
  std::stable_sort(order, order + a.K, [&](int x, int y) { return a.prows[x] < a.prows[y]; });
  const int64_t budget = (156 * 1024) / 4;                // floats, of the 160 KB of a compute unit
  int64_t used = 0;
  for (int q = 0; q < a.K; ++q) {
    const int k = order[q];
    if (a.ldp[k] != L || a.prows[k] * L > budget - used) continue;
    pl.off[k] = static_cast<int32_t>(used);
    used += (a.prows[k] * L + 3) / 4 * 4;                 // keeps every table 16-byte aligned
  }
  int in_lds = 0;
  for (int k = 0; k < a.K; ++k) in_lds += pl.off[k] >= 0 ? 1 : 0;
  // with most tables left in memory the streaming kernels, which keep more gathers in flight, are
  // faster (measured: one table of three in LDS at four outputs, 0.25 against 0.15 ms per 1e7 rows)
  if (2 * in_lds < a.K) return -1;
  pl.w_off = static_cast<int32_t>(used);
  pl.vec_x = (a.c_f == 4 || a.c_f == 8) && aligned(a.X, 16) && a.ldx % 4 == 0;
  pl.vec_y = aligned(a.Y, 4 * L) && a.ldy % L == 0;
  const size_t lds = (static_cast<size_t>(used) + (FL_MAX_CF + 1) * 4) * sizeof(float);
  if (L == 1) return launch_l<1>(a, pl, lds, s);
  if (L == 2) return launch_l<2>(a, pl, lds, s);
  return launch_l<4>(a, pl, lds, s);
}

}  // namespace lq
