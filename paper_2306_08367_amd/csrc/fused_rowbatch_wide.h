// (Internal header: the kernel template, instantiated in fused_rowbatch_wide_a.hip for fp32 with 8 / 16
// lanes per row, in fused_rowbatch_wide_b.hip for fp32 with 32 / 64, in fused_rowbatch_wide_c.hip for
// bf16 and in fused_rowbatch_wide_d.hip for 5 to 8 dimension tables, so that the parts compile in parallel.)
//
// Join-computation stage (last line of Eq. 1) as a linear operator or followed by a second layer of
// up to 16 outputs: the organisation of the width-64 kernel with a run-time pass loop, so that it
// covers 8 to 64 lanes per fact row, in fp32 (hidden widths 32 .. 256, 4 columns per lane) and in
// bf16 (hidden widths 64 .. 512, 8 columns per lane, fp32 arithmetic).
//
// A wavefront owns 64 consecutive fact rows at a time.  Their fact columns and keys are read once,
// coalesced (lane l holds row l).  With LPR lanes per row the wavefront is 64 / LPR lane groups; in
// pass t (0 .. LPR-1) group g works on fact row g LPR + t, lane c of the group owning the hidden
// columns of its 16-byte piece, so that a projected row (128 to 1024 bytes) is fetched by one group
// as one contiguous run.  The row's key and fact values reach the group through the cross-lane
// network (a lane read for 64 lanes per row, a permute otherwise).  Gathers are software-pipelined
// in groups of four (two, with many outputs or more than four dimensions) passes, across batches too.  A second layer is
// COLS x l_2 multiply-adds per lane and a sum over the lanes of the row per output (DPP adds); the
// results of pass t are parked in lane t of the group, so a batch ends with one store per row.
#ifndef LQ_FUSED_ROWBATCH_WIDE_H_
#define LQ_FUSED_ROWBATCH_WIDE_H_
#include "lq_common.h"

namespace lq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int RBW_THREADS = 256;

// What a 16-byte piece of a projected row holds.
template <typename T> struct Piece;
template <> struct Piece<float> {
  static constexpr int COLS = 4;
  static __device__ __forceinline__ void add(const v4u& raw, float (&z)[4]) {
#pragma unroll
    for (int v = 0; v < 4; ++v) z[v] += __uint_as_float(raw[v]);
  }
  static __device__ __forceinline__ v4u pack(const float (&z)[4]) {
    return v4u{__float_as_uint(z[0]), __float_as_uint(z[1]), __float_as_uint(z[2]), __float_as_uint(z[3])};
  }
};
template <> struct Piece<bf16_t> {
  static constexpr int COLS = 8;
  static __device__ __forceinline__ void add(const v4u& raw, float (&z)[8]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      z[2 * q] += __uint_as_float(raw[q] << 16);
      z[2 * q + 1] += __uint_as_float(raw[q] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ v4u pack(const float (&z)[8]) {
    v4u o;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      o[q] = f32x2_to_bf16x2(z[2 * q], z[2 * q + 1]);
    return o;
  }
};

template <int CTRL> __device__ __forceinline__ float dppw(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over the LPR (8 .. 64) lanes of a group, result in every lane.
template <int LPR> __device__ __forceinline__ float group_sum(float y) {
  y += dppw<0xB1>(y);                  // quad_perm [1,0,3,2]
  y += dppw<0x4E>(y);                  // quad_perm [2,3,0,1]
  y += dppw<0x141>(y);                 // row_half_mirror
  if (LPR >= 16) y += dppw<0x140>(y);  // row_mirror
  if (LPR >= 32) y += __shfl_xor(y, 16, 64);
  if (LPR >= 64) y += __shfl_xor(y, 32, 64);
  return y;
}
// Sums of y[0..15] over the 16 lanes of a row of the cross-lane network, scattered: lane L ends with the total of
// output L & 15.  Each step halves the outputs a lane still carries (it keeps the half its own lane bit selects and adds
// what its partner sends of that half): 8 + 4 + 2 + 1 exchanges instead of four per output.  The mirror steps come
// first: they also flip the lower lane bits, which is harmless only while those have not selected anything yet.
__device__ __forceinline__ float reduce_scatter16_row(const float (&y)[16], int lane) {
  const bool b3 = (lane & 8) != 0, b2 = (lane & 4) != 0, b1 = (lane & 2) != 0, b0 = (lane & 1) != 0;
  float a8[8], a4[4], a2[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) a8[i] = (b3 ? y[8 + i] : y[i]) + dppw<0x140>(b3 ? y[i] : y[8 + i]);          // row_mirror: i <-> 15 - i
#pragma unroll
  for (int i = 0; i < 4; ++i) a4[i] = (b2 ? a8[4 + i] : a8[i]) + dppw<0x141>(b2 ? a8[i] : a8[4 + i]);      // row_half_mirror: i <-> 7 - i
#pragma unroll
  for (int i = 0; i < 2; ++i) a2[i] = (b1 ? a4[2 + i] : a4[i]) + dppw<0x4E>(b1 ? a4[i] : a4[2 + i]);       // quad_perm [2,3,0,1]
  return (b0 ? a2[1] : a2[0]) + dppw<0xB1>(b0 ? a2[0] : a2[1]);                                            // quad_perm [1,0,3,2]
}
// The scattered form over a group of LPR = 16, 32 or 64 lanes: every lane L of the group ends with output L & 15.
template <int LPR> __device__ __forceinline__ float group_reduce_scatter16(const float (&y)[16], int lane) {
  static_assert(LPR >= 16, "a group of at least one row of 16 lanes");
  float r = reduce_scatter16_row(y, lane);
  if (LPR >= 32) r += __shfl_xor(r, 16, 64);
  if (LPR >= 64) r += __shfl_xor(r, 32, 64);
  return r;
}
// Value that lane (group base + t) holds, for every lane of the group.
template <int LPR> __device__ __forceinline__ int from_lane(int v, int t, int group_base) {
  if constexpr (LPR == 64) return __builtin_amdgcn_readlane(v, t);
  else return __shfl(v, group_base | t, 64);
}

// Per-batch registers: lane l holds fact row (batch * 64 + l); fact columns as fp32.
template <int K, int CFC> struct WRow {
  int fk[K];
  v4f x[CFC > 0 ? CFC : 1];
};
template <int K, int PG> struct WGather { v4u p[PG][K]; };

// x_vec: the row's fact columns are whole, aligned groups of four; otherwise they are read
// one by one and the groups padded with zeros (the matching rows of W_f are zero as well).
template <typename T, int K, int CFC>
__device__ __forceinline__ void load_rows(const PredictArgs& a, int64_t rr, bool x_vec, WRow<K, CFC>& r) {
#pragma unroll
  for (int k = 0; k < K; ++k) r.fk[k] = __builtin_nontemporal_load(a.fk[k] + rr);
  const T* xr = static_cast<const T*>(a.X) + rr * a.ldx;
  if (x_vec) {
#pragma unroll
    for (int q = 0; q < CFC; ++q) {
      if constexpr (sizeof(T) == 4) {
        r.x[q] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(xr) + q);
      } else {                                    // four bf16 values in 8 bytes
        const v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(xr) + q);
        r.x[q] = v4f{__uint_as_float(t[0] << 16), __uint_as_float(t[0] & 0xffff0000u),
                     __uint_as_float(t[1] << 16), __uint_as_float(t[1] & 0xffff0000u)};
      }
    }
  } else {
#pragma unroll
    for (int q = 0; q < CFC; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) r.x[q][e] = 4 * q + e < a.c_f ? Elem<T>::load(xr + 4 * q + e) : 0.f;
  }
}

// Keys become byte offsets of their rows once per batch (one 32-bit product per key: the host has
// checked that every projected table is smaller than 4 GiB), so that a gather costs a broadcast and one
// add on top of its load instead of a 64-bit multiply-add.
template <typename T, int K, int CFC>
__device__ __forceinline__ void keys_to_offsets(const PredictArgs& a, WRow<K, CFC>& r) {
#pragma unroll
  for (int k = 0; k < K; ++k)
    r.fk[k] = static_cast<int>(static_cast<uint32_t>(r.fk[k]) * (static_cast<uint32_t>(a.ldp[k]) * static_cast<uint32_t>(sizeof(T))));
}

// Gathers of passes PG grp .. PG grp + PG - 1.
template <typename T, int LPR, int K, int CFC, int PG>
__device__ __forceinline__ void issue_group(const PredictArgs& a, int c, bool active, int group_base, int grp,
                                            const WRow<K, CFC>& r, WGather<K, PG>& g) {
#pragma unroll
  for (int u = 0; u < PG; ++u)
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const uint32_t at = static_cast<uint32_t>(from_lane<LPR>(r.fk[k], PG * grp + u, group_base)) + 16u * static_cast<uint32_t>(c);
      g.p[u][k] = v4u{0u, 0u, 0u, 0u};
      if (active) g.p[u][k] = *reinterpret_cast<const v4u*>(static_cast<const char*>(a.P[k]) + at);
    }
}

// L2P: outputs of the second layer rounded up to 1, 4, 8 or 16 (weights of the padding are zero).
template <int COLS, int CFC, int L2P> struct WConsts {
  float wf[CFC > 0 ? CFC * 4 : 1][COLS];   // W_f rows x this lane's columns
  float b1[COLS];
  float w2[COLS][L2P];
  float b2[L2P];
};

template <typename T, int LPR, int K, int CFC, int NL, int L2P, int PG>
__device__ __forceinline__ void compute_group(const PredictArgs& a, int c, bool active, int nvalid, bool y_piece, int group_base,
                                              int grp, int64_t row0, const WRow<K, CFC>& r, const WGather<K, PG>& g,
                                              const WConsts<Piece<T>::COLS, CFC, L2P>& w, float (&ykeep)[L2P]) {
  constexpr int COLS = Piece<T>::COLS;
#pragma unroll
  for (int u = 0; u < PG; ++u) {
    const int t = PG * grp + u;
    float z[COLS];
#pragma unroll
    for (int v = 0; v < COLS; ++v) z[v] = w.b1[v];
#pragma unroll
    for (int q = 0; q < CFC; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float xe = __int_as_float(from_lane<LPR>(__float_as_int(r.x[q][e]), t, group_base));
#pragma unroll
        for (int v = 0; v < COLS; ++v) z[v] = fmaf(xe, w.wf[q * 4 + e][v], z[v]);
      }
#pragma unroll
    for (int k = 0; k < K; ++k) Piece<T>::add(g.p[u][k], z);
    // a hidden width that is not a multiple of COLS: the last piece of a row ends in the padding of the row
    // stride, whose contents are not ours; those elements count as zero
    if (a.wout[0] % COLS != 0) {
#pragma unroll
      for (int v = 0; v < COLS; ++v) z[v] = v < nvalid ? z[v] : 0.f;
    }
    if constexpr (NL == 1) {
      const int64_t row = row0 + group_base + t;
      if (a.accumulate_y && row < a.n && active) {
        const T* yo = static_cast<const T*>(a.Y) + row * a.ldy + COLS * c;
        if (y_piece) {
          Piece<T>::add(*reinterpret_cast<const v4u*>(yo), z);
        } else {
#pragma unroll
          for (int v = 0; v < COLS; ++v)
            if (v < nvalid) z[v] += Elem<T>::load(yo + v);
        }
      }
      if (a.relu_linear) {
#pragma unroll
        for (int v = 0; v < COLS; ++v) z[v] = fmaxf(z[v], 0.f);
      }
      if (row < a.n && active) {
        T* yr = static_cast<T*>(a.Y) + row * a.ldy + COLS * c;
        if (y_piece) {
          __builtin_nontemporal_store(Piece<T>::pack(z), reinterpret_cast<v4u*>(yr));
        } else {                       // Y rows that are not 16-byte aligned, or a partial last piece
#pragma unroll
          for (int v = 0; v < COLS; ++v)
            if (v < nvalid) Elem<T>::store(yr + v, z[v]);
        }
      }
    } else {
      float y[L2P];
#pragma unroll
      for (int o = 0; o < L2P; ++o) y[o] = 0.f;
#pragma unroll
      for (int v = 0; v < COLS; ++v) {
        const float h = fmaxf(z[v], 0.f);
#pragma unroll
        for (int o = 0; o < L2P; ++o) y[o] = fmaf(h, w.w2[v][o], y[o]);
      }
#pragma unroll
      for (int o = 0; o < L2P; ++o) {
        const float tot = group_sum<LPR>(y[o]);
        if (c == t) ykeep[o] = tot;
      }
    }
  }
}

// Three wavefronts per SIMD leave 170 registers each; the double-buffered gathers of many
// dimensions plus many fact columns, or the weights of a wide second layer, need more, and two per
// SIMD is faster than spilling.
constexpr int waves_per_simd(int COLS, int K, int CFC, int L2P) {
  return (L2P > 4 || (K > 4 ? 16 : 32) * K + (24 * CFC + 6 * L2P) * (COLS / 4) > 106) ? 2 : 3;
}

// T: element type of the model, the tables and the output.  LPR lanes per row (l_1 = COLS x LPR),
// K dimensions, CFC groups of four fact columns, NL layers, L2P padded outputs of the second layer.
template <typename T, int LPR, int K, int CFC, int NL, int L2P>
__global__ __launch_bounds__(RBW_THREADS)
__attribute__((amdgpu_waves_per_eu(waves_per_simd(Piece<T>::COLS, K, CFC, L2P), waves_per_simd(Piece<T>::COLS, K, CFC, L2P))))
void fused_rowbatch_wide_kernel(PredictArgs a) {
  constexpr int COLS = Piece<T>::COLS;
  constexpr int PG = (L2P > 4 || K > 4) ? 2 : 4;    // passes whose gathers travel together
  constexpr int NG = LPR / PG;           // such groups per batch (even)
  const int lane = threadIdx.x & 63, c = lane & (LPR - 1), group_base = lane & ~(LPR - 1);
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (RBW_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (RBW_THREADS / 64);
  const int64_t nb = (a.n + 63) / 64;
  if (wave >= nb) return;
  const int l2 = NL == 2 ? a.wout[1] : 0;
  const bool active = COLS * c < a.wout[0];   // lanes beyond the hidden width idle (widths that are not COLS x a power of two)
  const int nvalid = min(COLS, max(0, a.wout[0] - COLS * c));      // columns of this lane's piece that exist
  // (linear models) whole 16-byte pieces of Y: aligned rows and no partial piece in this lane
  const bool y_piece = a.ldy % COLS == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0 && nvalid == COLS;
  const bool x_vec = a.c_f == 4 * CFC && a.ldx % 4 == 0 && (reinterpret_cast<uintptr_t>(a.X) & (4 * sizeof(T) - 1)) == 0;
  const bool y_vec = l2 % 4 == 0 && a.ldy % 4 == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0;

  WConsts<COLS, CFC, L2P> w;
  {
    const T* W0 = static_cast<const T*>(a.W[0]);
#pragma unroll
    for (int q = 0; q < CFC * 4; ++q)
#pragma unroll
      for (int v = 0; v < COLS; ++v)
        w.wf[q][v] = (q < a.c_f && v < nvalid) ? Elem<T>::load(W0 + static_cast<int64_t>(q) * a.ldw[0] + COLS * c + v) : 0.f;
#pragma unroll
    for (int v = 0; v < COLS; ++v)
      w.b1[v] = (a.bias[0] && v < nvalid) ? Elem<T>::load(static_cast<const T*>(a.bias[0]) + COLS * c + v) : 0.f;
#pragma unroll
    for (int o = 0; o < L2P; ++o) {
      const bool real = NL == 2 && o < l2;
#pragma unroll
      for (int v = 0; v < COLS; ++v)
        w.w2[v][o] = (real && v < nvalid) ? Elem<T>::load(static_cast<const T*>(a.W[1]) + static_cast<int64_t>(COLS * c + v) * a.ldw[1] + o) : 0.f;
      w.b2[o] = (NL == 2 && o < l2 && a.bias[1]) ? Elem<T>::load(static_cast<const T*>(a.bias[1]) + o) : 0.f;
    }
  }

  int64_t b = wave;
  int64_t row = b * 64 + lane;
  WRow<K, CFC> cur, nxt;
  load_rows<T, K, CFC>(a, row < a.n ? row : a.n - 1, x_vec, cur);
  keys_to_offsets<T, K, CFC>(a, cur);
  WGather<K, PG> ga, gb;
  issue_group<T, LPR, K, CFC, PG>(a, c, active, group_base, 0, cur, ga);
  for (;;) {
    const int64_t bn = b + nwaves;
    const bool more = bn < nb;
    const int64_t rown = bn * 64 + lane;
    load_rows<T, K, CFC>(a, (more && rown < a.n) ? rown : a.n - 1, x_vec, nxt);
    float yk[L2P];
#pragma unroll
    for (int o = 0; o < L2P; ++o) yk[o] = 0.f;
    const int64_t row0 = b * 64;
#pragma unroll 1
    for (int grp = 0; grp < NG; grp += 2) {
      issue_group<T, LPR, K, CFC, PG>(a, c, active, group_base, grp + 1, cur, gb);
      compute_group<T, LPR, K, CFC, NL, L2P, PG>(a, c, active, nvalid, y_piece, group_base, grp, row0, cur, ga, w, yk);
      if (grp + 2 < NG) issue_group<T, LPR, K, CFC, PG>(a, c, active, group_base, grp + 2, cur, ga);
      else {                                       // first group of the next batch (valid rows repeated at the end)
        keys_to_offsets<T, K, CFC>(a, nxt);
        issue_group<T, LPR, K, CFC, PG>(a, c, active, group_base, 0, nxt, ga);
      }
      compute_group<T, LPR, K, CFC, NL, L2P, PG>(a, c, active, nvalid, y_piece, group_base, grp + 1, row0, cur, gb, w, yk);
    }
    if constexpr (NL == 2) {
      if (row < a.n) {
        T* yr = static_cast<T*>(a.Y) + row * a.ldy;
        if (L2P >= 4 && y_vec) {             // whole pieces of the output row
#pragma unroll
          for (int q = 0; q < L2P / 4; ++q)
            if (4 * q < l2) {
              const float o4[4] = {yk[4 * q] + w.b2[4 * q], yk[4 * q + 1] + w.b2[4 * q + 1],
                                   yk[4 * q + 2] + w.b2[4 * q + 2], yk[4 * q + 3] + w.b2[4 * q + 3]};
              if constexpr (sizeof(T) == 4) {
                *reinterpret_cast<v4f*>(yr + 4 * q) = v4f{o4[0], o4[1], o4[2], o4[3]};
              } else {
                *reinterpret_cast<v2u*>(yr + 4 * q) =
                    v2u{f32x2_to_bf16x2(o4[0], o4[1]), f32x2_to_bf16x2(o4[2], o4[3])};
              }
            }
        } else {
#pragma unroll
          for (int o = 0; o < L2P; ++o)
            if (o < l2) Elem<T>::store(yr + o, yk[o] + w.b2[o]);
        }
      }
    }
    if (!more) break;
    b = bn;
    row = rown;
    cur = nxt;
  }
}

template <typename T, int LPR, int K, int CFC, int NL, int L2P>
int launch_inst(const PredictArgs& a, hipStream_t s) {
  const int64_t nb = (a.n + 63) / 64;
  const int64_t blocks = std::min<int64_t>((nb + 3) / 4, static_cast<int64_t>(num_cus()) * waves_per_simd(Piece<T>::COLS, K, CFC, L2P));
  if (a.probe) return LQ_OK;
  hipLaunchKernelGGL((fused_rowbatch_wide_kernel<T, LPR, K, CFC, NL, L2P>), dim3(static_cast<unsigned>(blocks)),
                     dim3(RBW_THREADS), 0, s, a);
  LQ_LAUNCH_CHECK("fused_rowbatch_wide_kernel");
  return LQ_OK;
}

// MAXL2: the widest second layer this element type is instantiated for.
template <typename T, int LPR, int K, int CFC, int MAXL2>
int pick_layers(const PredictArgs& a, hipStream_t s) {
  if (a.n_layers == 1) return launch_inst<T, LPR, K, CFC, 1, 1>(a, s);
  const int l2 = a.wout[1];
  if (l2 > MAXL2) return -1;
  if constexpr (MAXL2 > 4) {
    if (l2 > 8) return launch_inst<T, LPR, K, CFC, 2, 16>(a, s);
    if (l2 > 4) return launch_inst<T, LPR, K, CFC, 2, 8>(a, s);
  }
  if (l2 == 1) return launch_inst<T, LPR, K, CFC, 2, 1>(a, s);
  return launch_inst<T, LPR, K, CFC, 2, 4>(a, s);
}

template <typename T, int LPR, int K, int MAXL2>
int pick_cf(const PredictArgs& a, hipStream_t s) {
  if (a.c_f == 0) return pick_layers<T, LPR, K, 0, MAXL2>(a, s);
  if (a.c_f <= 4) return pick_layers<T, LPR, K, 1, MAXL2>(a, s);
  if (a.c_f <= 8) return pick_layers<T, LPR, K, 2, MAXL2>(a, s);
  if constexpr (sizeof(T) == 4) {            // (bf16 lanes hold twice the columns: no room for more weights)
    if (a.c_f <= 16 && K <= 3) return pick_layers<T, LPR, K, 4, MAXL2 < 8 ? MAXL2 : 8>(a, s);
  }
  return -1;
}

// 5 to 8 dimensions: fp32, at most 4 fact columns, linear or one more layer of one output.
template <int LPR, int K>
int pick_many_dims(const PredictArgs& a, hipStream_t s) {
  if (a.c_f > 4 || (a.n_layers == 2 && a.wout[1] != 1)) return -1;
  if (a.c_f == 0) return a.n_layers == 1 ? launch_inst<float, LPR, K, 0, 1, 1>(a, s) : launch_inst<float, LPR, K, 0, 2, 1>(a, s);
  return a.n_layers == 1 ? launch_inst<float, LPR, K, 1, 1, 1>(a, s) : launch_inst<float, LPR, K, 1, 2, 1>(a, s);
}
template <int LPR>
int pick_k_many(const PredictArgs& a, hipStream_t s) {
  switch (a.K) {
    case 5: return pick_many_dims<LPR, 5>(a, s);
    case 6: return pick_many_dims<LPR, 6>(a, s);
    case 7: return pick_many_dims<LPR, 7>(a, s);
    case 8: return pick_many_dims<LPR, 8>(a, s);
    default: return -1;
  }
}

template <typename T, int LPR, int MAXL2>
int pick_k(const PredictArgs& a, hipStream_t s) {
  switch (a.K) {
    case 1: return pick_cf<T, LPR, 1, MAXL2>(a, s);
    case 2: return pick_cf<T, LPR, 2, MAXL2>(a, s);
    case 3: return pick_cf<T, LPR, 3, MAXL2>(a, s);
    case 4: return pick_cf<T, LPR, 4, MAXL2>(a, s);
    default: return -1;
  }
}

}  // namespace
}  // namespace lq
#endif  // LQ_FUSED_ROWBATCH_WIDE_H_
