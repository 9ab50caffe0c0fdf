// (Internal header: the kernel template, instantiated in fused_coltile_a.hip for fp32, in
// fused_coltile_b.hip for bf16 and in fused_coltile_c.hip for 5 to 8 dimension tables, so that the
// parts compile in parallel.)
//
// Join-computation stage (last line of Eq. 1) for wide linear operators: first-layer widths above one
// wavefront's worth of 16-byte pieces (256 fp32 / 512 bf16 columns), as in the paper's cardinality
// setting 2 where the operator's output shape grows to 2^11 (Q5 / Q6) -- as a linear operator or followed
// by a second layer of up to 16 outputs.
//
// The hidden row is cut into column tiles of 64 pieces.  A workgroup owns a batch of RB consecutive fact
// rows; its wavefronts share the tiles (wavefront w takes tiles w, w + NW, ..).  Within a tile the whole
// wavefront works on one fact row at a time: lane c owns piece c of the tile, so each projected row is
// fetched as one contiguous 1 KB run, the row's key and fact values are wavefront-uniform (lane reads),
// and gathers of four (two) rows travel together, software-pipelined across the batch.  A linear operator
// streams its tile of z straight out.  With a second layer every lane multiplies its columns by its
// rows of W_2, the lanes of the wavefront are summed per output, the row's partial result is parked in
// lane t and accumulates over the wavefront's tiles; the partial results of the wavefronts meet in LDS
// and the first wavefront adds them in a fixed order (deterministic) and stores the output rows.
#ifndef LQ_FUSED_COLTILE_H_
#define LQ_FUSED_COLTILE_H_
#include "fused_rowbatch_wide.h"

namespace lq {
namespace {

constexpr int CT_MAX_WAVES = 8;
constexpr int CT_THREADS = CT_MAX_WAVES * 64;

template <int K, int PG> struct CTGather { v4u p[PG][K]; };

// Rows whose gathers travel together: four when the registers allow it (two buffers of PG x K pieces next
// to the lane's weights), else two, else one; spilling costs more than a shorter pipeline.
constexpr int ct_rows_in_flight(int COLS, int K, int CFC, int L2P) {
  const int fixed = (4 * CFC + 1 + L2P) * COLS + 2 * L2P + 4 * CFC + 30;
  int pg = (L2P > 4 || K > 4) ? 2 : 4;
  while (pg > 1 && 8 * pg * K + fixed > 215) pg >>= 1;
  return pg;
}

template <int COLS, int CFC, int L2P> struct CTConsts {
  float wf[CFC > 0 ? CFC * 4 : 1][COLS];   // W_f rows x this lane's columns of the tile
  float b1[COLS];
  float w2[COLS][L2P];
};

template <typename T, int K, int PG>
__device__ __forceinline__ void ct_issue(const T* const (&pb)[K], const int64_t (&ldp)[K], bool active, int grp,
                                         const int (&fk)[K], CTGather<K, PG>& g) {
#pragma unroll
  for (int u = 0; u < PG; ++u)
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int j = __builtin_amdgcn_readlane(fk[k], PG * grp + u);
      g.p[u][k] = v4u{0u, 0u, 0u, 0u};
      if (active) g.p[u][k] = *reinterpret_cast<const v4u*>(pb[k] + static_cast<int64_t>(j) * ldp[k]);
    }
}

// T: element type of the model, the tables and the output.  K dimensions, CFC groups of four fact
// columns, NL layers (1 or 2), L2P outputs of the second layer rounded up to 1, 4 or 16.
template <typename T, int K, int CFC, int NL, int L2P>
__global__ __launch_bounds__(CT_THREADS) void fused_coltile_kernel(PredictArgs a, int tiles, int RB) {
  constexpr int COLS = Piece<T>::COLS;
  constexpr int TILE = 64 * COLS;
  constexpr int PG = ct_rows_in_flight(COLS, K, CFC, L2P);
  extern __shared__ float ct_red[];   // [NW][RB][L2P], second layer only
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, NW = blockDim.x >> 6;
  const int l1 = a.wout[0];
  const int l2 = NL == 2 ? a.wout[1] : 0;
  const bool x_vec = a.c_f == 4 * CFC && a.ldx % 4 == 0 && (reinterpret_cast<uintptr_t>(a.X) & (4 * sizeof(T) - 1)) == 0;
  const int NG = RB / PG;             // even: RB is a multiple of 8
  int64_t ldp[K];
#pragma unroll
  for (int k = 0; k < K; ++k) ldp[k] = a.ldp[k];

  CTConsts<COLS, CFC, L2P> cw;
  int loaded_tile = -1;
  const int64_t n_batches = (a.n + RB - 1) / RB;
  for (int64_t b = blockIdx.x; b < n_batches; b += gridDim.x) {
    const int64_t row0 = b * RB;
    WRow<K, CFC> r;
    {
      const int64_t row = row0 + lane;
      load_rows<T, K, CFC>(a, row < a.n ? row : a.n - 1, x_vec, r);   // lanes past the batch repeat valid rows
    }
    float ykeep[L2P];
#pragma unroll
    for (int o = 0; o < L2P; ++o) ykeep[o] = 0.f;
    if constexpr (NL == 2 && L2P == 16) {      // sixteen outputs accumulate in the wavefront's part of LDS (see below)
      for (int i = lane; i < RB * L2P; i += 64) ct_red[w * RB * L2P + i] = 0.f;
    }

    for (int tile = w; tile < tiles; tile += NW) {
      const int col = tile * TILE + COLS * lane;
      const bool active = col < l1;
      const int nvalid = min(COLS, max(0, l1 - col));          // columns of this lane's piece that exist
      // (linear models) a whole 16-byte piece of Y: aligned rows and no partial piece in this lane
      const bool y_piece = a.ldy % COLS == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0 && nvalid == COLS;
      if (tile != loaded_tile) {      // a wavefront with one tile keeps its weights for the whole launch
        loaded_tile = tile;
        const T* W0 = static_cast<const T*>(a.W[0]);
#pragma unroll
        for (int q = 0; q < CFC * 4; ++q)
#pragma unroll
          for (int v = 0; v < COLS; ++v)
            cw.wf[q][v] = (q < a.c_f && v < nvalid) ? Elem<T>::load(W0 + static_cast<int64_t>(q) * a.ldw[0] + col + v) : 0.f;
#pragma unroll
        for (int v = 0; v < COLS; ++v)
          cw.b1[v] = (a.bias[0] && v < nvalid) ? Elem<T>::load(static_cast<const T*>(a.bias[0]) + col + v) : 0.f;
#pragma unroll
        for (int o = 0; o < L2P; ++o) {
          const bool real = NL == 2 && o < l2;
#pragma unroll
          for (int v = 0; v < COLS; ++v)
            cw.w2[v][o] = (real && v < nvalid) ? Elem<T>::load(static_cast<const T*>(a.W[1]) + static_cast<int64_t>(col + v) * a.ldw[1] + o) : 0.f;
        }
      }
      const T* pb[K];
#pragma unroll
      for (int k = 0; k < K; ++k) pb[k] = static_cast<const T*>(a.P[k]) + (active ? col : 0);

      auto compute = [&](int grp, const CTGather<K, PG>& g) {
#pragma unroll
        for (int u = 0; u < PG; ++u) {
          const int t = PG * grp + u;
          float z[COLS];
#pragma unroll
          for (int v = 0; v < COLS; ++v) z[v] = cw.b1[v];
#pragma unroll
          for (int q = 0; q < CFC; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float xe = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r.x[q][e]), t));
#pragma unroll
              for (int v = 0; v < COLS; ++v) z[v] = fmaf(xe, cw.wf[q * 4 + e][v], z[v]);
            }
#pragma unroll
          for (int k = 0; k < K; ++k) Piece<T>::add(g.p[u][k], z);
          // a width that is not a multiple of COLS: the last piece of a row ends in the padding of the row stride,
          // whose contents are not ours; those elements count as zero
          if (l1 % COLS != 0) {
#pragma unroll
            for (int v = 0; v < COLS; ++v) z[v] = v < nvalid ? z[v] : 0.f;
          }
          if constexpr (NL == 1) {
            const int64_t row = row0 + t;
            if (a.accumulate_y && row < a.n && active) {
              const T* yo = static_cast<const T*>(a.Y) + row * a.ldy + col;
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
              T* yr = static_cast<T*>(a.Y) + row * a.ldy + col;
              if (y_piece) {
                __builtin_nontemporal_store(Piece<T>::pack(z), reinterpret_cast<v4u*>(yr));
              } else {                 // Y rows that are not 16-byte aligned, or a partial last piece
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
              for (int o = 0; o < L2P; ++o) y[o] = fmaf(h, cw.w2[v][o], y[o]);
            }
            if constexpr (L2P == 16) {
              // (one sum per output, six cross-lane steps each, made wide second layers arithmetic-bound)
              const float tot = group_reduce_scatter16<64>(y, lane);
              if (lane < 16) atomicAdd(&ct_red[(w * RB + t) * L2P + lane], tot);     // this wavefront's rows only
            } else {
#pragma unroll
              for (int o = 0; o < L2P; ++o) {
                const float tot = group_sum<64>(y[o]);
                if (lane == t) ykeep[o] += tot;
              }
            }
          }
        }
      };

      CTGather<K, PG> ga, gb;
      ct_issue<T, K, PG>(pb, ldp, active, 0, r.fk, ga);
#pragma unroll 1
      for (int grp = 0; grp < NG; grp += 2) {
        ct_issue<T, K, PG>(pb, ldp, active, grp + 1, r.fk, gb);
        compute(grp, ga);
        if (grp + 2 < NG) ct_issue<T, K, PG>(pb, ldp, active, grp + 2, r.fk, ga);
        compute(grp + 1, gb);
      }
    }

    if constexpr (NL == 2) {
      if (L2P != 16 && lane < RB) {
#pragma unroll
        for (int o = 0; o < L2P; ++o) ct_red[(w * RB + lane) * L2P + o] = ykeep[o];
      }
      __syncthreads();
      const int64_t row = row0 + lane;
      if (w == 0 && lane < RB && row < a.n) {
        T* yr = static_cast<T*>(a.Y) + row * a.ldy;
#pragma unroll
        for (int o = 0; o < L2P; ++o)
          if (o < l2) {
            float y = a.bias[1] ? Elem<T>::load(static_cast<const T*>(a.bias[1]) + o) : 0.f;
            for (int q = 0; q < NW; ++q) y += ct_red[(q * RB + lane) * L2P + o];
            Elem<T>::store(yr + o, y);
          }
      }
      __syncthreads();                // the next batch overwrites the partial results
    }
  }
}

template <typename T, int K, int CFC, int NL, int L2P>
int ct_launch(const PredictArgs& a, hipStream_t s) {
  constexpr int TILE = 64 * Piece<T>::COLS;
  const int tiles = (a.wout[0] + TILE - 1) / TILE;
  const int nw = std::min(tiles, CT_MAX_WAVES);
  // Rows per batch: enough batches to fill the compute units twice over when the fact table allows it.
  const int64_t want = 2LL * num_cus();
  int RB = 64;
  while (RB > 8 && (a.n + RB - 1) / RB < want) RB >>= 1;
  const int64_t batches = (a.n + RB - 1) / RB;
  const int64_t blocks = std::min<int64_t>(batches, 4LL * num_cus());
  const size_t lds = NL == 2 ? static_cast<size_t>(nw) * RB * L2P * sizeof(float) : 0;
  if (a.probe) return LQ_OK;
  hipLaunchKernelGGL((fused_coltile_kernel<T, K, CFC, NL, L2P>), dim3(static_cast<unsigned>(blocks)), dim3(nw * 64),
                     lds, s, a, tiles, RB);
  LQ_LAUNCH_CHECK("fused_coltile_kernel");
  return LQ_OK;
}

// MAXL2: the widest second layer this element type is instantiated for.
template <typename T, int K, int CFC, int MAXL2>
int ct_pick_layers(const PredictArgs& a, hipStream_t s) {
  if (a.n_layers == 1) return ct_launch<T, K, CFC, 1, 1>(a, s);
  const int l2 = a.wout[1];
  if (l2 > MAXL2) return -1;
  if constexpr (MAXL2 > 4) {
    if (l2 > 4) {
      // (bf16, eight columns per lane: with more than four fact columns the weights of sixteen outputs no longer fit
      // the registers, 32 to 160 bytes per lane would spill; such models take the layered form)
      if constexpr (sizeof(T) == 2 && CFC > 1) return -1;
      else return ct_launch<T, K, CFC, 2, 16>(a, s);
    }
  }
  if (l2 == 1) return ct_launch<T, K, CFC, 2, 1>(a, s);
  return ct_launch<T, K, CFC, 2, 4>(a, s);
}

template <typename T, int K, int MAXL2>
int ct_pick_cf(const PredictArgs& a, hipStream_t s) {
  if (a.c_f == 0) return ct_pick_layers<T, K, 0, MAXL2>(a, s);
  if (a.c_f <= 4) return ct_pick_layers<T, K, 1, MAXL2>(a, s);
  if (a.c_f <= 8) return ct_pick_layers<T, K, 2, MAXL2>(a, s);
  return -1;
}

template <typename T, int MAXL2>
int ct_pick_k(const PredictArgs& a, hipStream_t s) {
  switch (a.K) {
    case 1: return ct_pick_cf<T, 1, MAXL2>(a, s);
    case 2: return ct_pick_cf<T, 2, MAXL2>(a, s);
    case 3: return ct_pick_cf<T, 3, MAXL2>(a, s);
    case 4: return ct_pick_cf<T, 4, MAXL2>(a, s);
    default: return -1;
  }
}

// 5 to 8 dimensions: fp32, at most 4 fact columns, linear or one more layer of one output.
template <int K>
int ct_pick_many_dims(const PredictArgs& a, hipStream_t s) {
  if (a.c_f > 4 || (a.n_layers == 2 && a.wout[1] != 1)) return -1;
  if (a.c_f == 0) return a.n_layers == 1 ? ct_launch<float, K, 0, 1, 1>(a, s) : ct_launch<float, K, 0, 2, 1>(a, s);
  return a.n_layers == 1 ? ct_launch<float, K, 1, 1, 1>(a, s) : ct_launch<float, K, 1, 2, 1>(a, s);
}

// Shapes the column-tiled kernel takes, whatever the element type: one or two layers, all operands of
// one type, projected tables whose rows start 16 bytes apart.
inline bool ct_shape_ok(const PredictArgs& a, int cols) {
  if (a.n_layers > 2 || a.K < 1 || a.c_f > 8) return false;
  if (a.x_dtype != a.p_dtype || a.x_dtype != a.y_dtype) return false;
  // (any width: a row's last 16-byte piece may end in the padding of the row stride; a linear model's Y may have any alignment)
  for (int k = 0; k < a.K; ++k)
    if (!aligned(a.P[k], 16) || a.ldp[k] % cols) return false;
  return true;
}

}  // namespace
}  // namespace lq
#endif  // LQ_FUSED_COLTILE_H_
