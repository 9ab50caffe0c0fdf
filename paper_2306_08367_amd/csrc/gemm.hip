// Dense C = act(A * B + bias) on the matrix cores, fp32 accumulate.
//
// Used for the pre-fusion products P_k = D_k * (rows of L owned by dimension k) (underlined terms
// of Eq. 1) and for the layer-by-layer model evaluation of the non-fused pipeline (T * L, second
// line of Eq. 1).  Two kernels:
//   gemm_tiled_kernel  - 128 x BN tiles (BN = 64 or 128) staged through LDS, 4 wavefronts in a
//                        2 x 2 arrangement, each owning 64 x BN/2 as 32x32 MFMA accumulators.
//                        fp32 inputs use the 32x32x2 f32 MFMA; bf16 inputs stay bf16 in LDS and
//                        use the 32x32x16 bf16 MFMA.  The next k-tile is fetched into registers
//                        while the current one is multiplied.
//   gemm_rowsplit_kernel - fp32, N <= 8, 32 <= K: the shape of projecting a wide dimension table
//                        onto a handful of outputs, bound by reading A once.  The lanes of a
//                        wavefront read A as contiguous 16-byte pieces (a row is split over 8..64
//                        neighbouring lanes), multiply with the weights held in LDS and sum over
//                        the lanes of a row with DPP adds: no matrix cores, every load a full
//                        coalesced run.
//   gemm_skinny_kernel - N <= 16 (linear models with a handful of outputs).  Bandwidth-shaped:
//                        no LDS, every wavefront streams 16 rows of A at a time straight into
//                        16x16 MFMA operands; B is tiny and comes from cache.
#include "lq_common.h"

namespace lq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GemmArgs {
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  void* C; int64_t ldc;
  const void* bias;
  int64_t M; int32_t N; int32_t Kd;
  int32_t relu;
  int32_t a_vec_ok, b_vec_ok;   // 16-byte loads of A / B rows are legal
  int32_t tiles_n;
};

// Up to LQ_MAX_DIMS independent products of the same type in one launch (the projections of all
// dimension tables): workgroup b works on problem p where first_tile[p] <= b < first_tile[p + 1].
struct GemmBatch {
  GemmArgs g[LQ_MAX_DIMS];
  int32_t first_tile[LQ_MAX_DIMS + 1];
  int32_t count;
};

// ------------------------------------------------------------------ tiled --------------

constexpr int BM = 128;
constexpr int TILED_THREADS = 256;

template <typename T> struct Tile;
template <> struct Tile<float> {
  static constexpr int BK = 32;        // k per LDS tile
  static constexpr int VEC = 4;        // elements per 16-byte chunk
};
template <> struct Tile<bf16_t> {
  static constexpr int BK = 64;
  static constexpr int VEC = 8;
};

struct __attribute__((packed, aligned(4))) Words4 { unsigned int x, y, z, w; };

// 16 bytes starting at p, of which only the first `valid` elements exist (others read as zero).
template <typename T>
__device__ __forceinline__ v4u load_chunk(const T* p, int valid, bool vec_ok) {
  constexpr int VEC = Tile<T>::VEC;
  if (valid >= VEC && vec_ok) return *reinterpret_cast<const v4u*>(p);
  if constexpr (sizeof(T) == 4) {
    // Rows whose stride is not a multiple of four floats (a table with 683 columns): still one 16-byte
    // load, declared with the 4-byte alignment the pointer has.
    if (valid >= VEC) {
      const Words4 t = *reinterpret_cast<const Words4*>(p);
      return v4u{t.x, t.y, t.z, t.w};
    }
  }
  v4u r = {0u, 0u, 0u, 0u};
  if (valid <= 0) return r;
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (q < valid) r[q] = reinterpret_cast<const unsigned int*>(p)[q];
  } else {
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (q < valid) r[q >> 1] |= static_cast<unsigned int>(p[q]) << (16 * (q & 1));
  }
  return r;
}

template <typename TA, typename TC, int BN>
__global__ __launch_bounds__(TILED_THREADS) void gemm_tiled_kernel(GemmBatch batch) {
  int problem = 0;
  while (problem + 1 < batch.count && static_cast<int32_t>(blockIdx.x) >= batch.first_tile[problem + 1]) ++problem;
  const GemmArgs g = batch.g[problem];
  const int64_t tile = static_cast<int64_t>(blockIdx.x) - batch.first_tile[problem];
  constexpr int BK = Tile<TA>::BK, VEC = Tile<TA>::VEC;
  constexpr bool F32 = sizeof(TA) == 4;
  constexpr int WN = BN / 2;              // columns per wavefront
  constexpr int TN = WN / 32;             // 32-wide MFMA tiles per wavefront along n (1 or 2)
  constexpr int A_CHUNKS = BM * BK / VEC / TILED_THREADS;   // 16-byte chunks per thread
  constexpr int B_CHUNKS = BK * BN / VEC / TILED_THREADS;
  constexpr int A_CPR = BK / VEC;         // chunks per A row
  constexpr int B_CPR = BN / VEC;         // chunks per B row
  // fp32: k-major tiles  As[k][m], Bs[k][n] (one word per MFMA operand read).
  // bf16: As[m][k], Bs[n][k] with k contiguous (eight consecutive k per MFMA operand read).
  constexpr int PADF = 4, PADH = 8;
  constexpr int A_WORDS = F32 ? BK * (BM + PADF) : BM * (BK + PADH) / 2;
  constexpr int B_WORDS = F32 ? BK * (BN + PADF) : BN * (BK + PADH) / 2;
  __shared__ __align__(16) unsigned int smemA[A_WORDS];
  __shared__ __align__(16) unsigned int smemB[B_WORDS];

  const TA* __restrict__ A = static_cast<const TA*>(g.A);
  const TA* __restrict__ B = static_cast<const TA*>(g.B);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t tile_m = tile / g.tiles_n;
  const int tile_n = static_cast<int>(tile % g.tiles_n);
  const int64_t m0 = tile_m * BM;
  const int n0 = tile_n * BN;

  v16f acc[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  v4u ra[A_CHUNKS], rb[B_CHUNKS];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int c = 0; c < A_CHUNKS; ++c) {
      const int id = tid + c * TILED_THREADS;
      const int r = id / A_CPR, kc = (id % A_CPR) * VEC;
      const int64_t row = min(m0 + r, g.M - 1);            // rows past the end repeat the last row
      ra[c] = load_chunk<TA>(A + row * g.lda + k0 + kc, g.Kd - (k0 + kc), g.a_vec_ok);
    }
#pragma unroll
    for (int c = 0; c < B_CHUNKS; ++c) {
      const int id = tid + c * TILED_THREADS;
      const int kk = id / B_CPR, nc = (id % B_CPR) * VEC;
      const int k = k0 + kk;
      rb[c] = load_chunk<TA>(B + static_cast<int64_t>(min(k, g.Kd - 1)) * g.ldb + n0 + nc,
                             k < g.Kd ? g.N - (n0 + nc) : 0, g.b_vec_ok);
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int c = 0; c < A_CHUNKS; ++c) {
      const int id = tid + c * TILED_THREADS;
      const int r = id / A_CPR, kc = (id % A_CPR) * VEC;
      if constexpr (F32) {
#pragma unroll
        for (int q = 0; q < 4; ++q) smemA[(kc + q) * (BM + PADF) + r] = ra[c][q];
      } else {
        *reinterpret_cast<v4u*>(&smemA[(r * (BK + PADH) + kc) / 2]) = ra[c];
      }
    }
#pragma unroll
    for (int c = 0; c < B_CHUNKS; ++c) {
      const int id = tid + c * TILED_THREADS;
      const int kk = id / B_CPR, nc = (id % B_CPR) * VEC;
      if constexpr (F32) {
        *reinterpret_cast<v4u*>(&smemB[kk * (BN + PADF) + nc]) = rb[c];
      } else {
        unsigned short* sb = reinterpret_cast<unsigned short*>(smemB);
#pragma unroll
        for (int q = 0; q < 8; ++q)
          sb[(nc + q) * (BK + PADH) + kk] = static_cast<unsigned short>(rb[c][q >> 1] >> (16 * (q & 1)));
      }
    }
  };

  fetch(0);
  for (int k0 = 0; k0 < g.Kd; k0 += BK) {
    __syncthreads();          // previous tile fully consumed
    stage();
    __syncthreads();
    if (k0 + BK < g.Kd) fetch(k0 + BK);
    if constexpr (F32) {
      const float* As = reinterpret_cast<const float*>(smemA);
      const float* Bs = reinterpret_cast<const float*>(smemB);
#pragma unroll 4
      for (int kk = 0; kk < BK; kk += 2) {
        const int k = kk + (lane >> 5);
        float a[2], b[TN];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = As[k * (BM + PADF) + wm * 64 + i * 32 + (lane & 31)];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = Bs[k * (BN + PADF) + wn * WN + j * 32 + (lane & 31)];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        const int k = kk + 8 * (lane >> 5);
        v4u a[2], b[TN];
#pragma unroll
        for (int i = 0; i < 2; ++i)
          a[i] = *reinterpret_cast<const v4u*>(&smemA[((wm * 64 + i * 32 + (lane & 31)) * (BK + PADH) + k) / 2]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          b[j] = *reinterpret_cast<const v4u*>(&smemB[((wn * WN + j * 32 + (lane & 31)) * (BK + PADH) + k) / 2]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                                __builtin_bit_cast(bf16x8, b[j]), acc[i][j], 0, 0, 0);
      }
    }
  }

  // 32x32 accumulator: register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
  TC* __restrict__ C = static_cast<TC*>(g.C);
  const TA* bias = static_cast<const TA*>(g.bias);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * WN + j * 32 + (lane & 31);
    if (col >= g.N) continue;
    const float bv = bias ? Elem<TA>::load(bias + col) : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row >= g.M) continue;
        float x = acc[i][j][v] + bv;
        if (g.relu) x = fmaxf(x, 0.f);
        Elem<TC>::store(C + row * g.ldc + col, x);
      }
  }
}

// ------------------------------------------------------------------ skinny -------------

constexpr int SKINNY_THREADS = 256;

// N <= 16.  A wavefront takes 16 rows per pass; lane (g = lane / 16, i = lane % 16) loads 16-byte
// pieces of row i at k = kc + VEC*g and feeds them element by element as the K-slices of 16x16
// MFMAs whose B operand holds the matching rows of the weight matrix (which rows of k a slot
// means is irrelevant as long as A and B agree, and they are built from the same index).
template <typename TA, typename TC>
__global__ __launch_bounds__(SKINNY_THREADS) void gemm_skinny_kernel(GemmArgs g) {
  constexpr int VEC = Tile<TA>::VEC;
  constexpr bool F32 = sizeof(TA) == 4;
  constexpr int KSTEP = 4 * VEC;             // k covered by one 16-byte load per lane
  const TA* __restrict__ A = static_cast<const TA*>(g.A);
  const TA* __restrict__ B = static_cast<const TA*>(g.B);
  const int lane = threadIdx.x & 63, grp = lane >> 4, i = lane & 15;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (SKINNY_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (SKINNY_THREADS / 64);
  const int64_t npass = (g.M + 15) / 16;
  const float bv = (g.bias && i < g.N) ? Elem<TA>::load(static_cast<const TA*>(g.bias) + i) : 0.f;

  for (int64_t pass = wave; pass < npass; pass += nwaves) {
    const int64_t row = min(pass * 16 + i, g.M - 1);
    const TA* ar = A + row * g.lda;
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    for (int kc = 0; kc < g.Kd; kc += KSTEP) {
      const int k = kc + VEC * grp;
      const v4u a = load_chunk<TA>(ar + k, g.Kd - k, g.a_vec_ok);
      // B operand: lane (grp, n = i) needs W[k + t][n] for t = 0..VEC-1
      if constexpr (F32) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float b = (k + t < g.Kd && i < g.N) ? B[static_cast<int64_t>(k + t) * g.ldb + i] : 0.f;
          acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[t]), b, acc, 0, 0, 0);
        }
      } else {
        v4u b = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int t = 0; t < 8; ++t)
          if (k + t < g.Kd && i < g.N)
            b[t >> 1] |= static_cast<unsigned int>(B[static_cast<int64_t>(k + t) * g.ldb + i]) << (16 * (t & 1));
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                      acc, 0, 0, 0);
      }
    }
    // register v of lane (grp, n) is row 4*grp + v of the pass, column n
    if (i < g.N) {
      TC* __restrict__ C = static_cast<TC*>(g.C);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t r = pass * 16 + 4 * grp + v;
        if (r >= g.M) continue;
        float x = acc[v] + bv;
        if (g.relu) x = fmaxf(x, 0.f);
        Elem<TC>::store(C + r * g.ldc + i, x);
      }
    }
  }
}

// All problems of the batch share N (hence the tile width) and the element types.
template <typename TA, typename TC>
int launch_tiled_batch(GemmBatch& b, hipStream_t s) {
  const bool wide = b.g[0].N > 64;
  const int bn = wide ? 128 : 64;
  int64_t blocks = 0;
  for (int p = 0; p < b.count; ++p) {
    GemmArgs& g = b.g[p];
    g.a_vec_ok = aligned(g.A, 16) && (g.lda * sizeof(TA)) % 16 == 0;
    g.b_vec_ok = aligned(g.B, 16) && (g.ldb * sizeof(TA)) % 16 == 0;
    g.tiles_n = (g.N + bn - 1) / bn;
    b.first_tile[p] = static_cast<int32_t>(blocks);
    blocks += (g.M + BM - 1) / BM * g.tiles_n;
    if (blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "gemm: %lld tiles exceed one grid", (long long)blocks);
  }
  b.first_tile[b.count] = static_cast<int32_t>(blocks);
  if (blocks == 0) return LQ_OK;
  if (wide)
    hipLaunchKernelGGL((gemm_tiled_kernel<TA, TC, 128>), dim3(static_cast<unsigned>(blocks)), dim3(TILED_THREADS), 0, s, b);
  else
    hipLaunchKernelGGL((gemm_tiled_kernel<TA, TC, 64>), dim3(static_cast<unsigned>(blocks)), dim3(TILED_THREADS), 0, s, b);
  LQ_LAUNCH_CHECK("gemm_tiled_kernel");
  return LQ_OK;
}

template <typename TA, typename TC>
int launch_typed(GemmArgs g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return LQ_OK;
  const size_t es = sizeof(TA);
  constexpr int VEC = Tile<TA>::VEC;
  g.a_vec_ok = aligned(g.A, 16) && (g.lda * es) % 16 == 0;
  g.b_vec_ok = aligned(g.B, 16) && (g.ldb * es) % 16 == 0;
  (void)VEC;
  if (g.N <= 16) {
    const int64_t npass = (g.M + 15) / 16;
    const int64_t blocks = std::min<int64_t>((npass + 3) / 4, static_cast<int64_t>(num_cus()) * 8);
    hipLaunchKernelGGL((gemm_skinny_kernel<TA, TC>), dim3(static_cast<unsigned>(blocks)), dim3(SKINNY_THREADS),
                       0, s, g);
    LQ_LAUNCH_CHECK("gemm_skinny_kernel");
    return LQ_OK;
  }
  GemmBatch b{};
  b.g[0] = g;
  b.count = 1;
  return launch_tiled_batch<TA, TC>(b, s);
}

// ------------------------------------------------------------------ row split ----------

constexpr int RS_THREADS = 256;

template <int CTRL> __device__ __forceinline__ float rs_dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over groups of LPR adjacent lanes (8, 16, 32 or 64), result in every lane of the group.
template <int LPR> __device__ __forceinline__ float rs_allreduce(float y) {
  y += rs_dpp<0xB1>(y);                  // quad_perm [1,0,3,2]
  y += rs_dpp<0x4E>(y);                  // quad_perm [2,3,0,1]
  y += rs_dpp<0x141>(y);                 // row_half_mirror
  if (LPR >= 16) y += rs_dpp<0x140>(y);  // row_mirror
  if (LPR >= 32) y += __shfl_xor(y, 16, 64);
  if (LPR >= 64) y += __shfl_xor(y, 32, 64);
  return y;
}

// LPR lanes share a row (piece c, c + LPR, ... of its K / 4 pieces); a wavefront works on
// U x (64 / LPR) rows per step, all loads of a step issued before the first is used.
// NN = N rounded up to 4 or 8; the weights sit in LDS as [K][NN] with zero padding.  (With more
// outputs the products and the per-row sums outweigh the loads and the matrix-core kernel wins.)
template <int LPR, int NN>
__global__ __launch_bounds__(RS_THREADS) void gemm_rowsplit_kernel(GemmArgs g) {
  constexpr int RPW = 64 / LPR;             // rows per wavefront and sub-step
  constexpr int U = 4;                      // sub-steps in flight
  extern __shared__ __align__(16) float Bs[];
  const float* __restrict__ A = static_cast<const float*>(g.A);
  const float* __restrict__ B = static_cast<const float*>(g.B);
  for (int idx = threadIdx.x; idx < g.Kd * NN; idx += RS_THREADS) {
    const int k = idx / NN, n = idx - k * NN;
    Bs[idx] = n < g.N ? B[static_cast<int64_t>(k) * g.ldb + n] : 0.f;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, c = lane % LPR, sub = lane / LPR;
  const int ppr = g.Kd / 4;                 // 16-byte pieces per row
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (RS_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (RS_THREADS / 64);
  const int64_t nsteps = (g.M + RPW * U - 1) / (RPW * U);
  float bv[NN];
#pragma unroll
  for (int n = 0; n < NN; ++n) bv[n] = (g.bias && n < g.N) ? static_cast<const float*>(g.bias)[n] : 0.f;

  for (int64_t step = wave; step < nsteps; step += nwaves) {
    float acc[U][NN];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int n = 0; n < NN; ++n) acc[u][n] = 0.f;
    for (int p = c; p < ppr; p += LPR) {
      v4f a[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t row = (step * U + u) * RPW + sub;
        a[u] = v4f{0.f, 0.f, 0.f, 0.f};
        if (row < g.M) a[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(A + row * g.lda) + p);
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float b[NN];
#pragma unroll
        for (int q = 0; q < NN / 4; ++q) {
          const v4f bq = *reinterpret_cast<const v4f*>(Bs + (4 * p + t) * NN + 4 * q);
          b[4 * q] = bq[0]; b[4 * q + 1] = bq[1]; b[4 * q + 2] = bq[2]; b[4 * q + 3] = bq[3];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int n = 0; n < NN; ++n) acc[u][n] = fmaf(a[u][t], b[n], acc[u][n]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int n = 0; n < NN; ++n) acc[u][n] = rs_allreduce<LPR>(acc[u][n]);
      const int64_t row = (step * U + u) * RPW + sub;
      if (c == 0 && row < g.M) {
        float* cr = static_cast<float*>(g.C) + row * g.ldc;
#pragma unroll
        for (int n = 0; n < NN; ++n)
          if (n < g.N) {
            float x = acc[u][n] + bv[n];
            if (g.relu) x = fmaxf(x, 0.f);
            cr[n] = x;
          }
      }
    }
  }
}

template <int LPR>
int launch_rowsplit_n(const GemmArgs& g, hipStream_t s) {
  const int nn = g.N <= 4 ? 4 : 8;
  const size_t lds = static_cast<size_t>(g.Kd) * nn * sizeof(float);
  const int rows_per_step = (64 / LPR) * 4;
  const int64_t nsteps = (g.M + rows_per_step - 1) / rows_per_step;
  const int64_t blocks = std::min<int64_t>((nsteps + 3) / 4, static_cast<int64_t>(num_cus()) * 16);
  const dim3 grid(static_cast<unsigned>(blocks)), block(RS_THREADS);
  if (nn == 4) hipLaunchKernelGGL((gemm_rowsplit_kernel<LPR, 4>), grid, block, lds, s, g);
  else hipLaunchKernelGGL((gemm_rowsplit_kernel<LPR, 8>), grid, block, lds, s, g);
  LQ_LAUNCH_CHECK("gemm_rowsplit_kernel");
  return LQ_OK;
}

// Returns -1 when the shape is not one this kernel covers.  The choice depends on N, K, the row
// stride and the alignment only, never on M, so a row computed alone equals the same row computed
// as part of the whole table.
int try_rowsplit(const GemmArgs& g, hipStream_t s) {
  if (g.N > 8 || g.Kd < 32 || g.Kd % 4 || g.lda % 4 || !aligned(g.A, 16) || !aligned(g.C, 4)) return -1;
  if (static_cast<size_t>(g.Kd) * 8 * sizeof(float) > 64 * 1024) return -1;
  const int ppr = g.Kd / 4;
  if (ppr <= 8) return launch_rowsplit_n<8>(g, s);
  if (ppr <= 16) return launch_rowsplit_n<16>(g, s);
  if (ppr <= 32) return launch_rowsplit_n<32>(g, s);
  return launch_rowsplit_n<64>(g, s);
}

}  // namespace

// C[M x N] = act(A[M x Kd] * B[Kd x N] + bias).  A, B, bias share `in_dtype`.
int launch_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                const void* bias, int64_t M, int32_t N, int32_t Kd, int relu, int32_t in_dtype,
                int32_t out_dtype, hipStream_t s) {
  GemmArgs g{};
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.bias = bias;
  g.M = M; g.N = N; g.Kd = Kd; g.relu = relu;
  if (in_dtype == LQ_F32 && out_dtype == LQ_F32) {
    if (M > 0 && N > 0) {
      const int rc = try_rowsplit(g, s);
      if (rc >= 0) return rc;
    }
    return launch_typed<float, float>(g, s);
  }
  if (in_dtype == LQ_BF16 && out_dtype == LQ_F32) return launch_typed<bf16_t, float>(g, s);
  if (in_dtype == LQ_BF16 && out_dtype == LQ_BF16) return launch_typed<bf16_t, bf16_t>(g, s);
  return fail(LQ_ERR_DTYPE, "gemm: f32 inputs cannot produce a bf16 result");
}

int launch_project_dims(const lq_mat& D, const lq_mat& W, int32_t row_off, const lq_mat& P, hipStream_t s);

// P_k = D_k W[off_k .. off_k + c_k) for all K dimensions; one launch when the tiled kernel serves them.
int launch_project_dims_all(int32_t K, const lq_mat* D, const lq_mat& W, int32_t first_off, const lq_mat* P,
                            hipStream_t s) {
  const size_t es = dtype_size(W.dtype);
  bool batch = K > 1 && W.cols > 16;
  for (int k = 0; k < K && batch; ++k) batch = D[k].dtype == D[0].dtype && P[k].dtype == P[0].dtype;
  if (!batch) {
    int32_t off = first_off;
    for (int k = 0; k < K; ++k) {
      const int rc = launch_project_dims(D[k], W, off, P[k], s);
      if (rc) return rc;
      off += D[k].cols;
    }
    return LQ_OK;
  }
  GemmBatch b{};
  int32_t off = first_off;
  for (int k = 0; k < K; ++k) {
    GemmArgs& g = b.g[b.count];
    g.A = D[k].data; g.lda = D[k].ld;
    g.B = static_cast<const char*>(W.data) + static_cast<size_t>(off) * W.ld * es; g.ldb = W.ld;
    g.C = P[k].data; g.ldc = P[k].ld;
    g.M = D[k].rows; g.N = W.cols; g.Kd = D[k].cols;
    off += D[k].cols;
    if (g.M > 0) ++b.count;
  }
  if (b.count == 0) return LQ_OK;
  const int32_t in = D[0].dtype, out = P[0].dtype;
  if (in == LQ_F32 && out == LQ_F32) return launch_tiled_batch<float, float>(b, s);
  if (in == LQ_BF16 && out == LQ_F32) return launch_tiled_batch<bf16_t, float>(b, s);
  if (in == LQ_BF16 && out == LQ_BF16) return launch_tiled_batch<bf16_t, bf16_t>(b, s);
  return fail(LQ_ERR_DTYPE, "gemm: f32 inputs cannot produce a bf16 result");
}

int launch_project_dims(const lq_mat& D, const lq_mat& W, int32_t row_off, const lq_mat& P,
                        hipStream_t s) {
  const size_t es = dtype_size(W.dtype);
  const void* Wk = static_cast<const char*>(W.data) + static_cast<size_t>(row_off) * W.ld * es;
  return launch_gemm(D.data, D.ld, Wk, W.ld, P.data, P.ld, nullptr, D.rows, W.cols, D.cols, 0,
                     D.dtype, P.dtype, s);
}

}  // namespace lq
