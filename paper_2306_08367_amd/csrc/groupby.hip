// Filtered star join + GROUP BY + SUM/COUNT as linear algebra (Sections 2.2-2.4).
//
// The selection vectors of the dimensions are pushed through the row-mapping matrices
// (s_i = prod_k mask_k[fk_k[i]]) and the group-mapping matrix is applied row by row
// (g_i = mixed-radix number of code_k[fk_k[i]]); neither matrix is ever built.
//
// Three launches per call:
//   1. pack_kernel   - folds mask and code of every dimension into one compact side table
//                      per dimension (a bitmap for mask-only dimensions, one byte or one
//                      16-bit word "code, or all-ones if filtered out" for grouping
//                      dimensions).
//   2. scan_kernel   - streams the fact columns once.  The side tables sit in LDS when they
//                      fit (they are read through L2 otherwise); survivors add into int64
//                      accumulators in LDS, which each workgroup stores, as they are, into its
//                      own row of a partial-result matrix in the workspace.
//   3. fold_kernel   - adds the partial rows up into the caller's arrays.  (Flushing with
//                      global atomics instead costs more than this third launch: a few hundred
//                      workgroups queueing on the same few cache lines.)
// Integer addition commutes, so the result is exact and independent of scheduling.
#include "groupby_fast.h"

namespace lq {

int launch_fast_many(const FastArgs& a, const FastLaunch& L);     // groupby_many.hip
int launch_fast_bucket(const FastArgs& a, const FastLaunch& L);   // groupby_many.hip
int launch_fast_wide(const FastArgs& a, const FastLaunch& L, int mode);   // groupby_wide.hip (0 LDS, 1 atomics, 2 buckets)
int launch_agg_fast(const GbArgs& a, const AggFastArgs& x, const FastLaunch& L, int n_preds, int pack_here);   // groupby_agg_fast.hip

namespace {

constexpr int64_t GROUPBY_LDS_ACCUMULATORS = 8192;   // int64 accumulators a scan workgroup keeps in LDS

// ---------------------------------------------------------------- pack ------------------

__global__ __launch_bounds__(256) void pack_kernel(GbArgs a) {
  pack_tables(a, a.packed, static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x,
              static_cast<int64_t>(gridDim.x) * blockDim.x);
}

// ---------------------------------------------------------------- scan ------------------


// VEC fact rows at once: g[q] becomes the group number of row q, or -1 when the row is filtered
// out.  Dimensions form the outer loop so that the (wavefront-uniform) choice of side-table format
// is made once per dimension, not once per row.  fk is [row][dimension].
template <int VEC, int KMAX>
__device__ __forceinline__ void classify(const GbArgs& a, const uint8_t* tab,
                                         const int32_t (&fk)[VEC][KMAX], int32_t (&g)[VEC]) {
  bool alive[VEC];
#pragma unroll
  for (int q = 0; q < VEC; ++q) { alive[q] = true; g[q] = 0; }
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    if (k >= a.K) break;
    const GbDim& d = a.d[k];
    const uint8_t* t = tab + d.off;
    const int32_t stride = d.stride;
    uint32_t jj[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) {
      const int32_t j = fk[q][k];
      alive[q] = alive[q] && j >= 0;
      jj[q] = j < 0 ? 0u : static_cast<uint32_t>(j);   // keep the lookup in bounds
    }
    if (d.kind == DK_BITMAP) {
#pragma unroll
      for (int q = 0; q < VEC; ++q) {
        const uint32_t w = reinterpret_cast<const uint32_t*>(t)[jj[q] >> 5];
        alive[q] = alive[q] && ((w >> (jj[q] & 31)) & 1u);
      }
    } else if (d.kind == DK_BYTE) {
#pragma unroll
      for (int q = 0; q < VEC; ++q) {
        const uint32_t v = t[jj[q]];
        alive[q] = alive[q] && v != 0xffu;
        g[q] += static_cast<int32_t>(v) * stride;
      }
    } else if (d.kind == DK_U16) {
#pragma unroll
      for (int q = 0; q < VEC; ++q) {
        const uint32_t v = reinterpret_cast<const uint16_t*>(t)[jj[q]];
        alive[q] = alive[q] && v != 0xffffu;
        g[q] += static_cast<int32_t>(v) * stride;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < VEC; ++q)
    if (!alive[q]) g[q] = -1;
}

// Key columns (and fact mask) of VEC consecutive fact rows.
template <int VEC, int KMAX> struct KeyRegs {
  int32_t fk[VEC][KMAX];
  uint32_t fm;
};

template <int VEC, int KMAX>
__device__ __forceinline__ void load_keys(const GbArgs& a, int64_t v, KeyRegs<VEC, KMAX>& r) {
  r.fm = 0x01010101u;
  if constexpr (VEC == 4) {
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k >= a.K) break;
      const v4i t = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.d[k].fk) + v);
      r.fk[0][k] = t[0]; r.fk[1][k] = t[1]; r.fk[2][k] = t[2]; r.fk[3][k] = t[3];
    }
    if (a.fact_mask) r.fm = reinterpret_cast<const uint32_t*>(a.fact_mask)[v];
  } else {
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k >= a.K) break;
      r.fk[0][k] = a.d[k].fk[v];
    }
    if (a.fact_mask) r.fm = a.fact_mask[v];
  }
}

template <int VEC, int KMAX>
__device__ __forceinline__ void consume(const GbArgs& a, const uint8_t* tab, unsigned long long* acc,
                                        int64_t v, const KeyRegs<VEC, KMAX>& r) {
  int32_t g[VEC];
  classify<VEC, KMAX>(a, tab, r.fk, g);
  bool any = false;
#pragma unroll
  for (int q = 0; q < VEC; ++q) {
    if (((r.fm >> (8 * q)) & 0xffu) == 0) g[q] = -1;
    any = any || g[q] >= 0;
  }
  if (!any) return;   // the measure columns are only touched where a row survives
#pragma unroll
  for (int m = 0; m < LQ_MAX_MEASURES; ++m) {
    if (m >= a.M) break;
    int32_t val[VEC];
    if constexpr (VEC == 4) {
      const int4 t = reinterpret_cast<const int4*>(a.meas[m])[v];
      val[0] = t.x; val[1] = t.y; val[2] = t.z; val[3] = t.w;
    } else {
      val[0] = a.meas[m][v];
    }
#pragma unroll
    for (int q = 0; q < VEC; ++q)
      if (g[q] >= 0)
        atomicAdd(&acc[m * a.G + g[q]], static_cast<unsigned long long>(static_cast<long long>(val[q])));
  }
#pragma unroll
  for (int q = 0; q < VEC; ++q)
    if (g[q] >= 0) atomicAdd(&acc[a.M * a.G + g[q]], 1ull);
}

// Workgroup b streams the VEC-row groups [b * per_block, (b + 1) * per_block): consecutive
// workgroups sweep memory in order.  The first keys are requested before the side tables are
// copied into LDS, and each iteration requests the next keys before it consumes its own.
template <bool LDS_TABLES, int VEC, int KMAX>
__global__ __launch_bounds__(SCAN_THREADS) void scan_kernel(GbArgs a, int64_t per_block) {
  extern __shared__ __align__(16) uint8_t smem[];
  // layout: accumulators [(M+1) x G] int64, then (LDS_TABLES) the packed tables
  unsigned long long* acc = reinterpret_cast<unsigned long long*>(smem);
  const int n_acc = (a.M + 1) * a.G;
  uint8_t* tab_lds = smem + round_up(static_cast<size_t>(n_acc) * 8, 16);
  const int tid = threadIdx.x;

  const int64_t n_vec = a.n / VEC;   // full VEC-row groups; the tail is done by workgroup 0
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  int64_t v = v_begin + tid;
  KeyRegs<VEC, KMAX> cur, nxt;
  if (v < v_end) load_keys<VEC, KMAX>(a, v, cur);

  for (int i = tid; i < n_acc; i += SCAN_THREADS) acc[i] = 0ull;
  if (LDS_TABLES) {
    const uint4* src = reinterpret_cast<const uint4*>(a.packed);
    uint4* dst = reinterpret_cast<uint4*>(tab_lds);
    for (uint32_t i = tid; i < a.packed_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
  }
  __syncthreads();
  const uint8_t* tab = LDS_TABLES ? tab_lds : a.packed;

  while (v < v_end) {
    const int64_t vn = v + SCAN_THREADS;
    if (vn < v_end) load_keys<VEC, KMAX>(a, vn, nxt);
    consume<VEC, KMAX>(a, tab, acc, v, cur);
    cur = nxt;
    v = vn;
  }
  // ragged tail (n % VEC rows)
  if (VEC > 1 && blockIdx.x == 0) {
    const int64_t i = n_vec * VEC + tid;
    if (i < a.n) {
      int32_t fk1[1][KMAX];
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        if (k >= a.K) break;
        fk1[0][k] = a.d[k].fk[i];
      }
      int32_t g1[1];
      classify<1, KMAX>(a, tab, fk1, g1);
      int32_t g = g1[0];
      if (a.fact_mask && a.fact_mask[i] == 0) g = -1;
      if (g >= 0) {
        for (int m = 0; m < a.M; ++m)
          atomicAdd(&acc[m * a.G + g],
                    static_cast<unsigned long long>(static_cast<long long>(a.meas[m][i])));
        atomicAdd(&acc[a.M * a.G + g], 1ull);
      }
    }
  }
  __syncthreads();
  unsigned long long* mine = a.partial + static_cast<size_t>(blockIdx.x) * n_acc;
  for (int i = tid; i < n_acc; i += SCAN_THREADS) mine[i] = acc[i];
}


// ---------------------------------------------------------------- fold ------------------

constexpr int FOLD_THREADS = 512;
constexpr int FOLD_PARTS = 64;                       // threads sharing one accumulator
constexpr int FOLD_ACCS = FOLD_THREADS / FOLD_PARTS; // accumulators per workgroup

// sums / counts [i] = sum over workgroups b of partial[b][i].  Eight consecutive accumulators per
// workgroup, each summed by 64 threads striding over the partial rows, then combined in LDS.
__global__ __launch_bounds__(FOLD_THREADS) void fold_kernel(GbArgs a, int rows_written) {
  __shared__ unsigned long long part[FOLD_PARTS][FOLD_ACCS];
  const int n_acc = (a.M + 1) * a.G;
  const int il = threadIdx.x % FOLD_ACCS, p = threadIdx.x / FOLD_ACCS;
  const int i = blockIdx.x * FOLD_ACCS + il;
  unsigned long long t = 0ull;
  if (i < n_acc) {
#pragma unroll 8
    for (int b = p; b < rows_written; b += FOLD_PARTS) t += a.partial[static_cast<size_t>(b) * n_acc + i];
  }
  part[p][il] = t;
  __syncthreads();
  if (threadIdx.x < FOLD_ACCS && i < n_acc) {
    unsigned long long tot = 0ull;
#pragma unroll
    for (int q = 0; q < FOLD_PARTS; ++q) tot += part[q][il];
    if (i < a.M * a.G) a.sums[i] = tot;
    else if (a.counts) a.counts[i - a.M * a.G] = tot;
  }
}

// The same fold for results of up to a thousand accumulators (175 groups x (SUM, COUNT) is typical): one
// wavefront per accumulator, lane l adds partial rows l, l + 64, .. with all its loads in flight, then the
// lanes are added through the cross-lane network.  Fewer dependent steps than the two-level form above,
// which in turn touches eight times fewer cache lines per load and stays the form for large results.
constexpr int FOLD_WAVE_THREADS = 256;
constexpr int FOLD_WAVE_MAX_ACC = 1024;
__global__ __launch_bounds__(FOLD_WAVE_THREADS) void fold_wave_kernel(GbArgs a, int rows_written) {
  const int n_acc = (a.M + 1) * a.G;
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (FOLD_WAVE_THREADS / 64) + (threadIdx.x >> 6);
  if (i >= n_acc) return;
  unsigned long long t = 0ull;
  for (int b0 = lane; b0 < rows_written; b0 += 8 * 64) {
    unsigned long long v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int b = b0 + u * 64;
      v[u] = b < rows_written ? a.partial[static_cast<size_t>(b) * n_acc + i] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) t += v[u];
  }
  const unsigned long long tot = static_cast<unsigned long long>(wave_sum64(static_cast<long long>(t)));
  if (lane == 0) {
    if (i < a.M * a.G) a.sums[i] = tot;
    else if (a.counts) a.counts[i - a.M * a.G] = tot;
  }
}

// Launches whichever fold suits the number of accumulators.
static int launch_fold(const GbArgs& a, int rows_written, hipStream_t s) {
  const int n_acc = (a.M + 1) * a.G;
  if (n_acc <= FOLD_WAVE_MAX_ACC) {
    const unsigned blocks = static_cast<unsigned>((n_acc + FOLD_WAVE_THREADS / 64 - 1) / (FOLD_WAVE_THREADS / 64));
    hipLaunchKernelGGL(fold_wave_kernel, dim3(blocks), dim3(FOLD_WAVE_THREADS), 0, s, a, rows_written);
  } else {
    const unsigned blocks = static_cast<unsigned>((n_acc + FOLD_ACCS - 1) / FOLD_ACCS);
    hipLaunchKernelGGL(fold_kernel, dim3(blocks), dim3(FOLD_THREADS), 0, s, a, rows_written);
  }
  LQ_LAUNCH_CHECK("fold_kernel");
  return LQ_OK;
}

// ---------------------------------------------------------------- wider aggregate ----------

// Fact-side range predicates (selection vectors on the fact table), measures that are a column or
// the element-wise product / difference of two columns, SUM / MIN / MAX / COUNT per group.
constexpr int MAX_PREDS = 4;
struct AggExtra {
  int32_t n_preds;
  const int32_t* pcol[MAX_PREDS];
  int32_t lo[MAX_PREDS], hi[MAX_PREDS];
  int32_t op[LQ_MAX_MEASURES];                 // 0 column, 1 product, 2 difference
  const int32_t* b[LQ_MAX_MEASURES];
  unsigned long long* mins;                    // caller arrays (may be NULL), int64 bit patterns
  unsigned long long* maxs;
};
// Accumulator layout (LDS, partial rows): [sums M x G | counts G | mins M x G | maxs M x G].

__device__ __forceinline__ long long agg_init(int i, int M, int G) {
  return i < (M + 1) * G ? 0LL : (i < (2 * M + 1) * G ? AGG_MIN_INIT : AGG_MAX_INIT);
}

template <bool LDS_TABLES, int VEC, int KMAX>
// pack_here: the dimension tables are so small that every workgroup encodes its own copy of the side tables
// straight into LDS from the raw mask / code arrays (no separate launch); workgroup 0 also leaves them in the
// workspace, where a later call that reuses the side tables expects them.
__global__ __launch_bounds__(SCAN_THREADS) void agg_scan_kernel(GbArgs a, AggExtra x, int64_t per_block, int vec_ok, int pack_here) {
  extern __shared__ __align__(16) uint8_t smem[];
  long long* acc = reinterpret_cast<long long*>(smem);
  const int MG = a.M * a.G;
  const int n_acc = (3 * a.M + 1) * a.G;
  uint8_t* tab_lds = smem + round_up(static_cast<size_t>(n_acc) * 8, 16);
  const int tid = threadIdx.x;
  for (int i = tid; i < n_acc; i += SCAN_THREADS) acc[i] = agg_init(i, a.M, a.G);
  if (LDS_TABLES) {
    if (pack_here) {
      pack_tables(a, tab_lds, tid, SCAN_THREADS);
      if (blockIdx.x == 0) {
        __syncthreads();
        uint4* dst = reinterpret_cast<uint4*>(a.packed);
        const uint4* src = reinterpret_cast<const uint4*>(tab_lds);
        for (uint32_t i = tid; i < a.packed_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
      }
    } else {
      const uint4* src = reinterpret_cast<const uint4*>(a.packed);
      uint4* dst = reinterpret_cast<uint4*>(tab_lds);
      for (uint32_t i = tid; i < a.packed_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
    }
  }
  __syncthreads();
  const uint8_t* tab = LDS_TABLES ? tab_lds : a.packed;

  // VEC consecutive values of a column starting at row i0 (16-byte load when the column allows it)
  auto load4 = [&](const int32_t* col, int64_t i0, int cnt, int32_t (&out)[VEC]) {
    if (vec_ok && cnt == VEC) {
      const v4i t = *reinterpret_cast<const v4i*>(col + i0);
#pragma unroll
      for (int q = 0; q < VEC; ++q) out[q] = t[q];
    } else {
#pragma unroll
      for (int q = 0; q < VEC; ++q) out[q] = q < cnt ? col[i0 + q] : 0;
    }
  };
  // VEC rows starting at fact row i0 (rows >= a.n are skipped)
  auto rows = [&](int64_t i0, int cnt) {
    int32_t fk[VEC][KMAX];
    bool pass[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) pass[q] = q < cnt;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      int32_t t[VEC] = {0, 0, 0, 0};
      if (k < a.K) load4(a.d[k].fk, i0, cnt, t);
#pragma unroll
      for (int q = 0; q < VEC; ++q) fk[q][k] = t[q];
    }
    // all predicate columns are requested before the first comparison waits for one of them
    int32_t pv[MAX_PREDS][VEC];
#pragma unroll
    for (int pq = 0; pq < MAX_PREDS; ++pq)
      if (pq < x.n_preds) load4(x.pcol[pq], i0, cnt, pv[pq]);
#pragma unroll
    for (int pq = 0; pq < MAX_PREDS; ++pq)
      if (pq < x.n_preds) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) pass[q] = pass[q] && pv[pq][q] >= x.lo[pq] && pv[pq][q] <= x.hi[pq];
      }
    int32_t g[VEC];
    classify<VEC, KMAX>(a, tab, fk, g);
    bool any = false;
#pragma unroll
    for (int q = 0; q < VEC; ++q) { pass[q] = pass[q] && g[q] >= 0; any = any || pass[q]; }
    if (!any) return;            // measure columns are only touched where a row survives
    for (int m = 0; m < a.M; ++m) {
      int32_t av[VEC], bv[VEC];
      load4(a.meas[m], i0, cnt, av);
      if (x.op[m] != 0) load4(x.b[m], i0, cnt, bv);
#pragma unroll
      for (int q = 0; q < VEC; ++q) {
        if (!pass[q]) continue;
        long long v = av[q];
        if (x.op[m] == 1) v *= static_cast<long long>(bv[q]);
        else if (x.op[m] == 2) v -= static_cast<long long>(bv[q]);
        atomicAdd(reinterpret_cast<unsigned long long*>(&acc[m * a.G + g[q]]), static_cast<unsigned long long>(v));
        atomicMin(&acc[(a.M + 1) * a.G + m * a.G + g[q]], v);
        atomicMax(&acc[(2 * a.M + 1) * a.G + m * a.G + g[q]], v);
      }
    }
#pragma unroll
    for (int q = 0; q < VEC; ++q)
      if (pass[q]) atomicAdd(reinterpret_cast<unsigned long long*>(&acc[MG + g[q]]), 1ull);
  };

  const int64_t n_vec = (a.n + VEC - 1) / VEC;
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  for (int64_t v = v_begin + tid; v < v_end; v += SCAN_THREADS) {
    const int64_t i0 = v * VEC;
    rows(i0, static_cast<int>(min<int64_t>(VEC, a.n - i0)));
  }
  __syncthreads();
  long long* mine = reinterpret_cast<long long*>(a.partial) + static_cast<size_t>(blockIdx.x) * n_acc;
  for (int i = tid; i < n_acc; i += SCAN_THREADS) mine[i] = acc[i];
}

// Fold of the wider aggregate: add, min or max depending on the segment the accumulator is in.  One
// wavefront per accumulator: lane l combines partial rows l, l + 64, .. (all its loads requested before the
// first is used), then the 64 lanes are combined through the cross-lane network.
constexpr int FOLD_AGG_THREADS = 256;
__global__ __launch_bounds__(FOLD_AGG_THREADS) void fold_agg_kernel(GbArgs a, AggExtra x, int rows_written) {
  const int n_acc = (3 * a.M + 1) * a.G;
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (FOLD_AGG_THREADS / 64) + (threadIdx.x >> 6);
  if (i >= n_acc) return;
  const int seg = i < (a.M + 1) * a.G ? 0 : (i < (2 * a.M + 1) * a.G ? 1 : 2);
  const long long neutral = agg_init(i, a.M, a.G);
  long long t = neutral;
  const long long* partial = reinterpret_cast<const long long*>(a.partial);
  for (int b0 = lane; b0 < rows_written; b0 += 8 * 64) {
    long long v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int b = b0 + u * 64;
      v[u] = b < rows_written ? partial[static_cast<size_t>(b) * n_acc + i] : neutral;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) t = seg == 0 ? t + v[u] : (seg == 1 ? min(t, v[u]) : max(t, v[u]));
  }
  const long long tot = seg == 0 ? wave_sum64(t) : (seg == 1 ? wave_min64(t) : wave_max64(t));
  if (lane == 0) {
    const int MG = a.M * a.G;
    if (i < MG) { if (a.sums) a.sums[i] = static_cast<unsigned long long>(tot); }
    else if (i < MG + a.G) { if (a.counts) a.counts[i - MG] = static_cast<unsigned long long>(tot); }
    else if (i < 2 * MG + a.G) { if (x.mins) x.mins[i - MG - a.G] = static_cast<unsigned long long>(tot); }
    else if (x.maxs) x.maxs[i - 2 * MG - a.G] = static_cast<unsigned long long>(tot);
  }
}

// The scan of scan_kernel / agg_scan_kernel with the accumulators in memory.  x.n_preds == 0 and
// op == column give the plain masked group-by sum.
template <bool LDS_TABLES, int VEC, int KMAX>
__global__ __launch_bounds__(SCAN_THREADS) void scan_global_kernel(GbArgs a, AggExtra x, GlobalOut o, int64_t per_block,
                                                                   int vec_ok) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x;
  if (LDS_TABLES) {
    const uint4* src = reinterpret_cast<const uint4*>(a.packed);
    uint4* dst = reinterpret_cast<uint4*>(smem);
    for (uint32_t i = tid; i < a.packed_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
    __syncthreads();
  }
  const uint8_t* tab = LDS_TABLES ? smem : a.packed;

  auto load4 = [&](const int32_t* col, int64_t i0, int cnt, int32_t (&out)[VEC]) {
    if (VEC == 4 && vec_ok && cnt == VEC) {
      const v4i t = *reinterpret_cast<const v4i*>(col + i0);
#pragma unroll
      for (int q = 0; q < VEC; ++q) out[q] = t[q];
    } else {
#pragma unroll
      for (int q = 0; q < VEC; ++q) out[q] = q < cnt ? col[i0 + q] : 0;
    }
  };

  const int64_t n_vec = (a.n + VEC - 1) / VEC;
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  // every lane of a wavefront takes the same number of steps: the merge is a wavefront operation
  for (int64_t v0 = v_begin + (tid & ~63); v0 < v_end; v0 += SCAN_THREADS) {
    const int64_t v = v0 + (tid & 63);
    const int64_t i0 = v * VEC;
    const int cnt = v < v_end ? static_cast<int>(min<int64_t>(VEC, a.n - i0)) : 0;
    int32_t fk[VEC][KMAX];
    bool pass[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) pass[q] = q < cnt;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      int32_t t[VEC];
#pragma unroll
      for (int q = 0; q < VEC; ++q) t[q] = -1;
      if (k < a.K && cnt > 0) load4(a.d[k].fk, i0, cnt, t);
#pragma unroll
      for (int q = 0; q < VEC; ++q) fk[q][k] = t[q];
    }
    if (a.fact_mask && cnt > 0) {
#pragma unroll
      for (int q = 0; q < VEC; ++q) pass[q] = pass[q] && a.fact_mask[i0 + (q < cnt ? q : 0)] != 0;
    }
#pragma unroll
    for (int pq = 0; pq < MAX_PREDS; ++pq)
      if (pq < x.n_preds && cnt > 0) {
        int32_t pv[VEC];
        load4(x.pcol[pq], i0, cnt, pv);
#pragma unroll
        for (int q = 0; q < VEC; ++q) pass[q] = pass[q] && pv[q] >= x.lo[pq] && pv[q] <= x.hi[pq];
      }
    int32_t g[VEC];
    classify<VEC, KMAX>(a, tab, fk, g);
    bool any = false;
#pragma unroll
    for (int q = 0; q < VEC; ++q) { pass[q] = pass[q] && g[q] >= 0; any = any || pass[q]; }
    long long val[VEC][LQ_MAX_MEASURES];
#pragma unroll
    for (int q = 0; q < VEC; ++q)
#pragma unroll
      for (int m = 0; m < LQ_MAX_MEASURES; ++m) val[q][m] = 0;
    if (any) {                  // measure columns are only touched where a row survives
#pragma unroll
      for (int m = 0; m < LQ_MAX_MEASURES; ++m) {
        if (m >= a.M) break;
        int32_t av[VEC], bv[VEC];
        load4(a.meas[m], i0, cnt, av);
        if (x.op[m] != 0) load4(x.b[m], i0, cnt, bv);
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
          long long t = av[q];
          if (x.op[m] == 1) t *= static_cast<long long>(bv[q]);
          else if (x.op[m] == 2) t -= static_cast<long long>(bv[q]);
          val[q][m] = t;
        }
      }
    }
    if (__ballot(any) == 0ull) continue;
#pragma unroll
    for (int q = 0; q < VEC; ++q) merge_and_add<LQ_MAX_MEASURES>(pass[q], g[q], val[q], a.M, a.G, o);
  }
}

// AVG = SUM / COUNT per group, in fp64 (one correctly rounded division); NaN for a group without rows.
__global__ __launch_bounds__(256) void group_avg_kernel(const long long* __restrict__ sums, const long long* __restrict__ counts,
                                                        double* __restrict__ avgs, int64_t MG, int64_t G) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < MG; i += stride) {
    const long long c = counts[i % G];
    avgs[i] = c > 0 ? static_cast<double>(sums[i]) / static_cast<double>(c) : __longlong_as_double(0x7ff8000000000000LL);
  }
}

constexpr size_t LDS_BUDGET = 160 * 1024 - 1024;   // gfx950 workgroups may use the whole 160 KB

// Fills kind / off / bytes of every dimension; returns the packed size.  Tables are laid out by
// ascending size so that "the tables that fit in LDS" is always a prefix of the packed buffer;
// *lds_prefix receives the length of the longest prefix that fits `lds_room` bytes.
size_t plan_tables(int32_t K, const int64_t* rows, const uint8_t* const* mask,
                   const int32_t* const* code, const int32_t* card, GbDim* d, size_t lds_room,
                   size_t* lds_prefix) {
  size_t bytes[LQ_MAX_DIMS];
  int order[LQ_MAX_DIMS];
  for (int k = 0; k < K; ++k) {
    const bool has_mask = mask && mask[k];
    const bool has_code = code && code[k];
    const int64_t r = rows[k];
    size_t b = 0;
    int32_t kind = DK_NONE;
    if (has_code) {
      if (card[k] <= 255) { kind = DK_BYTE; b = static_cast<size_t>(r); }
      else { kind = DK_U16; b = static_cast<size_t>(r) * 2; }
    } else {
      // (also for a joined table with neither predicate nor grouping attribute, which can only drop rows through a
      // negative key: an all-ones bitmap keeps such calls on the specialised scans)
      kind = DK_BITMAP; b = static_cast<size_t>((r + 31) / 32) * 4;
    }
    (void)has_mask;
    bytes[k] = round_up(b, 16);
    d[k].kind = kind;
    order[k] = k;
  }
  std::stable_sort(order, order + K, [&](int x, int y) { return bytes[x] < bytes[y]; });
  size_t off = 0, prefix = 0;
  bool fits = true;
  for (int q = 0; q < K; ++q) {
    const int k = order[q];
    d[k].off = static_cast<uint32_t>(off);
    d[k].bytes = static_cast<uint32_t>(bytes[k]);
    d[k].in_lds = 0;
    off += bytes[k];
    if (fits && off <= lds_room) { prefix = off; d[k].in_lds = 1; } else fits = false;
  }
  if (lds_prefix) *lds_prefix = prefix;
  return off;
}

}  // namespace

// Workspace layout: [side tables | partial results, one row per scan workgroup].
size_t groupby_tables_bytes(int32_t K, const int64_t* rows) {
  // Upper bound that does not depend on which dimensions carry masks or codes:
  // two bytes per dimension row, each table rounded to 16 bytes.
  size_t t = 0;
  for (int k = 0; k < K; ++k) t += round_up(static_cast<size_t>(rows[k]) * 2, 16);
  return round_up(t, 256) + 256;
}
int groupby_max_workgroups() { return 2 * num_cus(); }
// Up to GROUPBY_LDS_ACCUMULATORS accumulators live in LDS and every scan workgroup leaves a partial row
// in the workspace; beyond that the accumulators are the caller's output arrays and the workspace only
// holds the side tables (plus the check's flag word).
size_t groupby_ws_bytes(int32_t K, const int64_t* rows, int64_t n_acc) {
  if (n_acc > GROUPBY_LDS_ACCUMULATORS) return groupby_tables_bytes(K, rows) + 256;
  return groupby_tables_bytes(K, rows) +
         round_up(static_cast<size_t>(groupby_max_workgroups()) * n_acc * 8, 256);
}

// Geometry of the bucketed many-groups form for n fact rows: false when it does not apply.
//   shift   a bucket covers 1 << shift neighbouring groups, whose (M + 1) accumulators each fit LDS
//   buckets at least 256 where G allows (one workgroup per bucket in the second pass), at most 8,192
//   cap     slots per bucket: twice the even share plus 1,024 (a bucket that overflows sends the rest through atomics)
bool bucket_plan(int64_t n, int64_t G, int32_t M, BucketArgs* b, size_t* bytes) {
  if (M < 1 || M > 2 || n < 1 || n > 0x7fffffffLL) return false;           // (the specialised scans take one or two measures)
  if ((M + 1) * G <= GROUPBY_LDS_ACCUMULATORS) return false;
  int shift = 0;
  while ((int64_t{2} << shift) * (M + 1) <= GROUPBY_LDS_ACCUMULATORS && (int64_t{2} << shift) * 256 <= G) ++shift;
  const int64_t buckets = (G + (int64_t{1} << shift) - 1) >> shift;
  if (buckets > 8192) return false;
  const int64_t cap = 2 * ((n + buckets - 1) / buckets) + 1024;
  if (cap > 0x7fffffffLL) return false;
  b->shift = shift;
  b->buckets = static_cast<int32_t>(buckets);
  b->cap = static_cast<uint32_t>(cap);
  *bytes = round_up(static_cast<size_t>(buckets) * 4, 256) + static_cast<size_t>(buckets) * cap * (1 + M) * 4;
  return true;
}

// Workspace that lets a group-by of n rows over more than 8,192 accumulators take the bucketed form (0: it does not apply).
// (Three or four measures run as two calls of two: sized for those, provided two measures alone pass the LDS limit.)
size_t groupby_bucket_ws_bytes(int64_t n, int32_t K, const int64_t* rows, int64_t G, int32_t M) {
  BucketArgs b{};
  size_t extra = 0;
  if (M > 2) {
    if (M > LQ_MAX_MEASURES || 3 * G <= GROUPBY_LDS_ACCUMULATORS) return 0;
    M = 2;
  }
  if (!bucket_plan(n, G, M, &b, &extra)) return 0;
  return round_up(groupby_ws_bytes(K, rows, G * (M + 1)), 256) + extra;
}

// sums[g] = two[g] - two[G + g]: SUM(a - b) from SUM(a) and SUM(b), exact in int64.
__global__ __launch_bounds__(256) void group_diff_kernel(const long long* __restrict__ two, long long* __restrict__ sums, int64_t G) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t g = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; g < G; g += stride) sums[g] = two[g] - two[G + g];
}

int launch_group_diff(int64_t G, const int64_t* two, int64_t* sums, hipStream_t s) {
  if (G == 0) return LQ_OK;
  const int64_t blocks = std::min<int64_t>((G + 255) / 256, static_cast<int64_t>(num_cus()) * 8);
  hipLaunchKernelGGL(group_diff_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                     reinterpret_cast<const long long*>(two), reinterpret_cast<long long*>(sums), G);
  LQ_LAUNCH_CHECK("group_diff_kernel");
  return LQ_OK;
}

int launch_group_avg(int32_t M, int64_t G, const int64_t* sums, const int64_t* counts, double* avgs, hipStream_t s) {
  const int64_t MG = static_cast<int64_t>(M) * G;
  if (MG == 0) return LQ_OK;
  const int64_t blocks = std::min<int64_t>((MG + 255) / 256, static_cast<int64_t>(num_cus()) * 8);
  hipLaunchKernelGGL(group_avg_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                     reinterpret_cast<const long long*>(sums), reinterpret_cast<const long long*>(counts), avgs, MG, G);
  LQ_LAUNCH_CHECK("group_avg_kernel");
  return LQ_OK;
}

// sums / counts = 0, mins / maxs = neutral elements, for the accumulators-in-memory form.
static int launch_init_outputs(const GlobalOut& o, int32_t M, int32_t G, hipStream_t s, unsigned int* words = nullptr,
                               int64_t n_words = 0) {
  const int64_t MG = std::max<int64_t>(static_cast<int64_t>(M) * G, G);
  const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>((MG + 255) / 256, static_cast<int64_t>(num_cus()) * 8));
  hipLaunchKernelGGL(init_outputs_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, o, MG, static_cast<int64_t>(G),
                     words, n_words);
  LQ_LAUNCH_CHECK("init_outputs_kernel");
  return LQ_OK;
}

static int launch_pack(const GbArgs& a, hipStream_t s) {
  size_t work = 1;
  for (int k = 0; k < a.K; ++k) {
    const size_t w = a.d[k].kind == DK_BITMAP ? static_cast<size_t>(a.d[k].bytes) * 8   // one lane per row
                                              : static_cast<size_t>(a.d[k].bytes) / 4;   // one thread per word
    work = std::max(work, w);
  }
  const int64_t blocks = std::min<int64_t>(static_cast<int64_t>((work + 255) / 256), static_cast<int64_t>(num_cus()) * 8);
  hipLaunchKernelGGL(pack_kernel, dim3(static_cast<unsigned>(std::max<int64_t>(blocks, 1))), dim3(256), 0, s, a);
  LQ_LAUNCH_CHECK("pack_kernel");
  return LQ_OK;
}

// The run-time generic scan with the accumulators in memory (side tables all in LDS or all in memory).
static int launch_scan_global(const GbArgs& a, const AggExtra& x, const GlobalOut& o, size_t lds_prefix, bool vec_ok,
                              hipStream_t s) {
  const int cus = num_cus();
  const int vec = vec_ok ? 4 : 1;
  const int64_t n_vec = (a.n + vec - 1) / vec;
  const bool lds_tables = lds_prefix == a.packed_bytes;
  const size_t lds = lds_tables ? a.packed_bytes : 0;
  const int per_cu = lds * 2 <= 160 * 1024 ? 2 : 1;
  int64_t b = std::max<int64_t>(1, std::min<int64_t>((n_vec + SCAN_THREADS - 1) / SCAN_THREADS, static_cast<int64_t>(cus) * per_cu));
  int64_t pb = (n_vec + b - 1) / b;
  pb = std::max<int64_t>(SCAN_THREADS, (pb + SCAN_THREADS - 1) / SCAN_THREADS * SCAN_THREADS);
  b = std::max<int64_t>(1, (n_vec + pb - 1) / pb);
  const unsigned blocks = static_cast<unsigned>(b);
  const int kmax = a.K <= 2 ? 2 : (a.K <= 4 ? 4 : 8);
#define LQ_SCANG(LT, V, KM)                                                                             \
  do {                                                                                                  \
    if (lds > 64 * 1024)                                                                                \
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&scan_global_kernel<LT, V, KM>),     \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
    hipLaunchKernelGGL((scan_global_kernel<LT, V, KM>), dim3(blocks), dim3(SCAN_THREADS), lds, s, a, x, o, pb, \
                       vec_ok ? 1 : 0);                                                                 \
  } while (0)
#define LQ_SCANG_K(LT, V)                                                                               \
  do {                                                                                                  \
    if (kmax == 2) LQ_SCANG(LT, V, 2); else if (kmax == 4) LQ_SCANG(LT, V, 4); else LQ_SCANG(LT, V, 8); \
  } while (0)
  if (lds_tables) { if (vec == 4) LQ_SCANG_K(true, 4); else LQ_SCANG_K(true, 1); }
  else            { if (vec == 4) LQ_SCANG_K(false, 4); else LQ_SCANG_K(false, 1); }
#undef LQ_SCANG_K
#undef LQ_SCANG
  LQ_LAUNCH_CHECK("scan_global_kernel");
  return LQ_OK;
}

int launch_groupby(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                   const uint8_t* const* mask, const int32_t* const* code, const int32_t* card,
                   const uint8_t* fact_mask, int32_t M, const int32_t* const* meas, int64_t* sums,
                   int64_t* counts, int32_t G, void* ws, size_t ws_bytes, bool reuse_tables, hipStream_t s) {
  GbArgs a{};
  a.n = n; a.K = K; a.fact_mask = fact_mask; a.M = M; a.G = G;
  a.sums = reinterpret_cast<unsigned long long*>(sums);
  a.counts = reinterpret_cast<unsigned long long*>(counts);
  a.packed = static_cast<uint8_t*>(ws);
  a.partial = reinterpret_cast<unsigned long long*>(a.packed + groupby_tables_bytes(K, rows));
  bool vec_ok = aligned(fact_mask, 4);
  for (int k = 0; k < K; ++k) {
    a.d[k].fk = fks[k];
    a.d[k].mask = mask ? mask[k] : nullptr;
    a.d[k].code = code ? code[k] : nullptr;
    a.d[k].rows = rows[k];
    a.d[k].card = (code && code[k]) ? card[k] : 1;
    vec_ok = vec_ok && aligned(fks[k], 16);
  }
  for (int m = 0; m < M; ++m) { a.meas[m] = meas[m]; vec_ok = vec_ok && aligned(meas[m], 16); }
  {   // mixed-radix weights, last grouping dimension fastest
    int32_t stride = 1;
    for (int k = K - 1; k >= 0; --k) {
      const bool grouping = code && code[k];
      a.d[k].stride = grouping ? stride : 0;
      if (grouping) stride *= card[k];
    }
  }
  // More accumulators than a workgroup keeps in LDS: the caller's arrays accumulate (no partial rows, no fold).
  const bool gacc = static_cast<int64_t>(M + 1) * G > GROUPBY_LDS_ACCUMULATORS;
  const int n_acc = gacc ? 0 : (M + 1) * G;
  const size_t acc_bytes = round_up(static_cast<size_t>(n_acc) * 8, 16);
  size_t lds_prefix = 0;
  const size_t packed = plan_tables(K, rows, mask, code, card, a.d, LDS_BUDGET - acc_bytes, &lds_prefix);
  if (packed > 0xffffffffull) return fail(LQ_ERR_UNSUPPORTED, "group-by: dimension side tables exceed 4 GiB");
  a.packed_bytes = static_cast<uint32_t>(packed);

  const int cus = num_cus();
  int rc0;
  const GlobalOut gout{a.sums, a.counts, nullptr, nullptr};
  // many groups: through buckets when the specialised scan applies and the caller's workspace has room for them
  // (their counters are cleared with the outputs), else through atomics
  BucketArgs bucket{};
  bool want_buckets = false;
  if (gacc && vec_ok && n > 0) {
    size_t extra = 0;
    const size_t base = round_up(groupby_ws_bytes(K, rows, static_cast<int64_t>(M + 1) * G), 256);
    if (bucket_plan(n, G, M, &bucket, &extra) && ws_bytes >= base + extra &&
        round_up(lds_prefix, 16) + static_cast<size_t>(bucket.buckets) * 8 <= LDS_BUDGET) {
      want_buckets = true;
      bucket.gcount = reinterpret_cast<unsigned int*>(static_cast<uint8_t*>(ws) + base);
      bucket.pairs = reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(ws) + base + round_up(static_cast<size_t>(bucket.buckets) * 4, 256));
    }
  }
  if (gacc && (rc0 = launch_init_outputs(gout, M, G, s, want_buckets ? bucket.gcount : nullptr, want_buckets ? bucket.buckets : 0)))
    return rc0;
  if (!reuse_tables && (n > 0 || !gacc) && (rc0 = launch_pack(a, s))) return rc0;
  if (n == 0) {   // nothing to scan: the fold alone writes the all-zero result
    if (gacc) return LQ_OK;
    return launch_fold(a, 0, s);
  }

  const int vec = vec_ok ? 4 : 1;
  const int64_t n_vec = n / vec;
  // Resident workgroups each take one contiguous slice (a multiple of the workgroup size).
  auto slices = [&](size_t lds_bytes, unsigned* blocks, int64_t* per_block) {
    // Workgroups per CU the LDS footprint allows (at most two 1024-thread workgroups fit a CU).
    const int per_cu = lds_bytes * 2 <= 160 * 1024 ? 2 : 1;
    int64_t b = std::max<int64_t>(1, std::min<int64_t>((n_vec + SCAN_THREADS - 1) / SCAN_THREADS,
                                                       static_cast<int64_t>(cus) * per_cu));
    b = std::min<int64_t>(b, groupby_max_workgroups());
    int64_t pb = (n_vec + b - 1) / b;
    pb = std::max<int64_t>(SCAN_THREADS, (pb + SCAN_THREADS - 1) / SCAN_THREADS * SCAN_THREADS);
    b = std::max<int64_t>(1, (n_vec + pb - 1) / pb);
    *blocks = static_cast<unsigned>(b);
    *per_block = pb;
  };

  // Common case: compile-time specialised kernel, side tables in LDS as far as they fit.
  if (vec == 4) {
    FastArgs f{};
    FastLaunch L{};
    bool ok = true;
    int slot = 0;
    // runs: byte in LDS, bitmap in LDS, bitmap in memory, byte in memory
    for (int run = 0; run < 4 && ok; ++run)
      for (int k = 0; k < K; ++k) {
        const bool wide = a.d[k].kind == DK_U16;               // a code table of 16-bit entries rides with the byte tables
        const int kind = wide ? static_cast<int>(DK_BYTE) : a.d[k].kind;
        if (kind != DK_BYTE && kind != DK_BITMAP) { ok = false; break; }
        const int want_kind = (run == 0 || run == 3) ? DK_BYTE : DK_BITMAP;
        const int want_lds = run < 2 ? 1 : 0;
        if (kind != want_kind || a.d[k].in_lds != want_lds) continue;
        f.fk[slot] = a.d[k].fk; f.off[slot] = a.d[k].off; f.stride[slot] = a.d[k].stride; f.wide[slot] = wide ? 1 : 0;
        ++slot;
        if (run == 0) ++L.nbl; else if (run == 1) ++L.nml; else if (run == 2) ++L.nmg; else ++L.nbg;
      }
    if (ok) {
      f.n = n; f.packed = a.packed; f.lds_bytes = static_cast<uint32_t>(lds_prefix); f.G = G; f.partial = a.partial;
      f.gsums = gacc ? a.sums : nullptr;
      f.gcounts = gacc ? a.counts : nullptr;
      for (int m = 0; m < M; ++m) f.meas[m] = meas[m];
      L.lds = acc_bytes + lds_prefix; L.s = s; L.M = M;
      const bool buckets = want_buckets;
      if (buckets) {
        L.bucket = bucket;
        L.lds = round_up(lds_prefix, 16) + static_cast<size_t>(bucket.buckets) * 8;
      }
      slices(L.lds, &L.blocks, &L.per_block);
      // (a fact mask is read by the instantiations that also take 16-bit code tables: calls without either do not pay for the test)
      f.fact_mask = fact_mask;
      bool any_wide = fact_mask != nullptr;
      for (int k = 0; k < slot; ++k) any_wide = any_wide || f.wide[k];
      auto run = [&](int mode) {
        if (any_wide) return launch_fast_wide(f, L, mode);
        return mode == 0 ? launch_fast<0>(f, L) : (mode == 1 ? launch_fast_many(f, L) : launch_fast_bucket(f, L));
      };
      int rc = run(gacc ? (buckets ? 2 : 1) : 0);
      if (rc == -1 && buckets) {                     // no bucketed instantiation for this mix: the atomic form
        L.lds = acc_bytes + lds_prefix;
        slices(L.lds, &L.blocks, &L.per_block);
        rc = run(1);
      }
      if (rc > 0) return rc;
      if (rc == 0) {
        if (gacc) return LQ_OK;
        return launch_fold(a, static_cast<int>(L.blocks), s);
      }
    }
  }

  // Everything else: the run-time generic kernel, side tables all in LDS or all in memory.
  if (gacc) {
    AggExtra x{};
    for (int m = 0; m < M; ++m) x.b[m] = meas[m];
    return launch_scan_global(a, x, gout, lds_prefix, vec_ok, s);
  }
  const bool lds_tables = lds_prefix == packed;
  const size_t lds = acc_bytes + (lds_tables ? packed : 0);
  unsigned blocks = 0;
  int64_t per_block = 0;
  slices(lds, &blocks, &per_block);
  const int kmax = K <= 2 ? 2 : (K <= 4 ? 4 : 8);

#define LQ_SCAN(LT, V, KM)                                                                    \
  do {                                                                                        \
    if (lds > 64 * 1024)                                                                      \
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&scan_kernel<LT, V, KM>),  \
                                     hipFuncAttributeMaxDynamicSharedMemorySize,              \
                                     static_cast<int>(lds)));                                 \
    hipLaunchKernelGGL((scan_kernel<LT, V, KM>), dim3(blocks), dim3(SCAN_THREADS), lds, s, a, \
                       per_block);                                                            \
  } while (0)
#define LQ_SCAN_K(LT, V)                                                                      \
  do {                                                                                        \
    if (kmax == 2) LQ_SCAN(LT, V, 2); else if (kmax == 4) LQ_SCAN(LT, V, 4); else LQ_SCAN(LT, V, 8); \
  } while (0)
  if (lds_tables) { if (vec == 4) LQ_SCAN_K(true, 4); else LQ_SCAN_K(true, 1); }
  else            { if (vec == 4) LQ_SCAN_K(false, 4); else LQ_SCAN_K(false, 1); }
#undef LQ_SCAN_K
#undef LQ_SCAN
  LQ_LAUNCH_CHECK("scan_kernel");
  return launch_fold(a, static_cast<int>(blocks), s);
}


int launch_groupby_agg(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                       const uint8_t* const* mask, const int32_t* const* code, const int32_t* card,
                       int32_t n_preds, const lq_range_pred* preds, int32_t M, const lq_measure* meas,
                       int64_t* sums, int64_t* mins, int64_t* maxs, int64_t* counts, int32_t G, void* ws,
                       bool reuse_tables, hipStream_t s) {
  GbArgs a{};
  AggExtra x{};
  a.n = n; a.K = K; a.fact_mask = nullptr; a.M = M; a.G = G;
  a.sums = reinterpret_cast<unsigned long long*>(sums);
  a.counts = reinterpret_cast<unsigned long long*>(counts);
  x.mins = reinterpret_cast<unsigned long long*>(mins);
  x.maxs = reinterpret_cast<unsigned long long*>(maxs);
  a.packed = static_cast<uint8_t*>(ws);
  a.partial = reinterpret_cast<unsigned long long*>(a.packed + groupby_tables_bytes(K, rows));
  bool vec_ok = true;
  for (int k = 0; k < K; ++k) {
    a.d[k].fk = fks[k];
    a.d[k].mask = mask ? mask[k] : nullptr;
    a.d[k].code = code ? code[k] : nullptr;
    a.d[k].rows = rows[k];
    a.d[k].card = (code && code[k]) ? card[k] : 1;
  }
  {
    int32_t stride = 1;
    for (int k = K - 1; k >= 0; --k) {
      const bool grouping = code && code[k];
      a.d[k].stride = grouping ? stride : 0;
      if (grouping) stride *= card[k];
    }
  }
  x.n_preds = n_preds;
  for (int k = 0; k < K; ++k) vec_ok = vec_ok && aligned(fks[k], 16);
  for (int q = 0; q < n_preds; ++q) { x.pcol[q] = preds[q].col; x.lo[q] = preds[q].lo; x.hi[q] = preds[q].hi; vec_ok = vec_ok && aligned(preds[q].col, 16); }
  for (int m = 0; m < M; ++m) {
    a.meas[m] = meas[m].a; x.op[m] = meas[m].op; x.b[m] = meas[m].b ? meas[m].b : meas[m].a;
    vec_ok = vec_ok && aligned(a.meas[m], 16) && aligned(x.b[m], 16);
  }
  if (static_cast<int64_t>(3 * M + 1) * G > GROUPBY_LDS_ACCUMULATORS) {   // accumulators in memory
    const GlobalOut o{a.sums, a.counts, reinterpret_cast<long long*>(mins), reinterpret_cast<long long*>(maxs)};
    size_t prefix = 0;
    const size_t pk = plan_tables(K, rows, mask, code, card, a.d, LDS_BUDGET, &prefix);
    if (pk > 0xffffffffull) return fail(LQ_ERR_UNSUPPORTED, "group-by: dimension side tables exceed 4 GiB");
    a.packed_bytes = static_cast<uint32_t>(pk);
    int rc0;
    if ((rc0 = launch_init_outputs(o, M, G, s))) return rc0;
    if (n == 0) return LQ_OK;
    if (!reuse_tables && (rc0 = launch_pack(a, s))) return rc0;
    return launch_scan_global(a, x, o, prefix, vec_ok, s);
  }
  const int n_acc = (3 * M + 1) * G;
  const size_t acc_bytes = round_up(static_cast<size_t>(n_acc) * 8, 16);
  size_t lds_prefix = 0;
  const size_t packed = plan_tables(K, rows, mask, code, card, a.d, LDS_BUDGET - acc_bytes, &lds_prefix);
  if (packed > 0xffffffffull) return fail(LQ_ERR_UNSUPPORTED, "group-by: dimension side tables exceed 4 GiB");
  a.packed_bytes = static_cast<uint32_t>(packed);
  const int cus = num_cus();
  // Small dimension tables (up to 16 KB of masks and codes in all, LDS-resident once encoded): every scan
  // workgroup encodes them itself, which saves the separate launch.
  size_t raw_bytes = 0;
  for (int k = 0; k < K; ++k)
    raw_bytes += static_cast<size_t>(rows[k]) * ((a.d[k].mask ? 1 : 0) + (a.d[k].code ? 4 : 0));
  const bool pack_here = !reuse_tables && n > 0 && lds_prefix == packed && raw_bytes <= 16 * 1024;
  if (!reuse_tables && !pack_here) {
    const int rc0 = launch_pack(a, s);
    if (rc0) return rc0;
  }
  const unsigned fold_blocks = static_cast<unsigned>((n_acc + FOLD_AGG_THREADS / 64 - 1) / (FOLD_AGG_THREADS / 64));
  unsigned blocks = 0;
  if (n > 0) {
    constexpr int VEC = 4;
    const bool lds_tables = lds_prefix == packed;
    const size_t lds = acc_bytes + (lds_tables ? packed : 0);
    const int per_cu = lds * 2 <= 160 * 1024 ? 2 : 1;
    const int64_t n_vec = (n + VEC - 1) / VEC;
    int64_t b = std::max<int64_t>(1, std::min<int64_t>((n_vec + SCAN_THREADS - 1) / SCAN_THREADS, static_cast<int64_t>(cus) * per_cu));
    b = std::min<int64_t>(b, groupby_max_workgroups());
    int64_t pb = (n_vec + b - 1) / b;
    pb = std::max<int64_t>(SCAN_THREADS, (pb + SCAN_THREADS - 1) / SCAN_THREADS * SCAN_THREADS);
    b = std::max<int64_t>(1, (n_vec + pb - 1) / pb);
    blocks = static_cast<unsigned>(b);
    // Common shapes: one measure, up to two predicates, every side table a byte table or a bitmap in LDS.
    if (M == 1 && n_preds <= 2 && vec_ok && lds_tables && K >= 1) {
      AggFastArgs fx{};
      FastLaunch L{};
      bool ok = true;
      int slot = 0;
      for (int run = 0; run < 2 && ok; ++run)          // byte tables first, then bitmaps
        for (int k = 0; k < K; ++k) {
          const int kind = a.d[k].kind;
          if (kind != DK_BYTE && kind != DK_BITMAP) { ok = false; break; }
          if (kind != (run == 0 ? DK_BYTE : DK_BITMAP)) continue;
          fx.f.fk[slot] = a.d[k].fk; fx.f.off[slot] = a.d[k].off; fx.f.stride[slot] = a.d[k].stride;
          ++slot;
          if (run == 0) ++L.nbl; else ++L.nml;
        }
      if (ok) {
        fx.f.n = n; fx.f.packed = a.packed; fx.f.lds_bytes = static_cast<uint32_t>(packed); fx.f.G = G; fx.f.partial = a.partial;
        fx.f.meas[0] = a.meas[0];
        fx.b = x.b[0]; fx.op = x.op[0];
        for (int q = 0; q < n_preds; ++q) { fx.pcol[q] = x.pcol[q]; fx.lo[q] = x.lo[q]; fx.hi[q] = x.hi[q]; }
        fx.minmax = (mins || maxs) ? 1 : 0;
        L.lds = lds; L.s = s; L.M = 1; L.blocks = blocks; L.per_block = pb;
        const int rc = launch_agg_fast(a, fx, L, n_preds, pack_here ? 1 : 0);
        if (rc > 0) return rc;
        if (rc == 0) {
          hipLaunchKernelGGL(fold_agg_kernel, dim3(fold_blocks), dim3(FOLD_AGG_THREADS), 0, s, a, x, static_cast<int>(blocks));
          LQ_LAUNCH_CHECK("fold_agg_kernel");
          return LQ_OK;
        }
      }
    }
#define LQ_AGG(LT, KM)                                                                           \
  do {                                                                                           \
    if (lds > 64 * 1024)                                                                         \
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&agg_scan_kernel<LT, 4, KM>), \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
    hipLaunchKernelGGL((agg_scan_kernel<LT, 4, KM>), dim3(blocks), dim3(SCAN_THREADS), lds, s, a, x, pb, \
                       vec_ok ? 1 : 0, pack_here ? 1 : 0);                                       \
  } while (0)
    if (lds_tables) { if (K <= 2) LQ_AGG(true, 2); else if (K <= 4) LQ_AGG(true, 4); else LQ_AGG(true, 8); }
    else            { if (K <= 2) LQ_AGG(false, 2); else if (K <= 4) LQ_AGG(false, 4); else LQ_AGG(false, 8); }
#undef LQ_AGG
    LQ_LAUNCH_CHECK("agg_scan_kernel");
  }
  hipLaunchKernelGGL(fold_agg_kernel, dim3(fold_blocks), dim3(FOLD_AGG_THREADS), 0, s, a, x, static_cast<int>(blocks));
  LQ_LAUNCH_CHECK("fold_agg_kernel");
  return LQ_OK;
}

}  // namespace lq
