// The wider aggregate (fact-side range predicates, a measure that is a column or the product / difference of
// two, SUM / MIN / MAX / COUNT per group; Sections 2.2-2.4) on a compile-time specialised scan: the shapes of
// the benchmark's query groups -- one to four joins whose side tables all sit in LDS, up to two predicates
// on fact columns, one measure.  Number of byte tables, bitmaps and predicates are template parameters, the
// key and predicate columns of the next step are requested before the current one is evaluated, the measure
// columns are only touched where a lane has a survivor.  Same accumulator layout and partial rows as the
// run-time generic scan, so the same fold finishes the call.
#include "groupby_fast.h"

namespace lq {
namespace {

// Accumulators (LDS, partial rows): [sum G | count G | min G | max G].
// DEFER: the measure columns of a step are requested when its survivors are known and added one step later, so
// that their latency passes under the next step's keys instead of ending every step.  It shortens a thread's
// critical path by one memory latency per step, which is what a scan of a few steps per thread is made of
// (6e6 rows: 3 steps, 22.9 -> 18.5 us); over many steps the other wavefronts cover that latency anyway and the
// later, second divergent region costs throughput (the same change made the plain group-by 11 % slower at 9.6e7
// rows), so long scans consume their measures at once.
template <int NBL, int NML, int NP, bool DEFER>
__global__ __launch_bounds__(SCAN_THREADS) void agg_fast_kernel(GbArgs a, AggFastArgs x, int64_t per_block, int pack_here) {
  extern __shared__ __align__(16) uint8_t smem[];
  constexpr int ND = NBL + NML, NC = ND + NP;
  const FastArgs& f = x.f;
  const int G = f.G, n_acc = 4 * G;
  long long* acc = reinterpret_cast<long long*>(smem);
  uint8_t* tab = smem + round_up(static_cast<size_t>(n_acc) * 8, 16);
  const int tid = threadIdx.x;

  const int64_t n_vec = f.n / 4;
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  int64_t v = v_begin + tid;
  auto column = [&](int c) { return c < ND ? f.fk[c] : x.pcol[c - ND]; };
  v4i cur[NC], nxt[NC];
  if (v < v_end) {
#pragma unroll
    for (int c = 0; c < NC; ++c) cur[c] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(column(c)) + v);
  }
  for (int i = tid; i < n_acc; i += SCAN_THREADS) acc[i] = i < 2 * G ? 0LL : (i < 3 * G ? AGG_MIN_INIT : AGG_MAX_INIT);
  if (pack_here) {      // tiny dimension tables: every workgroup encodes its own copy, workgroup 0 also leaves one in the workspace
    pack_tables(a, tab, tid, SCAN_THREADS);
    if (blockIdx.x == 0) {
      __syncthreads();
      uint4* dst = reinterpret_cast<uint4*>(a.packed);
      const uint4* src = reinterpret_cast<const uint4*>(tab);
      for (uint32_t i = tid; i < a.packed_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
    }
  } else {
    const uint4* src = reinterpret_cast<const uint4*>(f.packed);
    uint4* dst = reinterpret_cast<uint4*>(tab);
    for (uint32_t i = tid; i < f.lds_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
  }
  __syncthreads();

  auto measure = [&](int32_t av, int32_t bv) {
    long long t = av;
    if (x.op == 1) t *= static_cast<long long>(bv);
    else if (x.op == 2) t -= static_cast<long long>(bv);
    return t;
  };
  auto add = [&](int32_t g, long long t) {
    atomicAdd(reinterpret_cast<unsigned long long*>(&acc[g]), static_cast<unsigned long long>(t));
    atomicAdd(reinterpret_cast<unsigned long long*>(&acc[G + g]), 1ull);
    if (x.minmax) {
      atomicMin(&acc[2 * G + g], t);
      atomicMax(&acc[3 * G + g], t);
    }
  };

  uint32_t pending = 0;         // bit q: row q of the previous step survived (DEFER)
  int32_t pg[4] = {0, 0, 0, 0};
  v4i pav = {0, 0, 0, 0}, pbv = {0, 0, 0, 0};
  auto flush = [&]() {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (pending & (1u << q)) add(pg[q], measure(pav[q], pbv[q]));
  };
  while (v < v_end) {
    const int64_t vn = v + SCAN_THREADS;
    if (vn < v_end) {
#pragma unroll
      for (int c = 0; c < NC; ++c) nxt[c] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(column(c)) + vn);
    }
    int32_t g[4];
    uint32_t alive_bits = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bool alive = true;
#pragma unroll
      for (int p = 0; p < NP; ++p) alive = alive && cur[ND + p][q] >= x.lo[p] && cur[ND + p][q] <= x.hi[p];
      int32_t j[ND > 0 ? ND : 1];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = cur[k][q];
      g[q] = 0;
      classify_fast<NBL, NML, 0, 0>(f, tab, j, alive, g[q]);
      alive_bits |= alive ? (1u << q) : 0u;
    }
    if (DEFER && pending) flush();
    pending = alive_bits;
    if (pending) {
#pragma unroll
      for (int q = 0; q < 4; ++q) pg[q] = g[q];
      pav = *(reinterpret_cast<const v4i*>(f.meas[0]) + v);
      pbv = pav;
      if (x.op != 0) pbv = *(reinterpret_cast<const v4i*>(x.b) + v);
      if (!DEFER) flush();
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) cur[c] = nxt[c];
    v = vn;
  }
  if (DEFER && pending) flush();
  // ragged tail (n % 4 rows)
  if (blockIdx.x == 0) {
    const int64_t i = n_vec * 4 + tid;
    if (i < f.n) {
      bool alive = true;
#pragma unroll
      for (int p = 0; p < NP; ++p) alive = alive && x.pcol[p][i] >= x.lo[p] && x.pcol[p][i] <= x.hi[p];
      int32_t j[ND > 0 ? ND : 1];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = f.fk[k][i];
      int32_t g = 0;
      classify_fast<NBL, NML, 0, 0>(f, tab, j, alive, g);
      if (alive) add(g, measure(f.meas[0][i], x.op != 0 ? x.b[i] : 0));
    }
  }
  __syncthreads();
  long long* mine = reinterpret_cast<long long*>(f.partial) + static_cast<size_t>(blockIdx.x) * n_acc;
  for (int i = tid; i < n_acc; i += SCAN_THREADS) mine[i] = acc[i];
}

template <int NBL, int NML, int NP>
int agg_fast_inst(const GbArgs& a, const AggFastArgs& x, const FastLaunch& L, int pack_here) {
  const bool defer = L.per_block <= 8 * SCAN_THREADS;          // at most eight steps per thread
  auto kernel = defer ? &agg_fast_kernel<NBL, NML, NP, true> : &agg_fast_kernel<NBL, NML, NP, false>;
  if (L.lds > 64 * 1024)
    LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(L.lds)));
  hipLaunchKernelGGL(kernel, dim3(L.blocks), dim3(SCAN_THREADS), L.lds, L.s, a, x, L.per_block, pack_here);
  LQ_LAUNCH_CHECK("agg_fast_kernel");
  return LQ_OK;
}
template <int NBL, int NML>
int agg_fast_np(const GbArgs& a, const AggFastArgs& x, const FastLaunch& L, int n_preds, int pack_here) {
  if constexpr (NBL + NML == 0) return -1;
  else {
    switch (n_preds) {
      case 0: return agg_fast_inst<NBL, NML, 0>(a, x, L, pack_here);
      case 1: return agg_fast_inst<NBL, NML, 1>(a, x, L, pack_here);
      case 2: return agg_fast_inst<NBL, NML, 2>(a, x, L, pack_here);
      default: return -1;
    }
  }
}
template <int NBL>
int agg_fast_ml(const GbArgs& a, const AggFastArgs& x, const FastLaunch& L, int n_preds, int pack_here) {
  switch (L.nml) {
    case 0: return agg_fast_np<NBL, 0>(a, x, L, n_preds, pack_here);
    case 1: return agg_fast_np<NBL, 1>(a, x, L, n_preds, pack_here);
    case 2: return agg_fast_np<NBL, 2>(a, x, L, n_preds, pack_here);
    default: return -1;
  }
}

}  // namespace

// Returns -1 when there is no instantiation for this mix of dimensions and predicates.
int launch_agg_fast(const GbArgs& a, const AggFastArgs& x, const FastLaunch& L, int n_preds, int pack_here) {
  switch (L.nbl) {
    case 0: return agg_fast_ml<0>(a, x, L, n_preds, pack_here);
    case 1: return agg_fast_ml<1>(a, x, L, n_preds, pack_here);
    case 2: return agg_fast_ml<2>(a, x, L, n_preds, pack_here);
    default: return -1;
  }
}

}  // namespace lq
