// Key -> row mapping for the MM-Join (Algorithm 1): the "domain generation" step that turns the
// key values of a fact column into row numbers of the dimension table, i.e. into the one-nonzero-
// per-row matrix I that the fused paths consume as an int32 column.
//
// The paper builds a sorted key domain and looks keys up in it (two binary searches per join,
// its measured bottleneck) and proposes to cache the domain of the rarely changing side.  Here the
// cached object lives in a caller-owned buffer and takes one of two forms, chosen when it is built:
//   * direct: when the dimension keys span a range no wider than the buffer has 4-byte cells
//     (at least four times the key count; surrogate keys 1..r are the common case) the position of
//     a key in the domain is key - smallest key, and the buffer is the array "row of that key or -1":
//     one 4-byte read per fact row, no comparison, no probing;
//   * hashed: otherwise an open-addressing table over the keys (capacity a power of two of at least
//     twice the key count, linear probing, 8-byte slots "key << 32 | row"): one or two probes per
//     fact row instead of log2(r) dependent searches.
// Both take inserts for incremental updates (a direct map only inside its window), and the fact
// side streams through once.  A key that is not in the map gives -1 (the row does not appear in
// the join result, Section 2.3.2).  The row-mapping matrices I_R / I_S of Section 2.3.3 (COO index
// vectors aligned with m = <0..nnz-1>) come from a stable compaction of the matches.
#include "lq_common.h"

namespace lq {
namespace {

typedef unsigned long long u64;
constexpr u64 EMPTY = 0xffffffffffffffffull;
constexpr size_t HEADER = 256;
constexpr unsigned FLAG_DUPLICATE = 1u, FLAG_FULL = 2u, FLAG_WINDOW = 4u;
// The first bytes of the buffer; the cells / slots follow at byte HEADER.
struct Header {
  u64 capacity;            // 8-byte slots (= 2 * capacity 4-byte cells)
  unsigned flags;          // FLAG_* raised by inserts
  int32_t direct;          // 1: cells indexed by key - base
  int32_t base;
  int32_t min_key, max_key;   // of the keys given to the build
};

__device__ __forceinline__ uint32_t slot_of(int32_t key, uint32_t shift) {
  return (static_cast<uint32_t>(key) * 0x9E3779B1u) >> shift;
}

__global__ __launch_bounds__(256) void keymap_clear_kernel(u64* slots, u64 capacity, Header* header) {
  const u64 i = static_cast<u64>(blockIdx.x) * 256 + threadIdx.x;
  if (i < capacity) slots[i] = EMPTY;                     // all ones: an empty slot, and two cells holding -1
  if (i == 0) {
    header->capacity = capacity; header->flags = 0u; header->direct = 0; header->base = 0;
    header->min_key = 0x7fffffff; header->max_key = static_cast<int32_t>(0x80000000u);
  }
}

__global__ __launch_bounds__(256) void keymap_minmax_kernel(const int32_t* __restrict__ keys, int64_t r, Header* header) {
  int32_t lo = 0x7fffffff, hi = static_cast<int32_t>(0x80000000u);
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < r; i += static_cast<int64_t>(gridDim.x) * 256) {
    const int32_t k = keys[i];
    lo = min(lo, k); hi = max(hi, k);
  }
  for (int off = 32; off > 0; off >>= 1) {
    lo = min(lo, __shfl_xor(lo, off, 64));
    hi = max(hi, __shfl_xor(hi, off, 64));
  }
  __shared__ int32_t wlo[4], whi[4];
  if ((threadIdx.x & 63) == 0) { wlo[threadIdx.x >> 6] = lo; whi[threadIdx.x >> 6] = hi; }
  __syncthreads();
  if (threadIdx.x == 0) {                                 // one pair of atomics per workgroup
    atomicMin(&header->min_key, min(min(wlo[0], wlo[1]), min(wlo[2], wlo[3])));
    atomicMax(&header->max_key, max(max(whi[0], whi[1]), max(whi[2], whi[3])));
  }
}

// A key range that fits the buffer's 4-byte cells makes the map direct.
__device__ __forceinline__ bool range_fits(int32_t lo, int32_t hi, u64 capacity) {
  return hi >= lo && static_cast<u64>(static_cast<int64_t>(hi) - lo) < 2 * capacity;
}

// BUILD: called right after the min / max pass; every thread derives the form of the map from the
// key range and the first one records it.  Otherwise (incremental insert) the recorded form is used.
template <bool BUILD>
__global__ __launch_bounds__(256) void keymap_insert_kernel(u64* slots, uint32_t mask, uint32_t shift,
                                                            const int32_t* __restrict__ keys, int64_t r,
                                                            int64_t row0, Header* header) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  bool direct;
  int32_t base;
  if (BUILD) {
    const int32_t lo = header->min_key, hi = header->max_key;
    direct = range_fits(lo, hi, static_cast<u64>(mask) + 1);
    base = direct ? lo : 0;
    if (i == 0) { header->direct = direct ? 1 : 0; header->base = base; }
  } else {
    direct = header->direct != 0;
    base = header->base;
  }
  if (i >= r) return;
  const int32_t key = keys[i];
  if (direct) {
    const int64_t cell = static_cast<int64_t>(key) - base;
    if (cell < 0 || cell >= 2 * (static_cast<int64_t>(mask) + 1)) { atomicOr(&header->flags, FLAG_WINDOW); return; }
    const int old = atomicCAS(reinterpret_cast<int*>(slots) + cell, -1, static_cast<int>(row0 + i));
    if (old != -1) atomicOr(&header->flags, FLAG_DUPLICATE);
    if (!BUILD) atomicMax(&header->max_key, key);         // keeps "cells in use" current for the LDS copy
    return;
  }
  const u64 mine = (static_cast<u64>(static_cast<uint32_t>(key)) << 32) | static_cast<uint32_t>(row0 + i);
  uint32_t s = slot_of(key, shift) & mask;
  for (uint32_t probes = 0; probes <= mask; ++probes) {           // bounded: at most one sweep of the table
    const u64 old = atomicCAS(&slots[s], EMPTY, mine);
    if (old == EMPTY) return;
    if (static_cast<int32_t>(old >> 32) == key) { atomicOr(&header->flags, FLAG_DUPLICATE); return; }
    s = (s + 1) & mask;
  }
  atomicOr(&header->flags, FLAG_FULL);
}

// What the lookup kernels need to know about the map (read once per thread from the header).
struct Form { bool direct; int32_t base; int64_t cells; };
__device__ __forceinline__ Form form_of(const Header* header, uint32_t mask) {
  Form f;
  f.direct = header->direct != 0;
  f.base = header->base;
  f.cells = 2 * (static_cast<int64_t>(mask) + 1);
  return f;
}

__device__ __forceinline__ int32_t probe(const u64* slots, uint32_t mask, uint32_t shift, int32_t key) {
  uint32_t s = slot_of(key, shift) & mask;
  for (uint32_t probes = 0; probes <= mask; ++probes) {           // bounded: at most one sweep of the table
    const u64 v = slots[s];
    if (v == EMPTY) return -1;
    if (static_cast<int32_t>(v >> 32) == key) return static_cast<int32_t>(v & 0xffffffffu);
    s = (s + 1) & mask;
  }
  return -1;
}

template <typename SLOTS>
__device__ __forceinline__ int32_t find(SLOTS slots, uint32_t mask, uint32_t shift, const Form& f, int32_t key) {
  if (f.direct) {
    const int64_t cell = static_cast<int64_t>(key) - f.base;
    return (cell >= 0 && cell < f.cells) ? reinterpret_cast<const int32_t*>(slots)[cell] : -1;
  }
  return probe(slots, mask, shift, key);
}

typedef int v4i __attribute__((ext_vector_type(4)));

// Four keys per thread (one 16-byte load, four probes in flight); the tail is done one by one.
__global__ __launch_bounds__(256) void keymap_lookup_kernel(const Header* __restrict__ header,
                                                            const u64* __restrict__ slots, uint32_t mask,
                                                            uint32_t shift, const int32_t* __restrict__ keys,
                                                            int64_t n, int32_t* __restrict__ fk, int vec_ok) {
  const Form f = form_of(header, mask);
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (vec_ok) {
    const int64_t n4 = n / 4;
    if (t < n4) {
      const v4i k = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(keys) + t);
      v4i r;
#pragma unroll
      for (int q = 0; q < 4; ++q) r[q] = find(slots, mask, shift, f, k[q]);
      __builtin_nontemporal_store(r, reinterpret_cast<v4i*>(fk) + t);
    } else if (t - n4 < n - 4 * n4) {
      const int64_t i = 4 * n4 + (t - n4);
      fk[i] = find(slots, mask, shift, f, keys[i]);
    }
  } else if (t < n) {
    fk[t] = find(slots, mask, shift, f, keys[t]);
  }
}

// Small maps: every workgroup copies the whole cell / slot array into LDS and serves a contiguous
// slice of the fact keys from there, so lookups never leave the compute unit.  Two 16-byte key
// loads are in flight per thread.
constexpr int LDS_LOOKUP_THREADS = 1024;
__global__ __launch_bounds__(LDS_LOOKUP_THREADS) void keymap_lookup_lds_kernel(const Header* __restrict__ header,
                                                                              const u64* __restrict__ slots,
                                                                              uint32_t mask, uint32_t shift,
                                                                              const int32_t* __restrict__ keys,
                                                                              int64_t n, int32_t* __restrict__ fk,
                                                                              int64_t per_block) {
  extern __shared__ __align__(16) u64 lds_slots[];
  Form f = form_of(header, mask);
  if (f.direct) f.cells = static_cast<int64_t>(header->max_key) - f.base + 1;   // cells beyond hold -1 and are not copied
  {
    const uint4* src = reinterpret_cast<const uint4*>(slots);
    uint4* dst = reinterpret_cast<uint4*>(lds_slots);
    // a direct map only uses the cells up to its largest key
    const uint32_t pieces = f.direct ? static_cast<uint32_t>((static_cast<int64_t>(header->max_key) - f.base) / 4 + 1)
                                     : (mask + 1u) / 2u;
    for (uint32_t i = threadIdx.x; i < pieces; i += LDS_LOOKUP_THREADS) dst[i] = src[i];
  }
  __syncthreads();
  const int64_t n4 = n / 4;
  const int64_t lo = static_cast<int64_t>(blockIdx.x) * per_block, hi = min(n4, lo + per_block);
  for (int64_t t = lo + threadIdx.x; t < hi; t += 2 * LDS_LOOKUP_THREADS) {
    const int64_t t1 = t + LDS_LOOKUP_THREADS;
    const v4i k0 = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(keys) + t);
    v4i k1 = {0, 0, 0, 0};
    if (t1 < hi) k1 = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(keys) + t1);
    v4i r;
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = find(lds_slots, mask, shift, f, k0[q]);
    __builtin_nontemporal_store(r, reinterpret_cast<v4i*>(fk) + t);
    if (t1 < hi) {
#pragma unroll
      for (int q = 0; q < 4; ++q) r[q] = find(lds_slots, mask, shift, f, k1[q]);
      __builtin_nontemporal_store(r, reinterpret_cast<v4i*>(fk) + t1);
    }
  }
  if (blockIdx.x == 0) {
    const int64_t i = 4 * n4 + threadIdx.x;
    if (i < n) fk[i] = find(lds_slots, mask, shift, f, keys[i]);
  }
}

// ---- stable compaction of the matches: COO index vectors of I --------------------------------
constexpr int CB = 1024;   // rows per workgroup

__global__ __launch_bounds__(CB) void compact_count_kernel(const int32_t* __restrict__ fk, int64_t n,
                                                           int64_t* __restrict__ block_count) {
  __shared__ int wave_cnt[CB / 64];
  const int64_t i = static_cast<int64_t>(blockIdx.x) * CB + threadIdx.x;
  const bool hit = i < n && fk[i] >= 0;
  const int c = __popcll(__ballot(hit));
  if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < CB / 64; ++w) t += wave_cnt[w];
    block_count[blockIdx.x] = t;
  }
}

// One workgroup: exclusive scan of the per-workgroup counts (in place) and the total.
__global__ __launch_bounds__(1024) void compact_scan_kernel(int64_t* block_count, int64_t nb, int64_t* nnz) {
  __shared__ int64_t part[1024];
  const int tid = threadIdx.x;
  const int64_t per = (nb + 1023) / 1024;
  const int64_t lo = std::min<int64_t>(nb, tid * per), hi = std::min<int64_t>(nb, lo + per);
  int64_t s = 0;
  for (int64_t b = lo; b < hi; ++b) s += block_count[b];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) {
    int64_t run = 0;
    for (int t = 0; t < 1024; ++t) { const int64_t v = part[t]; part[t] = run; run += v; }
    *nnz = run;
  }
  __syncthreads();
  int64_t run = part[tid];
  for (int64_t b = lo; b < hi; ++b) { const int64_t v = block_count[b]; block_count[b] = run; run += v; }
}

__global__ __launch_bounds__(CB) void compact_scatter_kernel(const int32_t* __restrict__ fk, int64_t n,
                                                             const int64_t* __restrict__ block_off,
                                                             int64_t* __restrict__ rows, int32_t* __restrict__ cols) {
  __shared__ int wave_off[CB / 64];
  const int64_t i = static_cast<int64_t>(blockIdx.x) * CB + threadIdx.x;
  const int32_t v = i < n ? fk[i] : -1;
  const bool hit = v >= 0;
  const u64 bal = __ballot(hit);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) wave_off[wave] = __popcll(bal);
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int w = 0; w < CB / 64; ++w) { const int c = wave_off[w]; wave_off[w] = run; run += c; }
  }
  __syncthreads();
  if (hit) {
    const int64_t m = block_off[blockIdx.x] + wave_off[wave] + __popcll(bal & ((1ull << lane) - 1ull));
    rows[m] = i;
    cols[m] = v;
  }
}

struct Geometry { u64 capacity; uint32_t mask, shift; };
bool geometry(size_t table_bytes, Geometry* g) {
  if (table_bytes < HEADER + 16) return false;
  u64 cap = 2;
  while (cap * 2 * 8 + HEADER <= table_bytes && cap < (1ull << 31)) cap <<= 1;
  int log2 = 0;
  while ((1ull << log2) < cap) ++log2;
  g->capacity = cap; g->mask = static_cast<uint32_t>(cap - 1); g->shift = static_cast<uint32_t>(32 - log2);
  return true;
}

// Waits for the stream and turns the flags raised by inserts into an error.
int check_flags(const Header* header, hipStream_t s) {
  unsigned h = 0;
  LQ_HIP_TRY(hipMemcpyAsync(&h, &header->flags, sizeof(h), hipMemcpyDeviceToHost, s));
  LQ_HIP_TRY(hipStreamSynchronize(s));
  if (h & FLAG_DUPLICATE) return fail(LQ_ERR_DUPLICATE_KEY, "the dimension key column holds a value twice");
  if (h & FLAG_FULL) return fail(LQ_ERR_WORKSPACE, "key map is full");
  if (h & FLAG_WINDOW) return fail(LQ_ERR_WORKSPACE, "a key lies outside the window of this direct-address map: rebuild the map with all keys");
  return LQ_OK;
}

}  // namespace
}  // namespace lq

using namespace lq;

extern "C" {

size_t lq_keymap_bytes(int64_t max_keys) {
  if (max_keys < 0 || max_keys > (1ll << 29)) return 0;
  u64 cap = 2;
  while (cap < static_cast<u64>(max_keys) * 2) cap <<= 1;
  return HEADER + cap * 8;
}

int lq_keymap_insert(void* table, size_t table_bytes, const int32_t* keys, int64_t n_keys, int64_t first_row,
                     uint32_t flags, void* hip_stream) {
  clear_error();
  Geometry g;
  if (!table || !aligned(table, 256) || !geometry(table_bytes, &g)) return fail(LQ_ERR_WORKSPACE, "key map buffer is NULL, misaligned or too small");
  if (n_keys < 0 || first_row < 0 || first_row + n_keys > 0x7fffffffLL) return fail(LQ_ERR_SHAPE, "row numbers do not fit int32");
  if (n_keys > 0 && (!keys || !aligned(keys, 4))) return fail(LQ_ERR_NULL, "keys is NULL or misaligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Header* header = static_cast<Header*>(table);
  u64* slots = static_cast<u64*>(table) + HEADER / 8;
  if (n_keys > 0) {
    hipLaunchKernelGGL(keymap_insert_kernel<false>, dim3(static_cast<unsigned>((n_keys + 255) / 256)), dim3(256), 0, s,
                       slots, g.mask, g.shift, keys, n_keys, first_row, header);
    LQ_LAUNCH_CHECK("keymap_insert_kernel");
  }
  if (flags & LQ_CHECK_KEYS) return check_flags(header, s);
  return LQ_OK;
}

int lq_keymap_build(void* table, size_t table_bytes, const int32_t* keys, int64_t n_keys, uint32_t flags,
                    void* hip_stream) {
  clear_error();
  Geometry g;
  if (!table || !aligned(table, 256) || !geometry(table_bytes, &g)) return fail(LQ_ERR_WORKSPACE, "key map buffer is NULL, misaligned or too small");
  if (n_keys < 0 || static_cast<u64>(n_keys) * 2 > g.capacity) return fail(LQ_ERR_WORKSPACE, "key map buffer holds %llu slots, %lld keys need twice as many", (unsigned long long)g.capacity, (long long)n_keys);
  if (n_keys > 0x7fffffffLL) return fail(LQ_ERR_SHAPE, "row numbers do not fit int32");
  if (n_keys > 0 && (!keys || !aligned(keys, 4))) return fail(LQ_ERR_NULL, "keys is NULL or misaligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Header* header = static_cast<Header*>(table);
  u64* slots = static_cast<u64*>(table) + HEADER / 8;
  hipLaunchKernelGGL(keymap_clear_kernel, dim3(static_cast<unsigned>((g.capacity + 255) / 256)), dim3(256), 0, s,
                     slots, g.capacity, header);
  LQ_LAUNCH_CHECK("keymap_clear_kernel");
  if (n_keys > 0) {
    const unsigned mm_blocks = static_cast<unsigned>(std::min<int64_t>((n_keys + 1023) / 1024, 256));
    hipLaunchKernelGGL(keymap_minmax_kernel, dim3(mm_blocks), dim3(256), 0, s, keys, n_keys, header);
    LQ_LAUNCH_CHECK("keymap_minmax_kernel");
    hipLaunchKernelGGL(keymap_insert_kernel<true>, dim3(static_cast<unsigned>((n_keys + 255) / 256)), dim3(256), 0, s,
                       slots, g.mask, g.shift, keys, n_keys, static_cast<int64_t>(0), header);
    LQ_LAUNCH_CHECK("keymap_insert_kernel");
  }
  if (flags & LQ_CHECK_KEYS) return check_flags(header, s);
  return LQ_OK;
}

int lq_keymap_lookup(const void* table, size_t table_bytes, const int32_t* fact_keys, int64_t n, int32_t* fk,
                     void* hip_stream) {
  clear_error();
  Geometry g;
  if (!table || !aligned(table, 256) || !geometry(table_bytes, &g)) return fail(LQ_ERR_WORKSPACE, "key map buffer is NULL, misaligned or too small");
  if (n < 0) return fail(LQ_ERR_SHAPE, "n < 0");
  if (n == 0) return LQ_OK;
  if (!fact_keys || !fk || !aligned(fact_keys, 4) || !aligned(fk, 4)) return fail(LQ_ERR_NULL, "fact_keys or fk is NULL or misaligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const Header* header = static_cast<const Header*>(table);
  const u64* slots = static_cast<const u64*>(table) + HEADER / 8;
  const int vec_ok = aligned(fact_keys, 16) && aligned(fk, 16);
  const size_t slot_bytes = static_cast<size_t>(g.capacity) * 8;
  if (vec_ok && slot_bytes <= 128 * 1024 && n >= (1 << 20)) {
    const int64_t n4 = n / 4;
    const int per_cu = slot_bytes <= 64 * 1024 ? 2 : 1;       // workgroups whose copies fit one compute unit's LDS
    const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>((n4 + LDS_LOOKUP_THREADS - 1) / LDS_LOOKUP_THREADS,
                                                                  static_cast<int64_t>(num_cus()) * per_cu));
    const int64_t per_block = (n4 + blocks - 1) / blocks;
    if (slot_bytes > 64 * 1024)
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&keymap_lookup_lds_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(slot_bytes)));
    hipLaunchKernelGGL(keymap_lookup_lds_kernel, dim3(static_cast<unsigned>(blocks)), dim3(LDS_LOOKUP_THREADS), slot_bytes, s,
                       header, slots, g.mask, g.shift, fact_keys, n, fk, per_block);
    LQ_LAUNCH_CHECK("keymap_lookup_lds_kernel");
    return LQ_OK;
  }
  const int64_t threads = vec_ok ? n / 4 + n % 4 : n;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
  hipLaunchKernelGGL(keymap_lookup_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, header, slots, g.mask,
                     g.shift, fact_keys, n, fk, vec_ok);
  LQ_LAUNCH_CHECK("keymap_lookup_kernel");
  return LQ_OK;
}

size_t lq_compact_workspace_bytes(int64_t n) {
  if (n < 0) return 0;
  return round_up(static_cast<size_t>((n + CB - 1) / CB + 1) * 8, 256);
}

int lq_compact_matches(const int32_t* fk, int64_t n, int64_t* rows, int32_t* cols, int64_t* nnz, void* ws,
                       size_t ws_bytes, void* hip_stream) {
  clear_error();
  if (n < 0) return fail(LQ_ERR_SHAPE, "n < 0");
  if (!nnz || !aligned(nnz, 8)) return fail(LQ_ERR_NULL, "nnz is NULL or misaligned");
  if (n > 0 && (!fk || !rows || !cols)) return fail(LQ_ERR_NULL, "fk, rows or cols is NULL");
  if (!aligned(rows, 8) || !aligned(cols, 4) || !aligned(fk, 4)) return fail(LQ_ERR_SHAPE, "misaligned array");
  if (!ws || !aligned(ws, 256) || ws_bytes < lq_compact_workspace_bytes(n)) return fail(LQ_ERR_WORKSPACE, "compaction needs %zu bytes of 256-byte aligned workspace", lq_compact_workspace_bytes(n));
  const int64_t nb = (n + CB - 1) / CB;
  if (nb > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int64_t* counts = static_cast<int64_t*>(ws);
  if (nb > 0) {
    hipLaunchKernelGGL(compact_count_kernel, dim3(static_cast<unsigned>(nb)), dim3(CB), 0, s, fk, n, counts);
    LQ_LAUNCH_CHECK("compact_count_kernel");
  }
  hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(1024), 0, s, counts, nb, nnz);
  LQ_LAUNCH_CHECK("compact_scan_kernel");
  if (nb > 0) {
    hipLaunchKernelGGL(compact_scatter_kernel, dim3(static_cast<unsigned>(nb)), dim3(CB), 0, s, fk, n, counts, rows, cols);
    LQ_LAUNCH_CHECK("compact_scatter_kernel");
  }
  return LQ_OK;
}

}  // extern "C"
