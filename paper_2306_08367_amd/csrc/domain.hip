// Group discovery (Sections 2.4.1-2.4.2) and ordering of an aggregate's result (Section 2.5).
//
// The paper finds the groups of a table with a numerical unique (one attribute) or with a
// sort-unique over tuples (several attributes), i.e. by sorting every row.  Grouping attributes of
// a star schema have few distinct values next to the number of rows (the group-by keeps at most
// 65,535 per dimension), so the rows are not sorted here: they are deduplicated through an
// open-addressing hash set whose slots name a representative row, and only the distinct tuples are
// ordered (rank = number of smaller distinct tuples, tiles of them staged in LDS).  A row's code is
// the rank of its tuple, so codes number the distinct tuples in ascending lexicographic order, as
// the sorted domain of the paper does; a dense group-by result indexed by such codes is therefore
// already ordered by the grouping attributes (the way Section 2.5 folds sorting into the matrix
// form).  Ordering by an aggregate (ORDER BY revenue DESC) is a bitonic sort of the at most 8,192
// group indices inside one workgroup.
#include "lq_common.h"

namespace lq {
namespace {

constexpr int MAX_COLS = 4;
constexpr int32_t MAX_DISTINCT = 65535;
constexpr size_t HEADER = 256;            // [0] number of distinct tuples (u32)

struct Cols {
  const int32_t* c[MAX_COLS];
  int32_t n_cols;
};

__device__ __forceinline__ uint32_t hash_row(const Cols& t, int64_t i, uint32_t shift) {
  uint32_t h = 0x811C9DC5u;
  for (int q = 0; q < t.n_cols; ++q) {
    h ^= static_cast<uint32_t>(t.c[q][i]);
    h *= 0x9E3779B1u;
    h ^= h >> 15;
  }
  return (h * 0x85EBCA6Bu) >> shift;
}
__device__ __forceinline__ bool same_tuple(const Cols& t, int64_t i, int64_t j) {
  bool eq = true;
  for (int q = 0; q < t.n_cols; ++q) eq = eq && t.c[q][i] == t.c[q][j];
  return eq;
}

__global__ __launch_bounds__(256) void domain_clear_kernel(int32_t* slots, uint32_t capacity, uint32_t* header) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < capacity) slots[i] = -1;
  if (i == 0) header[0] = 0u;
}

// Every row either finds a slot whose representative row holds the same tuple or claims an empty
// slot for itself.  Claimed slots are listed in `reps` (the first MAX_DISTINCT + 1 of them).
__global__ __launch_bounds__(256) void domain_insert_kernel(Cols t, int64_t first, int64_t rows, int32_t* slots,
                                                            uint32_t mask, uint32_t shift, uint32_t* header,
                                                            uint32_t* reps) {
  const int64_t i = first + static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= rows) return;
  uint32_t s = hash_row(t, i, shift) & mask;
  for (uint32_t probes = 0; probes <= mask; ++probes) {           // bounded: at most one sweep of the table
    int32_t v = slots[s];
    if (v < 0) {
      v = atomicCAS(&slots[s], -1, static_cast<int32_t>(i));
      if (v < 0) {
        const uint32_t idx = atomicAdd(&header[0], 1u);
        if (idx <= static_cast<uint32_t>(MAX_DISTINCT)) reps[idx] = s;
        return;
      }
    }
    if (same_tuple(t, i, v)) return;
    s = (s + 1) & mask;
  }
}

__device__ __forceinline__ bool tuple_less(const int32_t* a, const int32_t* b, int n_cols) {
  for (int q = 0; q < n_cols; ++q) {
    if (a[q] != b[q]) return a[q] < b[q];
  }
  return false;
}

// rank of distinct tuple t = number of distinct tuples below it; writes the sorted value table.
constexpr int RANK_THREADS = 256;
__global__ __launch_bounds__(RANK_THREADS) void domain_rank_kernel(Cols t, int32_t d, const int32_t* __restrict__ slots,
                                                                  const uint32_t* __restrict__ reps,
                                                                  int32_t* __restrict__ slot_rank,
                                                                  int32_t* __restrict__ values) {
  __shared__ int32_t tile[RANK_THREADS][MAX_COLS];
  const int me = blockIdx.x * RANK_THREADS + threadIdx.x;
  int32_t mine[MAX_COLS] = {0, 0, 0, 0};
  if (me < d) {
    const int64_t row = slots[reps[me]];
    for (int q = 0; q < t.n_cols; ++q) mine[q] = t.c[q][row];
  }
  int rank = 0;
  for (int base = 0; base < d; base += RANK_THREADS) {
    const int j = base + threadIdx.x;
    if (j < d) {
      const int64_t row = slots[reps[j]];
      for (int q = 0; q < t.n_cols; ++q) tile[threadIdx.x][q] = t.c[q][row];
    }
    __syncthreads();
    const int cnt = min(RANK_THREADS, d - base);
    for (int u = 0; u < cnt; ++u) rank += tuple_less(tile[u], mine, t.n_cols) ? 1 : 0;
    __syncthreads();
  }
  if (me < d) {
    slot_rank[reps[me]] = rank;
    for (int q = 0; q < t.n_cols; ++q) values[static_cast<int64_t>(rank) * t.n_cols + q] = mine[q];
  }
}

__global__ __launch_bounds__(256) void domain_encode_kernel(Cols t, int64_t rows, const int32_t* __restrict__ slots,
                                                            uint32_t mask, uint32_t shift,
                                                            const int32_t* __restrict__ slot_rank,
                                                            int32_t* __restrict__ code) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= rows) return;
  uint32_t s = hash_row(t, i, shift) & mask;
  int32_t out = -1;
  for (uint32_t probes = 0; probes <= mask; ++probes) {           // bounded; every row was inserted, so it is found
    const int32_t v = slots[s];
    if (v < 0) break;
    if (same_tuple(t, i, v)) { out = slot_rank[s]; break; }
    s = (s + 1) & mask;
  }
  code[i] = out;
}

uint32_t domain_capacity(int64_t rows) {
  uint64_t c = 1024;
  while (c < 2 * static_cast<uint64_t>(rows)) c <<= 1;
  return static_cast<uint32_t>(c);
}

// ---- ordering of the populated groups -----------------------------------------------------------
constexpr int MAX_GROUPS = 8192;
constexpr int ORDER_THREADS = 1024;
constexpr int32_t UNPOPULATED = 0x40000000;

struct OrderArgs {
  int32_t G, Gp;                          // groups, next power of two
  int32_t n_keys;
  int32_t kind[4], index[4], desc[4];
  int32_t stride[LQ_MAX_DIMS], card[LQ_MAX_DIMS];
  const long long* sums;                  // [n_measures x G]
  const long long* counts;                // [G]
};

__device__ __forceinline__ long long key_value(const OrderArgs& a, int q, int32_t g) {
  long long v;
  if (a.kind[q] == LQ_KEY_GROUP_COLUMN) v = (g / a.stride[a.index[q]]) % a.card[a.index[q]];
  else if (a.kind[q] == LQ_KEY_SUM) v = a.sums[static_cast<int64_t>(a.index[q]) * a.G + g];
  else v = a.counts[g];
  return a.desc[q] ? ~v : v;              // ~v reverses the order of signed integers without overflow
}
// Order of two groups whose first keys are equal: the remaining keys, then the group index.
// Keys 1..n_lds are served from LDS, later ones (rarely reached) from memory.
__device__ __forceinline__ bool tie_before(const OrderArgs& a, const long long* vals, int n_lds, int32_t x, int32_t y) {
  if ((x | y) & UNPOPULATED) return x < y;               // populated first, then by group index
  for (int q = 1; q < a.n_keys; ++q) {
    const long long vx = q <= n_lds ? vals[(q - 1) * a.Gp + x] : key_value(a, q, x);
    const long long vy = q <= n_lds ? vals[(q - 1) * a.Gp + y] : key_value(a, q, y);
    if (vx != vy) return vx < vy;
  }
  return x < y;
}

// Bitonic sort of (first key, group index) pairs held in LDS by position, so that a compare-exchange
// reads its two elements and nothing else unless the first keys tie.
__global__ __launch_bounds__(ORDER_THREADS) void order_groups_kernel(OrderArgs a, int n_lds, int32_t* __restrict__ order,
                                                                    int32_t* __restrict__ n_out) {
  extern __shared__ __align__(16) long long lds_ll[];
  long long* k0 = lds_ll;                                // [Gp] first key, by position
  long long* vals = k0 + a.Gp;                           // [n_lds][Gp] keys 1..n_lds, by group
  int32_t* idx = reinterpret_cast<int32_t*>(vals + static_cast<size_t>(n_lds) * a.Gp);   // [Gp] group, by position
  __shared__ int populated;
  if (threadIdx.x == 0) populated = 0;
  __syncthreads();
  int mine = 0;
  for (int g = threadIdx.x; g < a.Gp; g += ORDER_THREADS) {
    const bool pop = g < a.G && a.counts[g] > 0;
    idx[g] = pop ? g : (g | UNPOPULATED);
    k0[g] = pop ? (a.n_keys > 0 ? key_value(a, 0, g) : 0) : 0x7fffffffffffffffll;
    mine += pop ? 1 : 0;
    for (int q = 1; q <= n_lds; ++q) vals[(q - 1) * a.Gp + g] = pop ? key_value(a, q, g) : 0;
  }
  if (mine) atomicAdd(&populated, mine);
  __syncthreads();
  const int half = a.Gp >> 1;
  for (int k = 2; k <= a.Gp; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll 4
      for (int t = threadIdx.x; t < half; t += ORDER_THREADS) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), p = i | j;
        const long long kx = k0[i], ky = k0[p];
        const int32_t x = idx[i], y = idx[p];
        const bool x_first = kx != ky ? kx < ky : tie_before(a, vals, n_lds, x, y);
        const bool up = (i & k) == 0;
        if (up != x_first) { k0[i] = ky; k0[p] = kx; idx[i] = y; idx[p] = x; }
      }
      __syncthreads();
    }
  }
  for (int g = threadIdx.x; g < a.G; g += ORDER_THREADS) order[g] = g < populated ? idx[g] : -1;
  if (threadIdx.x == 0) *n_out = populated;
}

}  // namespace
}  // namespace lq

using namespace lq;

extern "C" {

size_t lq_group_domain_workspace_bytes(int64_t rows) {
  if (rows < 0 || rows > 0x3fffffffLL) return 0;
  const size_t cap = domain_capacity(rows);
  return HEADER + 2 * cap * sizeof(int32_t) + round_up((static_cast<size_t>(MAX_DISTINCT) + 1) * sizeof(uint32_t), 256);
}

int lq_group_domain(int64_t rows, int32_t n_cols, const int32_t* const* cols, int32_t max_card, int32_t* code,
                    int32_t* values, int32_t* card, void* ws, size_t ws_bytes, void* hip_stream) {
  clear_error();
  if (rows < 0 || rows > 0x3fffffffLL) return fail(LQ_ERR_SHAPE, "rows out of range");
  if (n_cols < 1 || n_cols > MAX_COLS) return fail(LQ_ERR_SHAPE, "n_cols %d outside 1..%d", n_cols, MAX_COLS);
  if (max_card < 1 || max_card > MAX_DISTINCT) return fail(LQ_ERR_SHAPE, "max_card %d outside 1..%d", max_card, MAX_DISTINCT);
  if (!cols || !card) return fail(LQ_ERR_NULL, "cols or card is NULL");
  if (rows > 0 && (!code || !values)) return fail(LQ_ERR_NULL, "code or values is NULL");
  Cols t{};
  t.n_cols = n_cols;
  for (int q = 0; q < n_cols; ++q) {
    if (rows > 0 && !cols[q]) return fail(LQ_ERR_NULL, "cols[%d] is NULL", q);
    if (!aligned(cols[q], 4)) return fail(LQ_ERR_SHAPE, "cols[%d] is not 4-byte aligned", q);
    t.c[q] = cols[q];
  }
  if (!aligned(code, 4) || !aligned(values, 4)) return fail(LQ_ERR_SHAPE, "code / values are not 4-byte aligned");
  const size_t need = lq_group_domain_workspace_bytes(rows);
  if (!ws || !aligned(ws, 256) || ws_bytes < need)
    return fail(LQ_ERR_WORKSPACE, "group discovery needs a 256-byte aligned workspace of %zu bytes", need);
  *card = 0;
  if (rows == 0) return LQ_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t cap = domain_capacity(rows);
  uint32_t shift = 32;
  for (uint32_t c = cap; c > 1; c >>= 1) --shift;
  uint32_t* header = static_cast<uint32_t*>(ws);
  int32_t* slots = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(ws) + HEADER);
  int32_t* slot_rank = slots + cap;
  uint32_t* reps = reinterpret_cast<uint32_t*>(slot_rank + cap);
  const unsigned row_blocks = static_cast<unsigned>((rows + 255) / 256);
  hipLaunchKernelGGL(domain_clear_kernel, dim3((cap + 255) / 256), dim3(256), 0, s, slots, cap, header);
  LQ_LAUNCH_CHECK("domain_clear_kernel");
  // A small first slice claims the slots of the frequent tuples, so that the bulk of the rows only reads
  // them: with few distinct tuples, half a million lanes racing for the same empty slots cost 20x more.
  const int64_t head = std::min<int64_t>(rows, 8192);
  hipLaunchKernelGGL(domain_insert_kernel, dim3(static_cast<unsigned>((head + 255) / 256)), dim3(256), 0, s, t,
                     static_cast<int64_t>(0), head, slots, cap - 1, shift, header, reps);
  LQ_LAUNCH_CHECK("domain_insert_kernel");
  if (rows > head) {
    hipLaunchKernelGGL(domain_insert_kernel, dim3(static_cast<unsigned>((rows - head + 255) / 256)), dim3(256), 0, s, t,
                       head, rows, slots, cap - 1, shift, header, reps);
    LQ_LAUNCH_CHECK("domain_insert_kernel");
  }
  uint32_t d = 0;
  LQ_HIP_TRY(hipMemcpyAsync(&d, header, sizeof(d), hipMemcpyDeviceToHost, s));
  LQ_HIP_TRY(hipStreamSynchronize(s));
  if (d > static_cast<uint32_t>(max_card))
    return fail(LQ_ERR_UNSUPPORTED, "more than max_card = %d distinct tuples", max_card);
  hipLaunchKernelGGL(domain_rank_kernel, dim3((d + RANK_THREADS - 1) / RANK_THREADS), dim3(RANK_THREADS), 0, s, t,
                     static_cast<int32_t>(d), slots, reps, slot_rank, values);
  LQ_LAUNCH_CHECK("domain_rank_kernel");
  hipLaunchKernelGGL(domain_encode_kernel, dim3(row_blocks), dim3(256), 0, s, t, rows, slots, cap - 1, shift, slot_rank, code);
  LQ_LAUNCH_CHECK("domain_encode_kernel");
  *card = static_cast<int32_t>(d);
  return LQ_OK;
}

int lq_order_groups(int32_t n_group_cols, const int32_t* group_card, int32_t n_measures, const int64_t* sums,
                    const int64_t* counts, int32_t n_keys, const lq_sort_key* keys, int32_t* order, int32_t* n_out,
                    void* hip_stream) {
  clear_error();
  if (n_group_cols < 0 || n_group_cols > LQ_MAX_DIMS) return fail(LQ_ERR_SHAPE, "n_group_cols %d outside 0..%d", n_group_cols, LQ_MAX_DIMS);
  if (n_keys < 0 || n_keys > 4) return fail(LQ_ERR_SHAPE, "n_keys %d outside 0..4", n_keys);
  if (n_measures < 0 || n_measures > LQ_MAX_MEASURES) return fail(LQ_ERR_SHAPE, "n_measures %d outside 0..%d", n_measures, LQ_MAX_MEASURES);
  if ((n_group_cols > 0 && !group_card) || !counts || !order || !n_out || (n_keys > 0 && !keys))
    return fail(LQ_ERR_NULL, "group_card, counts, order, n_out or keys is NULL");
  if (!aligned(counts, 8) || !aligned(sums, 8) || !aligned(order, 4) || !aligned(n_out, 4))
    return fail(LQ_ERR_SHAPE, "an array is misaligned");
  OrderArgs a{};
  int64_t G = 1;
  for (int k = 0; k < n_group_cols; ++k) {
    if (group_card[k] < 1) return fail(LQ_ERR_SHAPE, "group_card[%d] < 1", k);
    G *= group_card[k];
    if (G > MAX_GROUPS) return fail(LQ_ERR_UNSUPPORTED, "more than %d groups", MAX_GROUPS);
  }
  {
    int32_t stride = 1;
    for (int k = n_group_cols - 1; k >= 0; --k) { a.card[k] = group_card[k]; a.stride[k] = stride; stride *= group_card[k]; }
  }
  for (int q = 0; q < n_keys; ++q) {
    const lq_sort_key& key = keys[q];
    if (key.kind == LQ_KEY_GROUP_COLUMN) {
      if (key.index < 0 || key.index >= n_group_cols) return fail(LQ_ERR_SHAPE, "keys[%d]: no grouping column %d", q, key.index);
    } else if (key.kind == LQ_KEY_SUM) {
      if (key.index < 0 || key.index >= n_measures || !sums) return fail(LQ_ERR_SHAPE, "keys[%d]: no measure %d", q, key.index);
    } else if (key.kind != LQ_KEY_COUNT) {
      return fail(LQ_ERR_SHAPE, "keys[%d].kind is unknown", q);
    }
    a.kind[q] = key.kind; a.index[q] = key.index; a.desc[q] = key.descending ? 1 : 0;
  }
  a.G = static_cast<int32_t>(G);
  a.Gp = 2;
  while (a.Gp < a.G) a.Gp <<= 1;
  a.n_keys = n_keys;
  a.sums = reinterpret_cast<const long long*>(sums);
  a.counts = reinterpret_cast<const long long*>(counts);
  // LDS: 12 bytes per position (first key + group) and 8 bytes per group for each further key that
  // fits into 144 KB; keys beyond that are only looked at on ties and read from memory
  const size_t base = static_cast<size_t>(a.Gp) * 12;
  const int n_lds = std::max(0, std::min<int>(n_keys - 1, static_cast<int>((144 * 1024 - base) / (static_cast<size_t>(a.Gp) * 8))));
  const size_t lds = base + static_cast<size_t>(n_lds) * a.Gp * 8;
  if (lds > 32 * 1024)
    LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&order_groups_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
  hipLaunchKernelGGL(order_groups_kernel, dim3(1), dim3(ORDER_THREADS), lds, static_cast<hipStream_t>(hip_stream), a,
                     n_lds, order, n_out);
  LQ_LAUNCH_CHECK("order_groups_kernel");
  return LQ_OK;
}

}  // extern "C"
