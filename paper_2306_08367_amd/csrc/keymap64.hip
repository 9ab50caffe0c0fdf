// Key -> row mapping for 64-bit key values: the same cached key domain as for 32-bit keys
// (Algorithm 1's domain generation), for tables whose keys do not fit an int32.
//
// Buffer: [256-byte header | capacity 8-byte key slots | capacity 4-byte row numbers].  Two forms,
// chosen when the map is built: direct, when largest - smallest key is below 2 x capacity (the key
// area then holds 4-byte cells "row of key base + i, or -1"), else an open-addressing hash table
// (a slot is claimed with a compare-and-swap on its key; the row number is written next to it).
// The smallest int64 marks an empty slot and is therefore not a legal key.
#include "lq_common.h"

namespace lq {
namespace {

typedef unsigned long long u64;
typedef long long i64;
constexpr i64 EMPTY_KEY = static_cast<i64>(0x8000000000000000ull);
constexpr size_t HEADER = 256;
constexpr unsigned FLAG_DUPLICATE = 1u, FLAG_FULL = 2u, FLAG_WINDOW = 4u, FLAG_RESERVED = 8u;

struct Header64 {
  u64 capacity;
  unsigned flags;
  int32_t direct;
  i64 base;
  i64 min_key, max_key;      // of the keys given to the build
};

__device__ __forceinline__ uint32_t slot_of(i64 key, uint32_t shift) {
  return static_cast<uint32_t>((static_cast<u64>(key) * 0x9E3779B97F4A7C15ull) >> shift);
}

__global__ void keymap64_init_kernel(Header64* header, u64 capacity) {
  header->capacity = capacity; header->flags = 0u; header->direct = 0; header->base = 0;
  header->min_key = 0x7fffffffffffffffll; header->max_key = EMPTY_KEY;
}

__global__ __launch_bounds__(256) void keymap64_minmax_kernel(const i64* __restrict__ keys, int64_t r, Header64* header) {
  i64 lo = 0x7fffffffffffffffll, hi = EMPTY_KEY;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < r; i += static_cast<int64_t>(gridDim.x) * 256) {
    const i64 k = keys[i];
    lo = min(lo, k); hi = max(hi, k);
  }
  for (int off = 32; off > 0; off >>= 1) {
    lo = min(lo, __shfl_xor(lo, off, 64));
    hi = max(hi, __shfl_xor(hi, off, 64));
  }
  __shared__ i64 wlo[4], whi[4];
  if ((threadIdx.x & 63) == 0) { wlo[threadIdx.x >> 6] = lo; whi[threadIdx.x >> 6] = hi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    atomicMin(&header->min_key, min(min(wlo[0], wlo[1]), min(wlo[2], wlo[3])));
    atomicMax(&header->max_key, max(max(whi[0], whi[1]), max(whi[2], whi[3])));
  }
}

// Decides the form from the key range (every thread alike, the first one records it) and empties
// the key area accordingly: cells of -1, or slots holding the empty key.
__global__ __launch_bounds__(256) void keymap64_clear_kernel(i64* key_slots, u64 capacity, Header64* header) {
  const i64 lo = header->min_key, hi = header->max_key;
  const bool direct = hi >= lo && static_cast<u64>(hi) - static_cast<u64>(lo) < 2 * capacity;
  const u64 i = static_cast<u64>(blockIdx.x) * 256 + threadIdx.x;
  if (i < capacity) key_slots[i] = direct ? -1ll : EMPTY_KEY;
  if (i == 0) { header->direct = direct ? 1 : 0; header->base = direct ? lo : 0; }
}

__global__ __launch_bounds__(256) void keymap64_insert_kernel(i64* key_slots, int32_t* row_slots, uint32_t mask,
                                                              uint32_t shift, const i64* __restrict__ keys, int64_t r,
                                                              int64_t row0, Header64* header) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= r) return;
  const i64 key = keys[i];
  if (header->direct) {
    const i64 base = header->base;
    const u64 cell = static_cast<u64>(key) - static_cast<u64>(base);
    if (key < base || cell >= 2 * (static_cast<u64>(mask) + 1)) { atomicOr(&header->flags, FLAG_WINDOW); return; }
    const int old = atomicCAS(reinterpret_cast<int*>(key_slots) + cell, -1, static_cast<int>(row0 + i));
    if (old != -1) atomicOr(&header->flags, FLAG_DUPLICATE);
    atomicMax(&header->max_key, key);
    return;
  }
  if (key == EMPTY_KEY) { atomicOr(&header->flags, FLAG_RESERVED); return; }
  uint32_t s = slot_of(key, shift) & mask;
  for (uint32_t probes = 0; probes <= mask; ++probes) {           // bounded: at most one sweep of the table
    const i64 old = static_cast<i64>(atomicCAS(reinterpret_cast<u64*>(&key_slots[s]), static_cast<u64>(EMPTY_KEY),
                                               static_cast<u64>(key)));
    if (old == EMPTY_KEY) { row_slots[s] = static_cast<int32_t>(row0 + i); return; }
    if (old == key) { atomicOr(&header->flags, FLAG_DUPLICATE); return; }
    s = (s + 1) & mask;
  }
  atomicOr(&header->flags, FLAG_FULL);
}

__device__ __forceinline__ int32_t find64(const Header64* header, bool direct, i64 base, const i64* key_slots,
                                          const int32_t* row_slots, uint32_t mask, uint32_t shift, i64 key) {
  if (direct) {
    const u64 cell = static_cast<u64>(key) - static_cast<u64>(base);
    return (key >= base && cell < 2 * (static_cast<u64>(mask) + 1)) ? reinterpret_cast<const int32_t*>(key_slots)[cell] : -1;
  }
  if (key == EMPTY_KEY) return -1;
  uint32_t s = slot_of(key, shift) & mask;
  for (uint32_t probes = 0; probes <= mask; ++probes) {           // bounded: at most one sweep of the table
    const i64 v = key_slots[s];
    if (v == EMPTY_KEY) return -1;
    if (v == key) return row_slots[s];
    s = (s + 1) & mask;
  }
  return -1;
}

typedef long long v2l __attribute__((ext_vector_type(2)));
typedef int v2i __attribute__((ext_vector_type(2)));

// Two keys per thread (one 16-byte load) when the columns allow it; the odd last key one by one.
__global__ __launch_bounds__(256) void keymap64_lookup_kernel(const Header64* __restrict__ header,
                                                              const i64* __restrict__ key_slots,
                                                              const int32_t* __restrict__ row_slots, uint32_t mask,
                                                              uint32_t shift, const i64* __restrict__ keys, int64_t n,
                                                              int32_t* __restrict__ fk, int vec_ok) {
  const bool direct = header->direct != 0;
  const i64 base = header->base;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (vec_ok) {
    const int64_t n2 = n / 2;
    if (t < n2) {
      const v2l k = __builtin_nontemporal_load(reinterpret_cast<const v2l*>(keys) + t);
      v2i r;
      r[0] = find64(header, direct, base, key_slots, row_slots, mask, shift, k[0]);
      r[1] = find64(header, direct, base, key_slots, row_slots, mask, shift, k[1]);
      __builtin_nontemporal_store(r, reinterpret_cast<v2i*>(fk) + t);
    } else if (t == n2 && (n & 1)) {
      fk[n - 1] = find64(header, direct, base, key_slots, row_slots, mask, shift, keys[n - 1]);
    }
  } else if (t < n) {
    fk[t] = find64(header, direct, base, key_slots, row_slots, mask, shift, keys[t]);
  }
}

struct Geometry64 { u64 capacity; uint32_t mask, shift; };
bool geometry64(size_t table_bytes, Geometry64* g) {
  if (table_bytes < HEADER + 2 * 12) return false;
  u64 cap = 2;
  while (HEADER + cap * 2 * 12 <= table_bytes && cap < (1ull << 31)) cap <<= 1;
  int log2 = 0;
  while ((1ull << log2) < cap) ++log2;
  g->capacity = cap; g->mask = static_cast<uint32_t>(cap - 1); g->shift = static_cast<uint32_t>(64 - log2);
  return true;
}

int check_flags64(const Header64* header, hipStream_t s) {
  unsigned h = 0;
  LQ_HIP_TRY(hipMemcpyAsync(&h, &header->flags, sizeof(h), hipMemcpyDeviceToHost, s));
  LQ_HIP_TRY(hipStreamSynchronize(s));
  if (h & FLAG_DUPLICATE) return fail(LQ_ERR_DUPLICATE_KEY, "the dimension key column holds a value twice");
  if (h & FLAG_FULL) return fail(LQ_ERR_WORKSPACE, "key map is full");
  if (h & FLAG_WINDOW) return fail(LQ_ERR_WORKSPACE, "a key lies outside the window of this direct-address map: rebuild the map with all keys");
  if (h & FLAG_RESERVED) return fail(LQ_ERR_UNSUPPORTED, "the smallest int64 is not a legal key");
  return LQ_OK;
}

}  // namespace
}  // namespace lq

using namespace lq;

extern "C" {

size_t lq_keymap64_bytes(int64_t max_keys) {
  if (max_keys < 0 || max_keys > (1ll << 29)) return 0;
  u64 cap = 2;
  while (cap < static_cast<u64>(max_keys) * 2) cap <<= 1;
  return HEADER + cap * 12;
}

int lq_keymap64_insert(void* table, size_t table_bytes, const int64_t* keys, int64_t n_keys, int64_t first_row,
                       uint32_t flags, void* hip_stream) {
  clear_error();
  Geometry64 g;
  if (!table || !aligned(table, 256) || !geometry64(table_bytes, &g)) return fail(LQ_ERR_WORKSPACE, "key map buffer is NULL, misaligned or too small");
  if (n_keys < 0 || first_row < 0 || first_row + n_keys > 0x7fffffffLL) return fail(LQ_ERR_SHAPE, "row numbers do not fit int32");
  if (n_keys > 0 && (!keys || !aligned(keys, 8))) return fail(LQ_ERR_NULL, "keys is NULL or misaligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Header64* header = static_cast<Header64*>(table);
  i64* key_slots = reinterpret_cast<i64*>(static_cast<char*>(table) + HEADER);
  int32_t* row_slots = reinterpret_cast<int32_t*>(key_slots + g.capacity);
  if (n_keys > 0) {
    hipLaunchKernelGGL(keymap64_insert_kernel, dim3(static_cast<unsigned>((n_keys + 255) / 256)), dim3(256), 0, s,
                       key_slots, row_slots, g.mask, g.shift, reinterpret_cast<const i64*>(keys), n_keys, first_row, header);
    LQ_LAUNCH_CHECK("keymap64_insert_kernel");
  }
  if (flags & LQ_CHECK_KEYS) return check_flags64(header, s);
  return LQ_OK;
}

int lq_keymap64_build(void* table, size_t table_bytes, const int64_t* keys, int64_t n_keys, uint32_t flags,
                      void* hip_stream) {
  clear_error();
  Geometry64 g;
  if (!table || !aligned(table, 256) || !geometry64(table_bytes, &g)) return fail(LQ_ERR_WORKSPACE, "key map buffer is NULL, misaligned or too small");
  if (n_keys < 0 || static_cast<u64>(n_keys) * 2 > g.capacity) return fail(LQ_ERR_WORKSPACE, "key map buffer holds %llu slots, %lld keys need twice as many", (unsigned long long)g.capacity, (long long)n_keys);
  if (n_keys > 0 && (!keys || !aligned(keys, 8))) return fail(LQ_ERR_NULL, "keys is NULL or misaligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Header64* header = static_cast<Header64*>(table);
  i64* key_slots = reinterpret_cast<i64*>(static_cast<char*>(table) + HEADER);
  hipLaunchKernelGGL(keymap64_init_kernel, dim3(1), dim3(1), 0, s, header, g.capacity);
  LQ_LAUNCH_CHECK("keymap64_init_kernel");
  if (n_keys > 0) {
    const unsigned mm_blocks = static_cast<unsigned>(std::min<int64_t>((n_keys + 1023) / 1024, 256));
    hipLaunchKernelGGL(keymap64_minmax_kernel, dim3(mm_blocks), dim3(256), 0, s, reinterpret_cast<const i64*>(keys), n_keys, header);
    LQ_LAUNCH_CHECK("keymap64_minmax_kernel");
  }
  hipLaunchKernelGGL(keymap64_clear_kernel, dim3(static_cast<unsigned>((g.capacity + 255) / 256)), dim3(256), 0, s,
                     key_slots, g.capacity, header);
  LQ_LAUNCH_CHECK("keymap64_clear_kernel");
  return lq_keymap64_insert(table, table_bytes, keys, n_keys, 0, flags, hip_stream);
}

int lq_keymap64_lookup(const void* table, size_t table_bytes, const int64_t* fact_keys, int64_t n, int32_t* fk,
                       void* hip_stream) {
  clear_error();
  Geometry64 g;
  if (!table || !aligned(table, 256) || !geometry64(table_bytes, &g)) return fail(LQ_ERR_WORKSPACE, "key map buffer is NULL, misaligned or too small");
  if (n < 0) return fail(LQ_ERR_SHAPE, "n < 0");
  if (n == 0) return LQ_OK;
  if (!fact_keys || !fk || !aligned(fact_keys, 8) || !aligned(fk, 4)) return fail(LQ_ERR_NULL, "fact_keys or fk is NULL or misaligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const Header64* header = static_cast<const Header64*>(table);
  const i64* key_slots = reinterpret_cast<const i64*>(static_cast<const char*>(table) + HEADER);
  const int32_t* row_slots = reinterpret_cast<const int32_t*>(key_slots + g.capacity);
  const int vec_ok = aligned(fact_keys, 16) && aligned(fk, 8);
  const int64_t threads = vec_ok ? n / 2 + 1 : n;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
  hipLaunchKernelGGL(keymap64_lookup_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, header, key_slots,
                     row_slots, g.mask, g.shift, reinterpret_cast<const i64*>(fact_keys), n, fk, vec_ok);
  LQ_LAUNCH_CHECK("keymap64_lookup_kernel");
  return LQ_OK;
}

}  // extern "C"
