// (Internal header: the compile-time specialised fact scan of the group-by, instantiated in groupby.hip with
// the accumulators in LDS and in groupby_many.hip with the accumulators in memory, so that the two families
// compile in parallel.)
#ifndef LQ_GROUPBY_FAST_H_
#define LQ_GROUPBY_FAST_H_
#include "lq_common.h"

namespace lq {

constexpr int SCAN_THREADS = 1024;

// The dimension side of a group-by call.
enum DimKind : int32_t { DK_NONE = 0, DK_BITMAP = 1, DK_BYTE = 2, DK_U16 = 3 };

struct GbDim {
  const int32_t* fk;
  const uint8_t* mask;   // raw, may be NULL
  const int32_t* code;   // raw, may be NULL
  int64_t rows;
  int32_t kind;
  int32_t card;          // 1 when not grouping
  int32_t stride;        // weight of this dimension's code in the group number (0 when not grouping)
  uint32_t off;          // byte offset of the packed table (16-byte aligned)
  uint32_t bytes;        // packed size, multiple of 16
  int32_t in_lds;        // 1 when the table is part of the LDS-resident prefix
};

struct GbArgs {
  int64_t n;
  int32_t K;
  GbDim d[LQ_MAX_DIMS];
  const uint8_t* fact_mask;
  int32_t M;
  const int32_t* meas[LQ_MAX_MEASURES];
  unsigned long long* sums;    // [M x G]
  unsigned long long* counts;  // [G] or NULL
  int32_t G;
  uint8_t* packed;             // workspace: all packed tables
  uint32_t packed_bytes;
  unsigned long long* partial; // workspace: [workgroups x (M+1) x G]
};


// The same scan with everything the generic kernel decides at run time fixed at compile time:
// no fact mask, 16-byte aligned columns, only byte tables (grouping dimensions, optionally
// masked) and bitmaps (mask-only dimensions).  The host orders the dimensions into four runs:
//   NBL byte tables in LDS, NML bitmaps in LDS, NMG bitmaps in memory, NBG byte tables in memory.
// Tables that do not fit LDS stay in memory (L2) and are only consulted for rows that survived
// every LDS-resident predicate, so a selective query sends few requests to L2.  Group numbers use
// per-dimension strides, so the order in which dimensions are visited does not matter.
struct FastArgs {
  int64_t n;
  const int32_t* fk[LQ_MAX_DIMS];    // in the order of the four runs above
  uint32_t off[LQ_MAX_DIMS];         // byte offset inside the packed buffer
  int32_t stride[LQ_MAX_DIMS];
  uint8_t wide[LQ_MAX_DIMS];         // 1: the code table has 16-bit entries (more than 255 values), else bytes
  const int32_t* meas[LQ_MAX_MEASURES];
  const uint8_t* packed;
  uint32_t lds_bytes;                // prefix of the packed buffer that is copied into LDS
  int32_t G;
  unsigned long long* partial;
  unsigned long long* gsums;         // not NULL: more groups than LDS holds, accumulate into the caller's
  unsigned long long* gcounts;       // arrays (gcounts may be NULL) instead of LDS + partial rows
  const uint8_t* fact_mask;          // NULL or one byte per fact row, 4-byte aligned (WIDE instantiations only)
};

// The wider aggregate on the specialised scan: one measure (a column, or the product / difference of two),
// up to two fact-side range predicates, every side table in LDS.
struct AggFastArgs {
  FastArgs f;                 // f.meas[0] is the measure's first column; f.partial rows hold [sum | count | min | max] x G
  const int32_t* b;           // second column of the measure (op != 0)
  int32_t op;                 // 0 column, 1 product, 2 difference
  const int32_t* pcol[2];
  int32_t lo[2], hi[2];
  int32_t minmax;             // MIN / MAX wanted (otherwise their accumulators keep the neutral elements)
};

// Many groups, second form: survivors are first sorted into buckets of neighbouring groups (a bucket's
// accumulators fit LDS), then one workgroup per bucket adds its bucket up in LDS and is the only writer of
// its groups.  A survivor costs one LDS atomic and one 8- or 12-byte store instead of two or three device-wide
// atomics; what does not fit a bucket's slots (skewed groups) goes the atomic way.
struct BucketArgs {
  unsigned int* gcount;      // [buckets] survivors sent to each bucket so far (may pass `cap`: the excess took the atomics)
  uint32_t* pairs;           // [buckets][cap][1 + measures]: group number inside the bucket, then the measures
  int32_t buckets;
  int32_t shift;             // bucket = group >> shift
  uint32_t cap;              // slots per bucket
};

struct FastLaunch { unsigned blocks; size_t lds; int64_t per_block; hipStream_t s; int nbl, nml, nmg, nbg, M; BucketArgs bucket; };

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// Encodes every dimension's side table into `dst` (memory, or a workgroup's LDS): thread gtid of gstride
// (gstride a multiple of 64, whole wavefronts take part).
// BITMAP: a wavefront turns 64 mask bytes into one 64-bit ballot word per step.
// BYTE / U16: one thread builds 4 (2) consecutive entries and stores them as one word.
__device__ __forceinline__ void pack_tables(const GbArgs& a, uint8_t* dst, int64_t gtid, int64_t gstride) {
  const int lane = threadIdx.x & 63;
  const int64_t gwave = gtid >> 6, nwave = gstride >> 6;
  for (int k = 0; k < a.K; ++k) {
    const GbDim& d = a.d[k];
    if (d.kind == DK_BITMAP) {
      unsigned long long* out = reinterpret_cast<unsigned long long*>(dst + d.off);
      const int64_t steps = d.bytes / 8;               // 64 rows per step
      for (int64_t q = gwave; q < steps; q += nwave) {
        const int64_t j = q * 64 + lane;
        const bool on = j < d.rows && (!d.mask || d.mask[j] != 0);     // (a table without predicate or code: all rows pass)
        const unsigned long long bits = __ballot(on);
        if (lane == 0) out[q] = bits;
      }
    } else if (d.kind == DK_BYTE) {
      uint32_t* out = reinterpret_cast<uint32_t*>(dst + d.off);
      for (int64_t q = gtid; q < d.bytes / 4; q += gstride) {
        uint32_t w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int64_t j = q * 4 + b;
          uint32_t v = 0xffu;
          if (j < d.rows && (!d.mask || d.mask[j])) v = d.code ? static_cast<uint32_t>(d.code[j]) & 0xffu : 0u;
          w |= v << (8 * b);
        }
        out[q] = w;
      }
    } else if (d.kind == DK_U16) {
      uint32_t* out = reinterpret_cast<uint32_t*>(dst + d.off);
      for (int64_t q = gtid; q < d.bytes / 4; q += gstride) {
        uint32_t w = 0;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int64_t j = q * 2 + b;
          uint32_t v = 0xffffu;
          if (j < d.rows && (!d.mask || d.mask[j])) v = static_cast<uint32_t>(d.code[j]) & 0xffffu;
          w |= v << (16 * b);
        }
        out[q] = w;
      }
    }
  }
}


// Neutral elements of MIN and MAX (what groups without rows keep).
constexpr long long AGG_MIN_INIT = 0x7fffffffffffffffLL;
constexpr long long AGG_MAX_INIT = -0x7fffffffffffffffLL - 1;

// ---------------------------------------------------------------- many groups ------------
//
// More accumulators than LDS holds (the multi-column group-by of Section 2.4.2 multiplies the
// cardinalities of its grouping attributes): the accumulators are the caller's own dense arrays in
// memory, cleared by a first launch, and survivors add into them with device-wide 64-bit atomics; no
// partial rows, no fold.  Before the atomics the lanes of a wavefront that hit the same group are
// merged (up to four distinct groups per step; a hot group then costs one atomic per wavefront step
// instead of one per row), the rest go out one by one.  Integer adds commute: exact whatever the order.

__device__ __forceinline__ long long wave_sum64(long long v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ long long wave_min64(long long v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ long long wave_max64(long long v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, 64));
  return v;
}

struct GlobalOut {
  unsigned long long* sums;     // [M x G] or NULL
  unsigned long long* counts;   // [G] or NULL
  long long* mins;              // [M x G] or NULL
  long long* maxs;              // [M x G] or NULL
};

// One row slot of every lane: `alive` lanes add val[0..M) into group g.  Wavefront-uniform control flow.
template <int MAXM>
__device__ __forceinline__ void merge_and_add(bool alive, int32_t g, const long long (&val)[MAXM], int M, int32_t G,
                                              const GlobalOut& o) {
  const int lane = threadIdx.x & 63;
  unsigned long long todo = __ballot(alive);
  for (int round = 0; round < 4 && todo; ++round) {
    const int leader = __ffsll(static_cast<long long>(todo)) - 1;
    const int32_t lg = __builtin_amdgcn_readlane(g, leader);
    const bool mine = alive && g == lg;
    const unsigned long long same = __ballot(mine);
    todo &= ~same;
    if (__popcll(same) < 2) continue;            // a single row: it goes out with the others below
#pragma unroll
    for (int m = 0; m < MAXM; ++m) {
      if (m >= M) break;
      if (o.sums) {
        const long long t = wave_sum64(mine ? val[m] : 0LL);
        if (lane == leader) atomicAdd(&o.sums[static_cast<size_t>(m) * G + lg], static_cast<unsigned long long>(t));
      }
      if (o.mins) {
        const long long t = wave_min64(mine ? val[m] : AGG_MIN_INIT);
        if (lane == leader) atomicMin(&o.mins[static_cast<size_t>(m) * G + lg], t);
      }
      if (o.maxs) {
        const long long t = wave_max64(mine ? val[m] : AGG_MAX_INIT);
        if (lane == leader) atomicMax(&o.maxs[static_cast<size_t>(m) * G + lg], t);
      }
    }
    if (o.counts && lane == leader) atomicAdd(&o.counts[lg], static_cast<unsigned long long>(__popcll(same)));
    alive = alive && !mine;
  }
  if (alive) {
#pragma unroll
    for (int m = 0; m < MAXM; ++m) {
      if (m >= M) break;
      const size_t at = static_cast<size_t>(m) * G + g;
      if (o.sums) atomicAdd(&o.sums[at], static_cast<unsigned long long>(val[m]));
      if (o.mins) atomicMin(&o.mins[at], val[m]);
      if (o.maxs) atomicMax(&o.maxs[at], val[m]);
    }
    if (o.counts) atomicAdd(&o.counts[g], 1ull);
  }
}

// sums / counts = 0, mins / maxs = their neutral elements (a fill kernel rather than a memset, so that
// callers may record the call into a HIP graph).
// `words` (may be NULL): n_words 32-bit counters cleared by the same launch (the bucket counters).
__global__ __launch_bounds__(256) void init_outputs_kernel(GlobalOut o, int64_t MG, int64_t G, unsigned int* words, int64_t n_words) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n_words; i += stride) words[i] = 0u;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < MG; i += stride) {
    if (o.sums) o.sums[i] = 0ull;
    if (o.mins) o.mins[i] = AGG_MIN_INIT;
    if (o.maxs) o.maxs[i] = AGG_MAX_INIT;
    if (o.counts && i < G) o.counts[i] = 0ull;
  }
}


// BYTE: a code table (entries of one byte, or of two when `wide`; all ones = filtered out), else a bitmap.
// WIDE: some code table of the call has 16-bit entries (decided per kernel instantiation, so that calls with byte
// tables only do not pay for the test).
template <bool BYTE, bool GUARDED, bool WIDE>
__device__ __forceinline__ void lookup(const uint8_t* t, int32_t j, int32_t stride, bool wide, bool& alive, int32_t& g) {
  alive = alive && j >= 0;
  if (GUARDED && !alive) return;
  const uint32_t jj = j < 0 ? 0u : static_cast<uint32_t>(j);   // keep the lookup in bounds
  if (BYTE) {
    uint32_t b;
    if (WIDE && wide) {                                        // (the same for every lane: a property of the table)
      b = reinterpret_cast<const uint16_t*>(t)[jj];
      alive = alive && b != 0xffffu;
    } else {
      b = t[jj];
      alive = alive && b != 0xffu;
    }
    g += static_cast<int32_t>(b) * stride;
  } else {
    const uint32_t w = reinterpret_cast<const uint32_t*>(t)[jj >> 5];
    alive = alive && ((w >> (jj & 31)) & 1u);
  }
}

// The fact table's own selection vector: the four mask bytes of rows 4 v .. 4 v + 3 (all ones without a mask), and the
// first key of row q with the row's byte applied (a row that is masked out gets the key -1, "no match").  Only the
// WIDE instantiations look at it, so that calls without a mask and with byte tables do not pay for the test.
template <bool WIDE>
__device__ __forceinline__ uint32_t fact_mask_word(const FastArgs& a, int64_t v) {
  if constexpr (WIDE) {
    if (a.fact_mask) return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(a.fact_mask) + v);
  }
  return ~0u;
}
template <bool WIDE>
__device__ __forceinline__ int32_t masked_key(uint32_t word, int q, int32_t key) {
  if constexpr (WIDE) return ((word >> (8 * q)) & 0xffu) != 0u ? key : -1;
  return key;
}
template <bool WIDE>
__device__ __forceinline__ int32_t masked_tail_key(const FastArgs& a, int64_t row, int32_t key) {
  if constexpr (WIDE) {
    if (a.fact_mask && a.fact_mask[row] == 0) return -1;
  }
  return key;
}

// All dimensions of one fact row.
template <int NBL, int NML, int NMG, int NBG, bool WIDE = false>
__device__ __forceinline__ void classify_fast(const FastArgs& a, const uint8_t* tab, const int32_t* j,
                                              bool& alive, int32_t& g) {
  constexpr int NL = NBL + NML, ND = NL + NMG + NBG;
#pragma unroll
  for (int k = 0; k < ND; ++k) {
    if (k < NBL) lookup<true, false, WIDE>(tab + a.off[k], j[k], a.stride[k], a.wide[k] != 0, alive, g);
    else if (k < NL) lookup<false, false, false>(tab + a.off[k], j[k], 0, false, alive, g);
    else if (k < NL + NMG) lookup<false, true, false>(a.packed + a.off[k], j[k], 0, false, alive, g);
    else lookup<true, true, WIDE>(a.packed + a.off[k], j[k], a.stride[k], a.wide[k] != 0, alive, g);
  }
}

template <int NBL, int NML, int NMG, int NBG, int MM, bool WIDE>
__global__ __launch_bounds__(SCAN_THREADS) void scan_fast_kernel(FastArgs a, int64_t per_block) {
  extern __shared__ __align__(16) uint8_t smem[];
  constexpr int ND = NBL + NML + NMG + NBG;
  unsigned long long* acc = reinterpret_cast<unsigned long long*>(smem);
  const int n_acc = (MM + 1) * a.G;
  uint8_t* tab = smem + round_up(static_cast<size_t>(n_acc) * 8, 16);
  const int tid = threadIdx.x;

  const int64_t n_vec = a.n / 4;
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  int64_t v = v_begin + tid;
  v4i cur[ND], nxt[ND];
  uint32_t fm_cur = ~0u, fm_nxt = ~0u;
  if (v < v_end) {
#pragma unroll
    for (int k = 0; k < ND; ++k) cur[k] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + v);
    fm_cur = fact_mask_word<WIDE>(a, v);
  }
  for (int i = tid; i < n_acc; i += SCAN_THREADS) acc[i] = 0ull;
  {
    const uint4* src = reinterpret_cast<const uint4*>(a.packed);
    uint4* dst = reinterpret_cast<uint4*>(tab);
    for (uint32_t i = tid; i < a.lds_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
  }
  __syncthreads();

  // No grouping dimension (a filtered sum, one group): every survivor would hit the same accumulator, so a lane adds up
  // its own rows in registers and a wavefront sends one sum per measure to LDS at the end.
  constexpr bool SINGLE = NBL + NBG == 0;
  if constexpr (SINGLE) {
    long long own[MM];
#pragma unroll
    for (int m = 0; m < MM; ++m) own[m] = 0;
    long long own_rows = 0;
    while (v < v_end) {
      const int64_t vn = v + SCAN_THREADS;
      if (vn < v_end) {
#pragma unroll
        for (int k = 0; k < ND; ++k) nxt[k] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + vn);
        fm_nxt = fact_mask_word<WIDE>(a, vn);
      }
      bool alive[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int32_t j[ND];
#pragma unroll
        for (int k = 0; k < ND; ++k) j[k] = cur[k][q];
        j[0] = masked_key<WIDE>(fm_cur, q, j[0]);
        int32_t g = 0;
        alive[q] = true;
        classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive[q], g);
      }
      if (alive[0] || alive[1] || alive[2] || alive[3]) {
#pragma unroll
        for (int m = 0; m < MM; ++m) {
          const v4i val = *(reinterpret_cast<const v4i*>(a.meas[m]) + v);
#pragma unroll
          for (int q = 0; q < 4; ++q) own[m] += alive[q] ? val[q] : 0;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) own_rows += alive[q] ? 1 : 0;
      }
#pragma unroll
      for (int k = 0; k < ND; ++k) cur[k] = nxt[k];
      fm_cur = fm_nxt;
      v = vn;
    }
#pragma unroll
    for (int m = 0; m < MM; ++m) {
      const long long t = wave_sum64(own[m]);
      if ((tid & 63) == 0) atomicAdd(&acc[m], static_cast<unsigned long long>(t));
    }
    const long long t = wave_sum64(own_rows);
    if ((tid & 63) == 0) atomicAdd(&acc[MM], static_cast<unsigned long long>(t));
  }
  while (!SINGLE && v < v_end) {
    const int64_t vn = v + SCAN_THREADS;
    if (vn < v_end) {
#pragma unroll
      for (int k = 0; k < ND; ++k) nxt[k] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + vn);
      fm_nxt = fact_mask_word<WIDE>(a, vn);
    }
    int32_t g[4];
    bool alive[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int32_t j[ND];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = cur[k][q];
      j[0] = masked_key<WIDE>(fm_cur, q, j[0]);
      g[q] = 0;
      alive[q] = true;
      classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive[q], g[q]);
    }
    if (alive[0] || alive[1] || alive[2] || alive[3]) {
#pragma unroll
      for (int m = 0; m < MM; ++m) {
        const v4i val = *(reinterpret_cast<const v4i*>(a.meas[m]) + v);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (alive[q])
            atomicAdd(&acc[m * a.G + g[q]], static_cast<unsigned long long>(static_cast<long long>(val[q])));
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (alive[q]) atomicAdd(&acc[MM * a.G + g[q]], 1ull);
    }
#pragma unroll
    for (int k = 0; k < ND; ++k) cur[k] = nxt[k];
    fm_cur = fm_nxt;
    v = vn;
  }
  // ragged tail (n % 4 rows)
  if (blockIdx.x == 0) {
    const int64_t i = n_vec * 4 + tid;
    if (i < a.n) {
      int32_t j[ND];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = a.fk[k][i];
      j[0] = masked_tail_key<WIDE>(a, i, j[0]);
      int32_t g = 0;
      bool alive = true;
      classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive, g);
      if (alive) {
#pragma unroll
        for (int m = 0; m < MM; ++m)
          atomicAdd(&acc[m * a.G + g], static_cast<unsigned long long>(static_cast<long long>(a.meas[m][i])));
        atomicAdd(&acc[MM * a.G + g], 1ull);
      }
    }
  }
  __syncthreads();
  unsigned long long* mine = a.partial + static_cast<size_t>(blockIdx.x) * n_acc;
  for (int i = tid; i < n_acc; i += SCAN_THREADS) mine[i] = acc[i];
}


// The same scan with the accumulators in memory: a.gsums [MM x G] and a.gcounts [G] (or NULL), cleared
// before the launch.  No partial rows, LDS only holds side tables.
template <int NBL, int NML, int NMG, int NBG, int MM, bool WIDE>
__global__ __launch_bounds__(SCAN_THREADS) void scan_fast_mem_kernel(FastArgs a, int64_t per_block) {
  extern __shared__ __align__(16) uint8_t smem[];
  constexpr int ND = NBL + NML + NMG + NBG;
  uint8_t* tab = smem;
  const int tid = threadIdx.x;
  const GlobalOut gout{a.gsums, a.gcounts, nullptr, nullptr};

  const int64_t n_vec = a.n / 4;
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  int64_t v = v_begin + tid;
  const v4i none = {-1, -1, -1, -1};
  v4i cur[ND], nxt[ND];
#pragma unroll
  for (int k = 0; k < ND; ++k)
    cur[k] = v < v_end ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + v) : none;
  uint32_t fm_cur = v < v_end ? fact_mask_word<WIDE>(a, v) : ~0u, fm_nxt = ~0u;
  {
    const uint4* src = reinterpret_cast<const uint4*>(a.packed);
    uint4* dst = reinterpret_cast<uint4*>(tab);
    for (uint32_t i = tid; i < a.lds_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
  }
  __syncthreads();

  // every lane of a wavefront takes the same number of steps (lanes past the end carry keys of -1, "no
  // match"): merging equal groups before the atomics is a wavefront operation
  while (v - (tid & 63) < v_end) {
    const int64_t vn = v + SCAN_THREADS;
#pragma unroll
    for (int k = 0; k < ND; ++k)
      nxt[k] = vn < v_end ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + vn) : none;
    fm_nxt = vn < v_end ? fact_mask_word<WIDE>(a, vn) : ~0u;
    int32_t g[4];
    bool alive[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int32_t j[ND];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = cur[k][q];
      j[0] = masked_key<WIDE>(fm_cur, q, j[0]);
      g[q] = 0;
      alive[q] = true;
      classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive[q], g[q]);
    }
    const bool any = alive[0] || alive[1] || alive[2] || alive[3];
    if (__ballot(any) != 0ull) {
      long long val[4][MM];
#pragma unroll
      for (int m = 0; m < MM; ++m) {   // measure columns are only touched where a lane has a survivor
        const v4i t = any ? *(reinterpret_cast<const v4i*>(a.meas[m]) + v) : none;
#pragma unroll
        for (int q = 0; q < 4; ++q) val[q][m] = t[q];
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) merge_and_add<MM>(alive[q], g[q], val[q], MM, a.G, gout);
    }
#pragma unroll
    for (int k = 0; k < ND; ++k) cur[k] = nxt[k];
    fm_cur = fm_nxt;
    v = vn;
  }
  // ragged tail (n % 4 rows): one row per lane, straight to memory
  if (blockIdx.x == 0) {
    const int64_t i = n_vec * 4 + tid;
    if (i < a.n) {
      int32_t j[ND];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = a.fk[k][i];
      j[0] = masked_tail_key<WIDE>(a, i, j[0]);
      int32_t g = 0;
      bool alive = true;
      classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive, g);
      if (alive) {
#pragma unroll
        for (int m = 0; m < MM; ++m)
          atomicAdd(&a.gsums[static_cast<size_t>(m) * a.G + g], static_cast<unsigned long long>(static_cast<long long>(a.meas[m][i])));
        if (a.gcounts) atomicAdd(&a.gcounts[g], 1ull);
      }
    }
  }
}

// First pass of the bucketed form.  Per round of the workgroup (up to 8 rows per thread): every survivor takes a
// rank inside its bucket from an LDS counter; one thread per bucket with survivors reserves that many slots
// of the bucket with one device-wide atomic; the survivors are then written to their slots.  Every thread
// of the workgroup takes the same number of steps (the barriers are inside the loop); lanes past the end
// carry keys of -1.  gcount is zero and the outputs are cleared before the launch.
template <int NBL, int NML, int NMG, int NBG, int MM, bool WIDE>
__global__ __launch_bounds__(SCAN_THREADS) void scan_fast_bucket_kernel(FastArgs a, BucketArgs b, int64_t per_block) {
  extern __shared__ __align__(16) uint8_t smem[];
  constexpr int ND = NBL + NML + NMG + NBG;
  uint8_t* tab = smem;
  unsigned int* lcount = reinterpret_cast<unsigned int*>(smem + round_up(static_cast<size_t>(a.lds_bytes), 16));
  unsigned int* lbase = lcount + b.buckets;
  const int tid = threadIdx.x;
  const GlobalOut gout{a.gsums, a.gcounts, nullptr, nullptr};

  const int64_t n_vec = a.n / 4;
  const int64_t v_begin = static_cast<int64_t>(blockIdx.x) * per_block;
  const int64_t v_end = min(n_vec, v_begin + per_block);
  const int64_t steps = v_begin < v_end ? (v_end - v_begin + SCAN_THREADS - 1) / SCAN_THREADS : 0;
  int64_t v = v_begin + tid;
  const v4i none = {-1, -1, -1, -1};
  v4i cur[ND], nxt[ND];
#pragma unroll
  for (int k = 0; k < ND; ++k)
    cur[k] = v < v_end ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + v) : none;
  uint32_t fm_cur = v < v_end ? fact_mask_word<WIDE>(a, v) : ~0u, fm_nxt = ~0u;
  {
    const uint4* src = reinterpret_cast<const uint4*>(a.packed);
    uint4* dst = reinterpret_cast<uint4*>(tab);
    for (uint32_t i = tid; i < a.lds_bytes / 16; i += SCAN_THREADS) dst[i] = src[i];
  }
  for (int i = tid; i < b.buckets; i += SCAN_THREADS) lcount[i] = 0u;
  __syncthreads();

  // A round is up to NS steps (4 NS rows per thread): their survivors stay in registers until the round's
  // slots are reserved, so that the two barriers and the reservation are paid once per 4 NS rows.
  constexpr int NS = 2;
  for (int64_t st0 = 0; st0 < steps; st0 += NS) {
    int32_t g[NS][4];
    int32_t val[NS][4][MM];
    unsigned int rank[NS][4];
    unsigned int alive_bits = 0u;                   // bit 4 s + q: row q of step s survives
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (st0 + s < steps) {                        // (the same for the whole workgroup)
        const int64_t vn = v + SCAN_THREADS;
#pragma unroll
        for (int k = 0; k < ND; ++k)
          nxt[k] = vn < v_end ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.fk[k]) + vn) : none;
        fm_nxt = vn < v_end ? fact_mask_word<WIDE>(a, vn) : ~0u;
        bool alive[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          int32_t j[ND];
#pragma unroll
          for (int k = 0; k < ND; ++k) j[k] = cur[k][q];
          j[0] = masked_key<WIDE>(fm_cur, q, j[0]);
          g[s][q] = 0;
          alive[q] = true;
          classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive[q], g[s][q]);
        }
        const bool any = alive[0] || alive[1] || alive[2] || alive[3];
#pragma unroll
        for (int m = 0; m < MM; ++m) {              // measure columns are only touched where a lane has a survivor
          const v4i t = any ? *(reinterpret_cast<const v4i*>(a.meas[m]) + v) : none;
#pragma unroll
          for (int q = 0; q < 4; ++q) val[s][q][m] = t[q];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          rank[s][q] = alive[q] ? atomicAdd(&lcount[g[s][q] >> b.shift], 1u) : 0u;
          alive_bits |= alive[q] ? 1u << (4 * s + q) : 0u;
        }
#pragma unroll
        for (int k = 0; k < ND; ++k) cur[k] = nxt[k];
        fm_cur = fm_nxt;
        v = vn;
      }
    }
    __syncthreads();
    for (int i = tid; i < b.buckets; i += SCAN_THREADS) {
      const unsigned int c = lcount[i];
      if (c) { lbase[i] = atomicAdd(&b.gcount[i], c); lcount[i] = 0u; }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        bool over = false;
        if ((alive_bits >> (4 * s + q)) & 1u) {
          const int bk = g[s][q] >> b.shift;
          const unsigned int pos = lbase[bk] + rank[s][q];
          if (pos < b.cap) {
            uint32_t* dst = b.pairs + (static_cast<size_t>(bk) * b.cap + pos) * (1 + MM);
            const uint32_t gl = static_cast<uint32_t>(g[s][q] & ((1 << b.shift) - 1));
            // (ordinary stores: the runs of a bucket are completed in L2 by later rounds and other workgroups;
            // streaming stores send every 8-byte piece to memory on its own and were measured 3.6x slower)
            if constexpr (MM == 1) {             // one 8-byte store (slots of two words are 8-byte aligned)
              typedef unsigned int v2u __attribute__((ext_vector_type(2)));
              *reinterpret_cast<v2u*>(dst) = v2u{gl, static_cast<uint32_t>(val[s][q][0])};
            } else {
              dst[0] = gl;
#pragma unroll
              for (int m = 0; m < MM; ++m) dst[1 + m] = static_cast<uint32_t>(val[s][q][m]);
            }
          } else {
            over = true;
          }
        }
        if (__ballot(over) != 0ull) {                // rare: a bucket is full, the rest of it takes the atomics
          long long wide[MM];
#pragma unroll
          for (int m = 0; m < MM; ++m) wide[m] = val[s][q][m];
          merge_and_add<MM>(over, g[s][q], wide, MM, a.G, gout);
        }
      }
  }
  // ragged tail (n % 4 rows): one row per lane, straight to memory
  if (blockIdx.x == 0) {
    const int64_t i = n_vec * 4 + tid;
    if (i < a.n) {
      int32_t j[ND];
#pragma unroll
      for (int k = 0; k < ND; ++k) j[k] = a.fk[k][i];
      j[0] = masked_tail_key<WIDE>(a, i, j[0]);
      int32_t g = 0;
      bool alive = true;
      classify_fast<NBL, NML, NMG, NBG, WIDE>(a, tab, j, alive, g);
      if (alive) {
#pragma unroll
        for (int m = 0; m < MM; ++m)
          atomicAdd(&a.gsums[static_cast<size_t>(m) * a.G + g], static_cast<unsigned long long>(static_cast<long long>(a.meas[m][i])));
        if (a.gcounts) atomicAdd(&a.gcounts[g], 1ull);
      }
    }
  }
}

// Second pass: workgroup `bucket` adds the bucket's survivors up in LDS and then adds its accumulators to the
// groups it alone owns (plain read-modify-write: the atomics of the first pass are complete).
constexpr int BUCKET_FOLD_THREADS = 1024;
template <int MM>
__global__ __launch_bounds__(BUCKET_FOLD_THREADS) void bucket_fold_kernel(BucketArgs b, unsigned long long* sums,
                                                                          unsigned long long* counts, int32_t G) {
  extern __shared__ __align__(16) unsigned long long bacc[];     // [MM + 1][groups of a bucket]
  const int R = 1 << b.shift;
  const int bucket = blockIdx.x;
  const unsigned int cnt = min(b.gcount[bucket], b.cap);
  if (cnt == 0u) return;                                         // (the same for the whole workgroup)
  for (int i = threadIdx.x; i < (MM + 1) * R; i += BUCKET_FOLD_THREADS) bacc[i] = 0ull;
  __syncthreads();
  const uint32_t* p = b.pairs + static_cast<size_t>(bucket) * b.cap * (1 + MM);
  for (unsigned int i = threadIdx.x; i < cnt; i += BUCKET_FOLD_THREADS) {
    const uint32_t* e = p + static_cast<size_t>(i) * (1 + MM);
    const uint32_t gl = e[0];
#pragma unroll
    for (int m = 0; m < MM; ++m)
      atomicAdd(&bacc[m * R + gl], static_cast<unsigned long long>(static_cast<long long>(static_cast<int32_t>(e[1 + m]))));
    atomicAdd(&bacc[MM * R + gl], 1ull);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < R; i += BUCKET_FOLD_THREADS) {
    const int64_t g = static_cast<int64_t>(bucket) * R + i;
    if (g >= G) break;
    const unsigned long long c = bacc[MM * R + i];
    if (c == 0ull) continue;
#pragma unroll
    for (int m = 0; m < MM; ++m) sums[static_cast<size_t>(m) * G + g] += bacc[m * R + i];
    if (counts) counts[g] += c;
  }
}

template <int MODE, bool WIDE, int NBL, int NML, int NMG, int NBG, int MM>
int launch_fast_inst(const FastArgs& a, const FastLaunch& L) {
  if constexpr (MODE == 2) {
    auto kernel = &scan_fast_bucket_kernel<NBL, NML, NMG, NBG, MM, WIDE>;
    if (L.lds > 64 * 1024)
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(L.lds)));
    // one resident set of workgroups (this kernel's registers allow fewer per compute unit than its LDS does)
    const int64_t resident = static_cast<int64_t>(num_cus()) * resident_per_cu(reinterpret_cast<const void*>(kernel), SCAN_THREADS, L.lds);
    const int64_t n_vec = a.n / 4;
    int64_t blocks = std::max<int64_t>(1, std::min<int64_t>(L.blocks, resident));
    int64_t per_block = (n_vec + blocks - 1) / blocks;
    per_block = std::max<int64_t>(SCAN_THREADS, (per_block + SCAN_THREADS - 1) / SCAN_THREADS * SCAN_THREADS);
    blocks = std::max<int64_t>(1, (n_vec + per_block - 1) / per_block);
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(SCAN_THREADS), L.lds, L.s, a, L.bucket, per_block);
    LQ_LAUNCH_CHECK("scan_fast_bucket_kernel");
    const size_t fold_lds = static_cast<size_t>(MM + 1) * (size_t{1} << L.bucket.shift) * 8;
    if (fold_lds > 64 * 1024)
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&bucket_fold_kernel<MM>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(fold_lds)));
    hipLaunchKernelGGL((bucket_fold_kernel<MM>), dim3(static_cast<unsigned>(L.bucket.buckets)), dim3(BUCKET_FOLD_THREADS),
                       fold_lds, L.s, L.bucket, a.gsums, a.gcounts, a.G);
    LQ_LAUNCH_CHECK("bucket_fold_kernel");
    return LQ_OK;
  } else {
    auto kernel = MODE == 1 ? &scan_fast_mem_kernel<NBL, NML, NMG, NBG, MM, WIDE> : &scan_fast_kernel<NBL, NML, NMG, NBG, MM, WIDE>;
    if (L.lds > 64 * 1024)
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(L.lds)));
    hipLaunchKernelGGL(kernel, dim3(L.blocks), dim3(SCAN_THREADS), L.lds, L.s, a, L.per_block);
    LQ_LAUNCH_CHECK("scan_fast_kernel");
    return LQ_OK;
  }
}
template <int MODE, bool WIDE, int NBL, int NML, int NMG, int NBG>
int launch_fast_m(const FastArgs& a, const FastLaunch& L) {
  // (more than 8,192 accumulators need at least two grouping dimensions of up to 255 values each)
  if constexpr (NBL + NML + NMG + NBG == 0 || (MODE != 0 && NBL + NBG < 2)) return -1;
  else {
    if (L.M == 1) return launch_fast_inst<MODE, WIDE, NBL, NML, NMG, NBG, 1>(a, L);
    if (L.M == 2) return launch_fast_inst<MODE, WIDE, NBL, NML, NMG, NBG, 2>(a, L);
    return -1;
  }
}
template <int MODE, bool WIDE, int NBL, int NML>
int launch_fast_g(const FastArgs& a, const FastLaunch& L) {
  if (L.nmg == 0 && L.nbg == 0) return launch_fast_m<MODE, WIDE, NBL, NML, 0, 0>(a, L);
  if (L.nmg == 1 && L.nbg == 0) return launch_fast_m<MODE, WIDE, NBL, NML, 1, 0>(a, L);
  if (L.nmg == 0 && L.nbg == 1) return launch_fast_m<MODE, WIDE, NBL, NML, 0, 1>(a, L);
  if (L.nmg == 1 && L.nbg == 1) return launch_fast_m<MODE, WIDE, NBL, NML, 1, 1>(a, L);
  // (two grouping attributes from tables too large for LDS: customer x supplier cities at large scale factors)
  if (L.nmg == 0 && L.nbg == 2) return launch_fast_m<MODE, WIDE, NBL, NML, 0, 2>(a, L);
  if (L.nmg == 1 && L.nbg == 2) return launch_fast_m<MODE, WIDE, NBL, NML, 1, 2>(a, L);
  return -1;
}
template <int MODE, bool WIDE, int NBL>
int launch_fast_ml(const FastArgs& a, const FastLaunch& L) {
  switch (L.nml) {
    case 0: return launch_fast_g<MODE, WIDE, NBL, 0>(a, L);
    case 1: return launch_fast_g<MODE, WIDE, NBL, 1>(a, L);
    case 2: return launch_fast_g<MODE, WIDE, NBL, 2>(a, L);
    case 3: return launch_fast_g<MODE, WIDE, NBL, 3>(a, L);
    default: return -1;
  }
}
// Returns -1 when there is no instantiation for this mix of dimensions.
// MODE: 0 accumulators in LDS, 1 in memory through atomics, 2 in memory through buckets.
// WIDE: instantiations that also take code tables of 16-bit entries (compiled in a source of their own).
template <int MODE, bool WIDE = false>
int launch_fast(const FastArgs& a, const FastLaunch& L) {
  switch (L.nbl) {
    case 0: return launch_fast_ml<MODE, WIDE, 0>(a, L);
    case 1: return launch_fast_ml<MODE, WIDE, 1>(a, L);
    case 2: return launch_fast_ml<MODE, WIDE, 2>(a, L);
    case 3: return launch_fast_ml<MODE, WIDE, 3>(a, L);
    default: return -1;
  }
}

}  // namespace
}  // namespace lq
#endif  // LQ_GROUPBY_FAST_H_
