// Decision-tree fusion (Section 3.3, Eq. 2): pre-fused per-dimension tables, the join-computation
// stage that adds them up per fact row and compares with h, and the non-fused pipeline
// ((T F > v) H) == h on the materialised join.
//
// Representation.  Instead of the signed partial sums of (D_k M_k F > v) H the tables hold, per
// dimension row r and leaf j, the number of nodes owned by that dimension on the path to leaf j
// whose outcome for r AGREES with the path (+1 node true, -1 node false).  This is the signed sum
// plus the number of the dimension's -1 entries in column j: never negative, at most the path
// length, so a byte suffices and packed 32-bit adds never carry between bytes.  Leaf j is reached
// iff the agreement counts of all tables add up to its path length (`target`), which is the same
// statement as R_j == h_j.
#include "lq_common.h"

namespace lq {
int launch_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                const void* bias, int64_t M, int32_t N, int32_t Kd, int relu, int32_t in_dtype,
                int32_t out_dtype, hipStream_t s);
namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct TreeArgs {
  int32_t p, l;
  int64_t ld;                 // row stride of the tables in bytes (multiple of 16)
  const int32_t* feature;
  const float* thr;
  const int8_t* H;
};

// ---------------------------------------------------------------- pre-fusion --------------

// target[j] = number of nonzeros in column j of H (the length of leaf j's path).  A workgroup takes 64
// leaves; its 16 wavefronts each count every 16th node (adjacent lanes read adjacent bytes of a row of
// H) and the partial counts meet in LDS.
constexpr int TT_THREADS = 1024;
__global__ __launch_bounds__(TT_THREADS) void tree_target_kernel(TreeArgs t, uint8_t* target) {
  __shared__ int part[TT_THREADS / 64][64];
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  int cnt = 0;
  if (j < t.l) {
    int q = slice;
    for (; q + 7 * (TT_THREADS / 64) < t.p; q += 8 * (TT_THREADS / 64)) {      // eight rows of H requested at a time
      int8_t hv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) hv[u] = t.H[static_cast<int64_t>(q + u * (TT_THREADS / 64)) * t.l + j];
#pragma unroll
      for (int u = 0; u < 8; ++u) cnt += hv[u] != 0;
    }
    for (; q < t.p; q += TT_THREADS / 64) cnt += t.H[static_cast<int64_t>(q) * t.l + j] != 0;
  }
  part[slice][lane] = cnt;
  __syncthreads();
  if (slice == 0 && j < t.ld) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < TT_THREADS / 64; ++w) total += part[w][lane];
    target[j] = j < t.l ? static_cast<uint8_t>(min(total, 255)) : 0xff;
  }
}

// One thread per (dimension row, leaf), leaves fastest.  col_off / c: the dimension's columns in T.
__global__ __launch_bounds__(256) void tree_project_kernel(TreeArgs t, const float* __restrict__ D,
                                                           int64_t ldd, int64_t rows, int32_t col_off,
                                                           int32_t c, uint8_t* __restrict__ out) {
  const int64_t total = rows * t.ld;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    const int64_t r = idx / t.ld;
    const int j = static_cast<int>(idx - r * t.ld);
    int agree = 0;
    if (j < t.l) {
      const float* dr = D + r * ldd;
      for (int q = 0; q < t.p; ++q) {
        const int f = t.feature[q] - col_off;
        if (f < 0 || f >= c) continue;                       // node owned by another table
        const int hv = t.H[static_cast<int64_t>(q) * t.l + j];
        if (hv == 0) continue;
        const bool bit = dr[f] > t.thr[q];
        agree += bit == (hv > 0);
      }
    }
    out[idx] = static_cast<uint8_t>(min(agree, 255));
  }
}


// Bit-mask version for trees of up to 256 nodes.  A wavefront takes one dimension row at a time:
// lane i evaluates node 64 w + i (if this dimension owns it) and a ballot packs the outcomes of 64
// nodes into one word; lane j then holds leaf j and counts the agreements with two popcounts per
// word against the +1 / -1 node masks of its path, which it built once from its column of H.
// r * (p + l) / 64 wavefront steps instead of r * l * p thread steps.
// All dimension tables go out in one launch: blockIdx.z selects the table.
struct ProjectArgs {
  const float* D[LQ_MAX_DIMS];
  uint8_t* out[LQ_MAX_DIMS];
  int64_t ldd[LQ_MAX_DIMS], rows[LQ_MAX_DIMS];
  int32_t col_off[LQ_MAX_DIMS], cols[LQ_MAX_DIMS];
};
template <int W>
__global__ __launch_bounds__(256) void tree_project_bits_kernel(TreeArgs t, ProjectArgs pa) {
  typedef unsigned long long u64;
  const int dim = blockIdx.z;
  const float* __restrict__ D = pa.D[dim];
  uint8_t* __restrict__ out = pa.out[dim];
  const int64_t ldd = pa.ldd[dim], rows = pa.rows[dim];
  const int32_t col_off = pa.col_off[dim], c = pa.cols[dim];
  if (static_cast<int64_t>(blockIdx.x) * 16 >= rows) return;      // (a workgroup starts at row 16 blockIdx.x)
  const int lane = threadIdx.x & 63;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * 4;
  int fcol[W];
  float thr[W];
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const int q = 64 * w + lane;
    fcol[w] = -1; thr[w] = 0.f;
    if (q < t.p) {
      const int f = t.feature[q] - col_off;
      if (f >= 0 && f < c) { fcol[w] = f; thr[w] = t.thr[q]; }
    }
  }
  u64 owned[W];
#pragma unroll
  for (int w = 0; w < W; ++w) owned[w] = __ballot(fcol[w] >= 0);
  {                                       // blockIdx.y selects the 64 leaves this workgroup writes
    const int j0 = blockIdx.y * 64;
    const int j = j0 + lane;
    u64 plus[W], minus[W];
#pragma unroll
    for (int w = 0; w < W; ++w) { plus[w] = 0; minus[w] = 0; }
    // sixteen entries of the leaf's column of H are requested at a time; which nodes this dimension owns
    // is known from the lanes' own nodes (owned[w], the same for every lane)
    if (j < t.l) {
#pragma unroll
      for (int w = 0; w < W; ++w)
        for (int b0 = 0; b0 < 64 && 64 * w + b0 < t.p; b0 += 16) {
          int hv[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) {
            const int q = 64 * w + b0 + u;
            const bool use = q < t.p && ((owned[w] >> (b0 + u)) & 1ull);
            hv[u] = use ? t.H[static_cast<int64_t>(q) * t.l + j] : 0;
          }
#pragma unroll
          for (int u = 0; u < 16; ++u) {
            if (hv[u] > 0) plus[w] |= 1ull << (b0 + u);
            if (hv[u] < 0) minus[w] |= 1ull << (b0 + u);
          }
        }
    }
    for (int64_t r0 = wave * 4; r0 < rows; r0 += nwaves * 4) {
      float v[4][W];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t r = min(r0 + u, rows - 1);
#pragma unroll
        for (int w = 0; w < W; ++w) v[u][w] = fcol[w] >= 0 ? D[r * ldd + fcol[w]] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int agree = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
          const u64 bits = __ballot(fcol[w] >= 0 && v[u][w] > thr[w]);
          agree += __popcll(bits & plus[w]) + __popcll(~bits & minus[w]);
        }
        if (r0 + u < rows && j < t.ld) out[(r0 + u) * t.ld + j] = static_cast<uint8_t>(min(agree, 255));
      }
    }
  }
}

// Sparse version of the same computation.  A column of H has at most 255 nonzeros (longer paths are
// unsupported), so a workgroup first turns the H columns of its 64 leaves into per-leaf lists of the
// nodes this dimension owns (node number, sign bit) in LDS and then walks only those lists for every
// (dimension row, leaf): r * l * depth / K evaluations instead of r * l * p.
constexpr int TP_COLS = 8;          // leaves per workgroup (4: slower on large tables, 32: the lists are built four times as often)
constexpr int TP_MAXPATH = 255;     // list capacity per leaf (longer paths are unsupported: a byte holds the count)
// The lists hold, per entry, the column within the dimension table (bit 31: the path wants the test
// false) and the threshold; entry e of all leaves lies side by side, so the lanes of a wavefront
// (lane = leaf) read neighbouring LDS words.
constexpr int TPS_THREADS = 1024;   // a large workgroup builds its lists in two rounds of loads and then has 16 wavefronts of row work
__global__ __launch_bounds__(TPS_THREADS) void tree_project_sparse_kernel(TreeArgs t, const float* __restrict__ D,
                                                                          int64_t ldd, int64_t rows, int32_t col_off,
                                                                          int32_t c, uint8_t* __restrict__ out,
                                                                          int64_t rows_per_block, int32_t col_tiles) {
  __shared__ unsigned int ent[TP_MAXPATH][TP_COLS];
  __shared__ float thr_l[TP_MAXPATH][TP_COLS];
  __shared__ int count[TP_COLS];
  const int tid = threadIdx.x;
  // Workgroups are dealt to the eight XCDs in turn (blockIdx.x % 8).  The 16 column tiles that share a
  // 128-byte line of an output row should meet in one L2, so each XCD takes a contiguous eighth of the tiles.
  int tile = blockIdx.x;
  if (col_tiles % 8 == 0) tile = (blockIdx.x % 8) * (col_tiles / 8) + blockIdx.x / 8;
  const int j0 = tile * TP_COLS;
  const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
  const int64_t r1 = min(rows, r0 + rows_per_block);
  if (tid < TP_COLS) count[tid] = 0;
  __syncthreads();
  {
    constexpr int QS = TPS_THREADS / TP_COLS;             // nodes covered by one round of the workgroup
    const int j = tid % TP_COLS;
    if (j0 + j < t.l)
      for (int q0 = tid / TP_COLS; q0 < t.p; q0 += 8 * QS) {   // eight entries of H requested at a time
        int hv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int q = q0 + u * QS;
          hv[u] = q < t.p ? t.H[static_cast<int64_t>(q) * t.l + j0 + j] : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (hv[u] == 0) continue;
          const int q = q0 + u * QS;
          const int f = t.feature[q] - col_off;
          if (f < 0 || f >= c) continue;                     // node owned by another table
          const int slot = atomicAdd(&count[j], 1);
          if (slot < TP_MAXPATH) {
            ent[slot][j] = static_cast<unsigned int>(f) | (hv[u] < 0 ? 0x80000000u : 0u);
            thr_l[slot][j] = t.thr[q];
          }
        }
      }
  }
  __syncthreads();
  const int64_t total = (r1 - r0) * TP_COLS;
  for (int64_t idx = tid; idx < total; idx += TPS_THREADS) {
    const int64_t r = r0 + idx / TP_COLS;
    const int j = static_cast<int>(idx % TP_COLS);
    if (j0 + j >= t.ld) continue;
    int agree = 0;
    if (j0 + j < t.l) {
      const float* dr = D + r * ldd;
      const int n = min(count[j], TP_MAXPATH);
      for (int e = 0; e < n; ++e) {
        const unsigned int v = ent[e][j];
        const bool bit = dr[v & 0x7fffffffu] > thr_l[e][j];
        agree += bit == ((v & 0x80000000u) == 0u);
      }
    }
    out[r * t.ld + j0 + j] = static_cast<uint8_t>(min(agree, 255));
  }
}

// ---------------------------------------------------------------- fused join ---------------

struct FusedTreeArgs {
  int64_t n;
  int32_t K;
  const uint8_t* T[LQ_MAX_DIMS];
  const int32_t* fk[LQ_MAX_DIMS];
  int32_t chunks;              // ld / 16
  const uint8_t* target;
  int32_t* leaf;
  uint8_t* onehot;
  int32_t onehot_vec_ok;       // 16-byte stores into onehot rows are legal
  // nodes that test fact-table columns (evaluated per fact row)
  const float* X; int64_t ldx; int32_t c_f; int32_t has_fact_nodes;
  int32_t lists;               // the workgroup builds per-leaf lists of the fact-side nodes in LDS
  TreeArgs t;
};

// 0x80 in every byte of w that is zero, 0 elsewhere (exact, no borrow effects).
__device__ __forceinline__ unsigned int zero_bytes(unsigned int w) {
  const unsigned int t = (w & 0x7f7f7f7fu) + 0x7f7f7f7fu;
  return ~(t | w | 0x7f7f7f7fu);
}

// G lanes per fact row; lane c handles 16-leaf chunks c, c + G, ...
// The nodes that test fact columns are listed once per workgroup (in LDS, in any order), so that the
// per-row work on them is proportional to their number rather than to the size of the tree.
// With such nodes (dynamic LDS of 16 * chunks bytes and more) the workgroup also works out, once, what the tables
// alone must add up to for leaf j: target_j minus the number of fact-side nodes on its path (each table's
// count reaches at most the number of nodes that table owns there).  A row then evaluates fact-side nodes
// only for the leaves whose table sum equals that number - a few per row instead of all of them - and a
// workgroup strides over many groups of rows, so that the once-per-workgroup part stays small.
// With `lists` (trees of up to FT_LISTS_MAX_L leaves) the same pass over H also leaves, per leaf, the list of fact-side
// nodes on its path in LDS, so that a possible leaf costs a few LDS reads instead of a column of H.
constexpr int FT_LIST = 1024;           // listed nodes; a tree with more of them walks all nodes instead
constexpr int FT_NEED_MAX = 48 * 1024;  // leaves (padded) whose table-only targets fit in LDS (trees have at most 16,384)
constexpr int FT_LISTS_MAX_L = 8192;    // leaves (padded) up to which per-leaf lists are built
constexpr int FT_LISTS_CAP = 8192;      // list entries in all (2 bytes each: place in the node list, bit 15 = wants the test false)
inline size_t ft_lds_bytes(int chunks, bool lists) {
  return 16 * static_cast<size_t>(chunks) +
         (lists ? 8 * FT_LIST + round_up(2 * (16 * static_cast<size_t>(chunks) + 1), 16) + 2 * FT_LISTS_CAP : 0);
}
template <int G>
__global__ __launch_bounds__(256) void fused_tree_kernel(FusedTreeArgs a) {
  constexpr int RPB = 256 / G;
  __shared__ int fact_q[FT_LIST];
  __shared__ int fact_cnt;
  extern __shared__ __align__(16) uint8_t need[];
  if (a.has_fact_nodes) {
    if (threadIdx.x == 0) fact_cnt = 0;
    __syncthreads();
    for (int q0 = 0; q0 < a.t.p; q0 += 256) {
      const int q = q0 + threadIdx.x;
      const bool mine = q < a.t.p && static_cast<unsigned int>(a.t.feature[q]) < static_cast<unsigned int>(a.c_f);
      const unsigned long long bal = __ballot(mine);
      int base = 0;
      if ((threadIdx.x & 63) == 0 && bal) base = atomicAdd(&fact_cnt, __builtin_popcountll(bal));
      base = __shfl(base, 0, 64);
      const int pos = base + __builtin_popcountll(bal & ((1ull << (threadIdx.x & 63)) - 1ull));
      if (mine && pos < FT_LIST) fact_q[pos] = q;
      __syncthreads();
    }
  }
  const int n_fact = a.has_fact_nodes ? fact_cnt : 0;
  const bool listed = n_fact <= FT_LIST;
  const int n_walk = listed ? n_fact : a.t.p;
  const int padded = 16 * a.chunks;
  uint2* ft = reinterpret_cast<uint2*>(need + padded);                        // {column, threshold bits} of listed node i
  unsigned short* off = reinterpret_cast<unsigned short*>(need + padded + 8 * FT_LIST);
  unsigned short* ent = off + (2 * (padded + 1) + 15) / 16 * 8;
  __shared__ int seg[257];
  bool lists = a.lists && listed;
  if (a.has_fact_nodes) {
    for (int j = threadIdx.x; j < padded; j += 256) {
      int own = 0;
      if (j < a.t.l)
        for (int i = 0; i < n_walk; ++i) {
          const int q = listed ? fact_q[i] : i;
          if (!listed && static_cast<unsigned int>(a.t.feature[q]) >= static_cast<unsigned int>(a.c_f)) continue;
          own += a.t.H[static_cast<int64_t>(q) * a.t.l + j] != 0 ? 1 : 0;
        }
      need[j] = static_cast<uint8_t>(a.target[j] - own);       // (padding: 0xFF, which no sum of table entries reaches)
      if (lists) off[j + 1] = static_cast<unsigned short>(own);
    }
    __syncthreads();
    if (lists) {
      // running sums of the list lengths: a thread owns a run of consecutive leaves
      const int per = (padded + 255) / 256, lo = min(padded, per * static_cast<int>(threadIdx.x)), hi = min(padded, lo + per);
      int sum = 0;
      for (int j = lo; j < hi; ++j) sum += off[j + 1];
      seg[threadIdx.x + 1] = sum;
      __syncthreads();
      if (threadIdx.x == 0) {
        seg[0] = 0;
        for (int i = 1; i <= 256; ++i) seg[i] += seg[i - 1];
        off[0] = 0;
      }
      __syncthreads();
      lists = seg[256] <= FT_LISTS_CAP;
      if (lists) {
        int run = seg[threadIdx.x];
        for (int j = lo; j < hi; ++j) { run += off[j + 1]; off[j + 1] = static_cast<unsigned short>(run); }
        for (int i = threadIdx.x; i < n_fact; i += 256) {
          const int q = fact_q[i];
          ft[i] = make_uint2(static_cast<unsigned int>(a.t.feature[q]), __float_as_uint(a.t.thr[q]));
        }
      }
      __syncthreads();
      if (lists) {
        for (int j = threadIdx.x; j < a.t.l; j += 256) {
          int at = off[j];
          for (int i = 0; i < n_fact; ++i) {
            const int hv = a.t.H[static_cast<int64_t>(fact_q[i]) * a.t.l + j];
            if (hv != 0) ent[at++] = static_cast<unsigned short>(i | (hv < 0 ? 0x8000 : 0));
          }
        }
        __syncthreads();
      }
    }
  }
  const int sub = threadIdx.x / G, c = threadIdx.x % G;
  const int64_t groups = (a.n + RPB - 1) / RPB;
  for (int64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const int64_t row = grp * RPB + sub;
    const bool live = row < a.n;
    const int64_t rr = live ? row : a.n - 1;
    int64_t base[LQ_MAX_DIMS];
#pragma unroll
    for (int k = 0; k < LQ_MAX_DIMS; ++k)
      if (k < a.K) base[k] = static_cast<int64_t>(a.fk[k][rr]) * a.t.ld;
    const float* xr = a.has_fact_nodes ? a.X + rr * a.ldx : nullptr;
    int first = 0x7fffffff;
    for (int ch = c; ch < a.chunks; ch += G) {
      v4u sum = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int k = 0; k < LQ_MAX_DIMS; ++k)
        if (k < a.K) sum += *reinterpret_cast<const v4u*>(a.T[k] + base[k] + 16 * ch);
      v4u hit;
      if (a.has_fact_nodes) {
        const v4u nd = *reinterpret_cast<const v4u*>(need + 16 * ch);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          hit[d] = 0u;
          for (unsigned int cand = zero_bytes(sum[d] ^ nd[d]); cand != 0u; cand &= cand - 1u) {
            const int at = __builtin_ctz(cand) >> 3;             // byte of this word whose tables are all at their maximum
            const int j = 16 * ch + 4 * d + at;
            bool ok = true;
            if (lists) {
              for (int e = off[j]; ok && e < off[j + 1]; ++e) {
                const unsigned int en = ent[e];
                const uint2 node = ft[en & 0x7fffu];
                ok = (xr[node.x] > __uint_as_float(node.y)) == ((en & 0x8000u) == 0u);
              }
            } else {
              for (int i = 0; ok && i < n_walk; ++i) {
                const int q = listed ? fact_q[i] : i;
                const int hv = a.t.H[static_cast<int64_t>(q) * a.t.l + j];
                if (hv == 0) continue;
                const int f = a.t.feature[q];
                if (static_cast<unsigned int>(f) >= static_cast<unsigned int>(a.c_f)) continue;
                ok = (xr[f] > a.t.thr[q]) == (hv > 0);
              }
            }
            if (ok) hit[d] |= 0x80u << (8 * at);
          }
        }
      } else {
        const v4u tg = *reinterpret_cast<const v4u*>(a.target + 16 * ch);
#pragma unroll
        for (int d = 0; d < 4; ++d) hit[d] = zero_bytes(sum[d] ^ tg[d]);
      }
#pragma unroll
      for (int d = 0; d < 4; ++d)
        if (hit[d] != 0u) first = min(first, 16 * ch + 4 * d + (__builtin_ctz(hit[d]) >> 3));
      if (a.onehot && live) {
        uint8_t* o = a.onehot + row * a.t.l + 16 * ch;
        if (a.onehot_vec_ok && 16 * ch + 16 <= a.t.l) {
          const v4u ones = {hit[0] >> 7, hit[1] >> 7, hit[2] >> 7, hit[3] >> 7};
          __builtin_nontemporal_store(ones, reinterpret_cast<v4u*>(o));
        } else {
#pragma unroll
          for (int b = 0; b < 16; ++b)
            if (16 * ch + b < a.t.l) o[b] = static_cast<uint8_t>((hit[b >> 2] >> (8 * (b & 3) + 7)) & 1u);
        }
      }
    }
#pragma unroll
    for (int m = 1; m < G; m <<= 1) first = min(first, __shfl_xor(first, m, 64));
    if (a.leaf && live && c == 0) a.leaf[row] = first == 0x7fffffff ? -1 : first;
  }
}

// The same join stage for trees of up to 4,096 leaves without fact-table nodes, organised so that a
// wavefront has many gathers in flight: it owns 64 consecutive fact rows, reads their keys once,
// coalesced (lane = row), and hands them to the G-lane groups through the cross-lane network; in
// pass t group g works on row (64 / G) t + g.  The gathers of up to four passes are issued before
// the first is consumed.
// KT: number of dimensions when it is 1..4 (loops unroll without guards), 0 = any number.
// CPL: 16-leaf chunks per lane (1; 2 or 4 with G = 64, for 1,025 to 4,096 leaves: lane c takes chunks c, c + 64, ...).
template <int G, int KT, int CPL = 1>
__global__ __launch_bounds__(256) void fused_tree_batch_kernel(FusedTreeArgs a) {
  static_assert(CPL == 1 || G == 64, "several chunks per lane: all lanes on one row");
  constexpr int KK = KT > 0 ? KT : LQ_MAX_DIMS;
  constexpr int RPP = 64 / G;                 // rows per pass
  constexpr int PB = (G < 4 ? G : 4) / CPL;   // passes in flight together (G passes cover the 64 rows)
  const int lane = threadIdx.x & 63, g = lane / G, c = lane % G;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t row0 = wave * 64;
  if (row0 >= a.n) return;
  const int64_t myrow = min(row0 + lane, a.n - 1);
  int key[KK];
  const uint8_t* tab[KK];
#pragma unroll
  for (int k = 0; k < KK; ++k) {
    const bool used = KT > 0 || k < a.K;
    key[k] = used ? a.fk[k][myrow] : 0;
    tab[k] = (used ? a.T[k] : a.T[0]) + 16 * c;
  }
  bool active[CPL];
  v4u tg[CPL];
#pragma unroll
  for (int h = 0; h < CPL; ++h) {
    active[h] = c + G * h < a.chunks;
    tg[h] = v4u{0u, 0u, 0u, 0u};
    if (active[h]) tg[h] = *reinterpret_cast<const v4u*>(a.target + 16 * (c + G * h));
  }
  for (int pb = 0; pb < G; pb += PB) {
    v4u sum[PB][CPL];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int src = RPP * (pb + u) + g;     // the lane that holds this row's keys
#pragma unroll
      for (int h = 0; h < CPL; ++h) sum[u][h] = v4u{0u, 0u, 0u, 0u};
#pragma unroll
      for (int k = 0; k < KK; ++k)
        if (KT > 0 || k < a.K) {
          const int64_t j = __shfl(key[k], src, 64);
#pragma unroll
          for (int h = 0; h < CPL; ++h)
            if (active[h]) sum[u][h] += *reinterpret_cast<const v4u*>(tab[k] + j * a.t.ld + 16 * G * h);
        }
    }
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int64_t row = row0 + RPP * (pb + u) + g;
      const bool live = row < a.n;
      int first = 0x7fffffff;
#pragma unroll
      for (int h = 0; h < CPL; ++h) {
        v4u hit = {0u, 0u, 0u, 0u};
        if (active[h]) {
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            hit[d] = zero_bytes(sum[u][h][d] ^ tg[h][d]);
            // 0x80 marks a matching byte: its position is that of the lowest set bit
            const int at = 16 * (c + G * h) + 4 * d + ((__builtin_ctz(hit[d] | 0x80000000u)) >> 3);
            first = min(first, hit[d] != 0u ? at : 0x7fffffff);
          }
          if (a.onehot && live) {               // (this kernel is only chosen when whole 16-byte stores fit)
            const v4u ones = {hit[0] >> 7, hit[1] >> 7, hit[2] >> 7, hit[3] >> 7};
            __builtin_nontemporal_store(ones, reinterpret_cast<v4u*>(a.onehot + row * a.t.l + 16 * (c + G * h)));
          }
        }
      }
#pragma unroll
      for (int m = 1; m < G; m <<= 1) first = min(first, __shfl_xor(first, m, 64));
      if (a.leaf && live && c == 0) a.leaf[row] = first == 0x7fffffff ? -1 : first;
    }
  }
}

// ---------------------------------------------------------------- non-fused ----------------

// The non-fused pipeline in the matrix form of Section 3.3.1 on a chunk of the materialised join:
//   step 1-2  B = (T F > v): F holds a single 1 per column, so T F is the gather of one column of
//             T per node; B is written as bf16 0 / 1, its row padded with zeros to a multiple of 8
//   step 3    R = B H as a dense product on the matrix cores (H in bf16; 0 / +-1 values and counts
//             up to 255 are exact in bf16 x bf16 -> fp32)
//   step 4    (R == h), h_j = number of +1 entries of column j of H
__global__ __launch_bounds__(256) void tree_bits_kernel(TreeArgs t, const float* __restrict__ T, int64_t ldt,
                                                        int64_t rows, bf16_t* __restrict__ B, int64_t ldb) {
  const int64_t total = rows * ldb;
  for (int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; idx < total;
       idx += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t r = idx / ldb;
    const int q = static_cast<int>(idx - r * ldb);
    const bool bit = q < t.p && T[r * ldt + t.feature[q]] > t.thr[q];
    B[idx] = bit ? static_cast<bf16_t>(0x3F80) : static_cast<bf16_t>(0);
  }
}

// H as bf16 [p_pad x ldh] (zero padding) and h as fp32 [l].
__global__ __launch_bounds__(256) void tree_h_kernel(TreeArgs t, int32_t p_pad, bf16_t* __restrict__ Hb, int64_t ldh,
                                                     float* __restrict__ hplus) {
  const int64_t total = static_cast<int64_t>(p_pad) * ldh;
  for (int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; idx < total;
       idx += static_cast<int64_t>(gridDim.x) * 256) {
    const int q = static_cast<int>(idx / ldh), j = static_cast<int>(idx - static_cast<int64_t>(q) * ldh);
    const int hv = (q < t.p && j < t.l) ? t.H[static_cast<int64_t>(q) * t.l + j] : 0;
    Hb[idx] = hv > 0 ? static_cast<bf16_t>(0x3F80) : (hv < 0 ? static_cast<bf16_t>(0xBF80) : static_cast<bf16_t>(0));
  }
  for (int j = blockIdx.x * 256 + threadIdx.x; j < t.l; j += gridDim.x * 256) {
    int cnt = 0;
    for (int q = 0; q < t.p; ++q) cnt += t.H[static_cast<int64_t>(q) * t.l + j] > 0;
    hplus[j] = static_cast<float>(cnt);
  }
}

// One wavefront per row: lanes sweep the leaves, a ballot finds the first match.
__global__ __launch_bounds__(256) void tree_match_kernel(int32_t l, const float* __restrict__ R, int64_t ldr,
                                                         int64_t rows, int64_t row0, const float* __restrict__ hplus,
                                                         int32_t* __restrict__ leaf, uint8_t* __restrict__ onehot) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * 4;
  for (int64_t r = wave; r < rows; r += nwaves) {
    int first = -1;
    for (int j0 = 0; j0 < l; j0 += 64) {
      const int j = j0 + lane;
      const bool hit = j < l && R[r * ldr + j] == hplus[j];
      if (onehot && j < l) onehot[(row0 + r) * l + j] = hit;
      const unsigned long long m = __ballot(hit);
      if (first < 0 && m != 0ull) first = j0 + __builtin_ctzll(m);
    }
    if (leaf && lane == 0) leaf[row0 + r] = first;
  }
}

// ---------------------------------------------------------------- leaf masks ---------------
//
// Compressed form of the pre-fused tables.  The agreement count of dimension k for (row r, leaf j)
// is at most the number of nodes k owns on the path to j, and the counts of all dimensions add up
// to the path length exactly when each of them reaches its own maximum.  One bit per (row, leaf) -
// "this dimension row agrees with the path to leaf j on every node the dimension owns" - therefore
// carries all the join stage needs, and the sum-and-compare of Eq. 2 becomes a bitwise AND of one
// mask row per dimension: 8 bytes instead of 64 gathered per dimension for a 64-leaf tree.

typedef unsigned long long u64;

// Workgroup (blockIdx.y = word w) for up to 1,024 rows.  First the number of nodes this dimension
// owns on the path to each of the 64 leaves of the word (lane = leaf, the wavefronts split the
// nodes, eight loads in flight each, H only read for nodes the dimension owns); then every thread compares
// the 64 table bytes of its row with those counts, four bytes per operation, and packs the 64 outcomes
// into the mask word of its row.
constexpr int CMP_THREADS = 1024;   // sixteen wavefronts split the nodes (256 threads: 0.117 ms for the three tables at 1,024 leaves)
// All dimension tables in one launch: blockIdx.z selects the table, workgroups past its rows leave at once.
struct CompressArgs {
  const uint8_t* table[LQ_MAX_DIMS];
  u64* masks[LQ_MAX_DIMS];
  int64_t rows[LQ_MAX_DIMS];
  int32_t col_off[LQ_MAX_DIMS], cols[LQ_MAX_DIMS];
};
__global__ __launch_bounds__(CMP_THREADS) void tree_compress_kernel(TreeArgs t, CompressArgs ca, int32_t words) {
  constexpr int WAVES = CMP_THREADS / 64;
  const int dim = blockIdx.z;
  const int64_t rows = ca.rows[dim];
  if (static_cast<int64_t>(blockIdx.x) * CMP_THREADS >= rows) return;
  const uint8_t* __restrict__ table = ca.table[dim];
  u64* __restrict__ masks = ca.masks[dim];
  const int32_t col_off = ca.col_off[dim], c = ca.cols[dim];
  __shared__ int part[WAVES][64];
  __shared__ unsigned int own_dw[16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, w = blockIdx.y;
  const int j = 64 * w + lane;
  int own = 0;
  for (int q0 = wave; q0 < t.p; q0 += 8 * WAVES) {
    int h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int q = q0 + WAVES * e;                       // (the same for every lane: the test on the column is uniform)
      const int f = q < t.p ? t.feature[q] - col_off : -1;
      h[e] = (f >= 0 && f < c && j < t.l) ? t.H[static_cast<int64_t>(q) * t.l + j] : 0;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) own += h[e] != 0 ? 1 : 0;
  }
  part[wave][lane] = own;
  __syncthreads();
  if (threadIdx.x < 64) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) tot += part[i][lane];
    tot = j < t.l ? min(tot, 255) : 0xff;               // leaves past l never match (their table bytes are 0)
    part[0][lane] = tot;
  }
  __syncthreads();
  if (threadIdx.x < 16)
    own_dw[threadIdx.x] = static_cast<unsigned int>(part[0][4 * threadIdx.x]) | (static_cast<unsigned int>(part[0][4 * threadIdx.x + 1]) << 8) |
                          (static_cast<unsigned int>(part[0][4 * threadIdx.x + 2]) << 16) | (static_cast<unsigned int>(part[0][4 * threadIdx.x + 3]) << 24);
  __syncthreads();
  const int pieces = static_cast<int>(min<int64_t>(4, (t.ld - 64 * w) / 16));   // 16-byte pieces of a row that exist in this word
  // (several runs of rows per workgroup, so that fewer workgroups scan H, changed nothing: 0.066 against 0.070 ms)
  const int64_t r = static_cast<int64_t>(blockIdx.x) * CMP_THREADS + threadIdx.x;
  if (r >= rows) return;
  const uint8_t* src = table + r * t.ld + 64 * w;
  v4u tb[4];
#pragma unroll
  for (int pc = 0; pc < 4; ++pc) tb[pc] = pc < pieces ? *reinterpret_cast<const v4u*>(src + 16 * pc) : v4u{0u, 0u, 0u, 0u};
  u64 word = 0ull;
#pragma unroll
  for (int pc = 0; pc < 4; ++pc)
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const unsigned int fl = zero_bytes(tb[pc][d] ^ own_dw[4 * pc + d]) >> 7;     // bit 0, 8, 16, 24: the byte matches
      const unsigned int nib = (fl & 1u) | ((fl >> 7) & 2u) | ((fl >> 14) & 4u) | ((fl >> 21) & 8u);
      word |= static_cast<u64>(nib) << (16 * pc + 4 * d);
    }
  masks[r * words + w] = word;
}

// Nodes that test the fact table's own columns have no table to be folded into: their outcome is
// known only per fact row.  For such a node two mask rows say which leaves stay possible when the
// test comes out true (every leaf whose path does not need it false) and when it comes out false;
// the join stage evaluates the node on the fact row and ANDs the row that applies.  The nodes are
// packed (tree order) into one buffer: count, column and threshold per node, then the mask pairs.
struct FactSide {
  const float* X;               // NULL: the fact table has no columns
  int64_t ldx;
  int32_t c_f, vec_x;           // vec_x: rows of X can be read as 16-byte pieces
  const int32_t* cnt;
  const int32_t* feat;
  const float* thr;
  const u64* tf;                // [(node * words + w) * 2 + {0: test true, 1: test false}]
  // Per leaf, the fact-side nodes on its path (cnt[1] != 0: the lists are there): entries leaf_off[j] .. leaf_off[j + 1),
  // each {column, 1 when the path wants the test false, threshold bits, position of the node in tf}.
  const int32_t* leaf_off;
  const uint4* leaf_ent;
};
struct FactBuf { int32_t* cnt; int32_t* feat; float* thr; u64* tf; int32_t* leaf_off; uint4* leaf_ent; };
constexpr int FACT_LIST_PER_LEAF = 64;     // list entries the buffer has room for, per leaf on average
// cnt[0]: fact-side nodes, cnt[1]: the per-leaf lists are complete, cnt[2]: their total length.
FactBuf fact_buf(void* p, int32_t n_nodes, int32_t n_leaves) {
  char* b = static_cast<char*>(p);
  const size_t tf = round_up(16 + 8 * static_cast<size_t>(n_nodes), 16);
  const size_t off = tf + static_cast<size_t>(n_nodes) * lq_tree_mask_words(n_leaves) * 16;
  const size_t ent = off + round_up(4 * (static_cast<size_t>(n_leaves) + 1), 16);
  return FactBuf{reinterpret_cast<int32_t*>(b), reinterpret_cast<int32_t*>(b + 16),
                 reinterpret_cast<float*>(b + 16 + 4 * static_cast<size_t>(n_nodes)), reinterpret_cast<u64*>(b + tf),
                 reinterpret_cast<int32_t*>(b + off), reinterpret_cast<uint4*>(b + ent)};
}

// The per-leaf lists: count, running sum (one workgroup), fill.  A leaf's list has the fact-side nodes with a nonzero
// entry in its column of H, in node order.
// Count and fill: a workgroup takes 64 leaves (lane = leaf) and its 16 wavefronts take consecutive runs of the nodes,
// so that a list stays in node order: a wavefront's entries follow those of the wavefronts before it.
constexpr int FL_WAVES = 16;
__device__ __forceinline__ int fact_list_count_run(const TreeArgs& t, int32_t c_f, int j, int q_lo, int q_hi) {
  int count = 0;
  for (int q = q_lo; q < q_hi; ++q)
    if (static_cast<unsigned int>(t.feature[q]) < static_cast<unsigned int>(c_f))       // (the same for every lane)
      count += (j < t.l && t.H[static_cast<int64_t>(q) * t.l + j] != 0) ? 1 : 0;
  return count;
}
__global__ __launch_bounds__(64 * FL_WAVES) void tree_fact_list_count_kernel(TreeArgs t, int32_t c_f, int32_t* leaf_off) {
  __shared__ int part[FL_WAVES][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  const int run = (t.p + FL_WAVES - 1) / FL_WAVES;
  part[wave][lane] = fact_list_count_run(t, c_f, j, min(t.p, wave * run), min(t.p, (wave + 1) * run));
  __syncthreads();
  if (wave == 0) {
    int count = 0;
#pragma unroll
    for (int w = 0; w < FL_WAVES; ++w) count += part[w][lane];
    if (j == 0) leaf_off[0] = 0;
    if (j < t.l) leaf_off[j + 1] = count;
  }
}
__global__ __launch_bounds__(1024) void tree_fact_list_scan_kernel(int32_t* leaf_off, int32_t l, int32_t* cnt, int64_t capacity) {
  __shared__ int part[1024];
  __shared__ long long carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 1; base <= l; base += 1024) {
    const int i = base + threadIdx.x;
    const int v = i <= l ? leaf_off[i] : 0;
    part[threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
      const int add = threadIdx.x >= d ? part[threadIdx.x - d] : 0;
      __syncthreads();
      part[threadIdx.x] += add;
      __syncthreads();
    }
    const long long total = carry + part[threadIdx.x];
    if (i <= l) leaf_off[i] = total > 0x7fffffffLL ? 0x7fffffff : static_cast<int32_t>(total);
    __syncthreads();
    if (threadIdx.x == 1023) carry = total;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    cnt[2] = carry > 0x7fffffffLL ? 0x7fffffff : static_cast<int32_t>(carry);
    cnt[1] = carry <= capacity ? 1 : 0;
  }
}
__global__ __launch_bounds__(64 * FL_WAVES) void tree_fact_list_fill_kernel(TreeArgs t, int32_t c_f, const int32_t* cnt,
                                                                            const int32_t* leaf_off, uint4* ent) {
  __shared__ int part[FL_WAVES][64];      // entries of the leaf in the wavefront's run of nodes
  __shared__ int before[FL_WAVES];        // fact-side nodes before the wavefront's run (their place in the packed list)
  if (cnt[1] == 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  const int run = (t.p + FL_WAVES - 1) / FL_WAVES;
  const int q_lo = min(t.p, wave * run), q_hi = min(t.p, (wave + 1) * run);
  part[wave][lane] = fact_list_count_run(t, c_f, j, q_lo, q_hi);
  if (lane == 0) {
    int nodes = 0;
    for (int q = q_lo; q < q_hi; ++q) nodes += static_cast<unsigned int>(t.feature[q]) < static_cast<unsigned int>(c_f) ? 1 : 0;
    before[wave] = nodes;
  }
  __syncthreads();
  if (j >= t.l) return;
  int at = leaf_off[j], pos = 0;
  for (int w = 0; w < wave; ++w) { at += part[w][lane]; pos += before[w]; }
  for (int q = q_lo; q < q_hi; ++q) {
    const int f = t.feature[q];
    if (static_cast<unsigned int>(f) >= static_cast<unsigned int>(c_f)) continue;
    const int h = t.H[static_cast<int64_t>(q) * t.l + j];
    if (h != 0) ent[at++] = make_uint4(static_cast<unsigned int>(f), h < 0 ? 1u : 0u, __float_as_uint(t.thr[q]), static_cast<unsigned int>(pos));
    ++pos;
  }
}

// Workgroup = 16 consecutive nodes, wavefront = 4 of them, lane = leaf of the current mask word.
// The position of a fact-owned node in the packed list is the number of such nodes before it.
__global__ __launch_bounds__(256) void tree_fact_masks_kernel(TreeArgs t, int32_t c_f, int32_t words, FactBuf out) {
  __shared__ int part[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q_lo = 16 * blockIdx.x;
  int before = 0;
  for (int q = threadIdx.x; q < q_lo; q += 256) before += static_cast<unsigned int>(t.feature[q]) < static_cast<unsigned int>(c_f) ? 1 : 0;
#pragma unroll
  for (int m = 32; m; m >>= 1) before += __shfl_xor(before, m, 64);
  if (lane == 0) part[wave] = before;
  __syncthreads();
  const int base = part[0] + part[1] + part[2] + part[3];
  const bool owned = lane < 16 && q_lo + lane < t.p &&
                     static_cast<unsigned int>(t.feature[q_lo + lane]) < static_cast<unsigned int>(c_f);   // (a negative column belongs to no table)
  const unsigned int chunk = static_cast<unsigned int>(__ballot(owned));     // bit i: node q_lo + i is the fact table's
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *out.cnt = base + __builtin_popcount(chunk);
  if (((chunk >> (4 * wave)) & 0xfu) == 0u) return;
  for (int w = 0; w < words; ++w) {
    const int j = 64 * w + lane;
    int h[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int q = q_lo + 4 * wave + e;
      h[e] = (q < t.p && j < t.l) ? t.H[static_cast<int64_t>(q) * t.l + j] : 0;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = 4 * wave + e;
      const u64 when_true = __ballot(j < t.l && h[e] >= 0), when_false = __ballot(j < t.l && h[e] <= 0);
      if (((chunk >> i) & 1u) && lane == 0) {
        const int pos = base + __builtin_popcount(chunk & ((1u << i) - 1u));
        const int64_t o = (static_cast<int64_t>(pos) * words + w) * 2;
        out.tf[o] = when_true;
        out.tf[o + 1] = when_false;
        if (w == 0) { out.feat[pos] = t.feature[q_lo + i]; out.thr[pos] = t.thr[q_lo + i]; }
      }
    }
  }
}

struct MaskJoinArgs {
  int64_t n;
  int32_t K, l, words;
  const u64* M[LQ_MAX_DIMS];
  const int32_t* fk[LQ_MAX_DIMS];
  int32_t* leaf;
  uint8_t* onehot;
  int32_t onehot_vec;       // whole 16-byte stores of one-hot rows are legal (l % 16 == 0, aligned)
  int32_t onehot_w4;        // 4-byte stores are (l % 4 == 0, rows start at multiples of 4 bytes)
  int32_t skip_when_lists;  // fused_tree_mask_kernel returns at once when the fact side has its per-leaf lists (the walk ran)
  FactSide f;
};

// The fact columns of R rows: in registers when there are at most eight of them (the node's column
// is then picked with selects, the column number being the same for every lane), else re-read per node.
constexpr int FACT_REG_COLS = 8;
typedef float v4f __attribute__((ext_vector_type(4)));
template <int R>
struct FactRows {
  v4f lo[R], hi[R];             // columns 0..3 and 4..7
  const float* ptr[R];
};
template <int R>
__device__ __forceinline__ void fact_rows_load(const FactSide& fs, const int64_t (&row)[R], FactRows<R>& fr) {
#pragma unroll
  for (int u = 0; u < R; ++u) {
    const float* p = fs.X + row[u] * fs.ldx;
    fr.ptr[u] = p;
    v4f lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    if (fs.c_f <= FACT_REG_COLS) {
      if (fs.vec_x) {
        lo = *reinterpret_cast<const v4f*>(p);
        if (fs.c_f > 4) hi = *reinterpret_cast<const v4f*>(p + 4);
      } else {
        lo.x = p[0];
        if (fs.c_f > 1) lo.y = p[1];
        if (fs.c_f > 2) lo.z = p[2];
        if (fs.c_f > 3) lo.w = p[3];
        if (fs.c_f > 4) hi.x = p[4];
        if (fs.c_f > 5) hi.y = p[5];
        if (fs.c_f > 6) hi.z = p[6];
        if (fs.c_f > 7) hi.w = p[7];
      }
    }
    fr.lo[u] = lo;
    fr.hi[u] = hi;
  }
}
// One fact-side node on R rows: m &= (x[f] > v) ? when_true : when_false.  f is the same for every
// lane, so the column is picked by a scalar branch rather than by selects.
template <int R>
__device__ __forceinline__ void fact_node_and(const FactSide& fs, const FactRows<R>& fr, int f, float v,
                                              u64 when_true, u64 when_false, u64 (&m)[R]) {
  auto run = [&](auto pick) {
#pragma unroll
    for (int u = 0; u < R; ++u) m[u] &= pick(u) > v ? when_true : when_false;
  };
  if (fs.c_f > FACT_REG_COLS) {
    run([&](int u) { return fr.ptr[u][f]; });
    return;
  }
  switch (f) {
    case 0: run([&](int u) { return fr.lo[u].x; }); break;
    case 1: run([&](int u) { return fr.lo[u].y; }); break;
    case 2: run([&](int u) { return fr.lo[u].z; }); break;
    case 3: run([&](int u) { return fr.lo[u].w; }); break;
    case 4: run([&](int u) { return fr.hi[u].x; }); break;
    case 5: run([&](int u) { return fr.hi[u].y; }); break;
    case 6: run([&](int u) { return fr.hi[u].z; }); break;
    default: run([&](int u) { return fr.hi[u].w; }); break;
  }
}
template <int R>
__device__ __forceinline__ void fact_masks_and(const FactSide& fs, const FactRows<R>& fr, int cnt, int words, int w, u64 (&m)[R]) {
  for (int q = 0; q < cnt; ++q) {
    const int f = __builtin_amdgcn_readfirstlane(fs.feat[q]);
    const float v = fs.thr[q];
    const int64_t o = (static_cast<int64_t>(q) * words + w) * 2;
    fact_node_and(fs, fr, f, v, fs.tf[o], fs.tf[o + 1], m);
  }
}

// Join stage on the masks.  A thread owns four fact rows (row = 256 wave + 64 u + lane, so that key
// loads and leaf stores are coalesced) and has all their gathers of one load step in flight at once.
// KT: number of dimensions when it is 1..4, 0 = any number.  WMAX: mask words kept per row for the
// cooperative one-hot store (trees of up to 64 WMAX leaves), 0 = no one-hot output or the plain store.
// WPL: mask words per load (2 = 16-byte loads, for an even number of words and 16-byte aligned masks).
template <int KT, int WMAX, int WPL>
__global__ __launch_bounds__(256) void fused_tree_mask_kernel(MaskJoinArgs a) {
  constexpr int KK = KT > 0 ? KT : LQ_MAX_DIMS, R = 4;
  typedef u64 wvec __attribute__((ext_vector_type(WPL)));
  const int lane = threadIdx.x & 63;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t row0 = wave * (64 * R);
  if (row0 >= a.n) return;
  if (a.skip_when_lists && a.f.cnt[1] != 0) return;
  int key[R][KK];
#pragma unroll
  for (int u = 0; u < R; ++u) {
    const int64_t row = min(row0 + 64 * u + lane, a.n - 1);
#pragma unroll
    for (int k = 0; k < KK; ++k) key[u][k] = (KT > 0 || k < a.K) ? a.fk[k][row] : 0;
  }
  FactRows<R> fr;
  int fact_nodes = 0;
  if (a.f.X) {
    int64_t rows[R];
#pragma unroll
    for (int u = 0; u < R; ++u) rows[u] = min(row0 + 64 * u + lane, a.n - 1);
    fact_rows_load(a.f, rows, fr);
    fact_nodes = *a.f.cnt;
  }
  int first[R];
  u64 kept[R][WMAX > 0 ? WMAX : 1];
#pragma unroll
  for (int u = 0; u < R; ++u) {
    first[u] = -1;
#pragma unroll
    for (int x = 0; x < (WMAX > 0 ? WMAX : 1); ++x) kept[u][x] = 0ull;
  }
  for (int w0 = 0; w0 < a.words; w0 += WPL) {
    wvec mv[R];
#pragma unroll
    for (int u = 0; u < R; ++u) {
#pragma unroll
      for (int e = 0; e < WPL; ++e) mv[u][e] = ~0ull;
#pragma unroll
      for (int k = 0; k < KK; ++k)
        if (KT > 0 || k < a.K) mv[u] &= *reinterpret_cast<const wvec*>(a.M[k] + static_cast<int64_t>(key[u][k]) * a.words + w0);
    }
#pragma unroll
    for (int e = 0; e < WPL; ++e) {
      const int w = w0 + e;
      if (fact_nodes > 0) {
        u64 mm[R];
#pragma unroll
        for (int u = 0; u < R; ++u) mm[u] = mv[u][e];
        fact_masks_and(a.f, fr, fact_nodes, a.words, w, mm);
#pragma unroll
        for (int u = 0; u < R; ++u) mv[u][e] = mm[u];
      }
#pragma unroll
      for (int u = 0; u < R; ++u) {
        const u64 m = (a.K == 0 && fact_nodes == 0) ? 0ull : mv[u][e];
        if (first[u] < 0 && m != 0ull) first[u] = 64 * w + __builtin_ctzll(m);
        if constexpr (WMAX > 0) {
#pragma unroll
          for (int x = 0; x < WMAX; ++x)
            if (x == w) kept[u][x] = m;
        } else if (a.onehot) {             // plain store: every thread writes the bytes of its own rows
          const int64_t row = row0 + 64 * u + lane;
          if (row < a.n)
            for (int b = 0; b < 64 && 64 * w + b < a.l; ++b) a.onehot[row * a.l + 64 * w + b] = (m >> b) & 1ull;
        }
      }
    }
    if (!a.onehot) {                     // leaf only: done once every row of the wavefront has its leaf
      bool done = true;
#pragma unroll
      for (int u = 0; u < R; ++u) done = done && first[u] >= 0;
      if (__all(done)) break;
    }
  }
  if (a.leaf) {
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int64_t row = row0 + 64 * u + lane;
      if (row < a.n) a.leaf[row] = first[u];
    }
  }
  if constexpr (WMAX > 0) {
    // one-hot rows, 16 bytes per lane: the C = l / 16 pieces of a row are written by neighbouring lanes
    const int C = a.l / 16;
#pragma unroll
    for (int u = 0; u < R; ++u) {
      for (int tpos = lane; tpos - lane < 64 * C; tpos += 64) {
        const int ri = tpos / C, piece = tpos - ri * C;          // row 0..63 of this group, 16-byte piece of its row
        u64 word = 0ull;
#pragma unroll
        for (int x = 0; x < WMAX; ++x) {
          const u64 other = __shfl(kept[u][x], ri, 64);
          if (x == piece / 4) word = other;
        }
        const int64_t row = row0 + 64 * u + ri;
        if (row < a.n) {
          const unsigned int bits = static_cast<unsigned int>(word >> (16 * (piece & 3))) & 0xffffu;
          v4u out;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const unsigned int b = (bits >> (4 * d)) & 0xfu;
            out[d] = (b & 1u) | ((b & 2u) << 7) | ((b & 4u) << 14) | ((b & 8u) << 21);
          }
          __builtin_nontemporal_store(out, reinterpret_cast<v4u*>(a.onehot + row * a.l + 16 * piece));
        }
      }
    }
  }
}

struct __attribute__((packed, aligned(4))) Words4At4 { unsigned int v[4]; };     // 16 bytes at a 4-byte boundary

// One-hot row of a fact row whose mask words are spread over the G lanes of a group (lane c: words 2c, 2c + 1), for l
// a multiple of 4 and rows aligned likewise (16-byte stores when both are multiples of 16).  The lanes hand their
// words to each other through LDS (`mine`: this wavefront's 64 x 16 bytes) so that a store instruction writes
// neighbouring 16-byte pieces of the row, eight instructions for its 128 G bytes.  Every lane of the wavefront calls it.
template <int G>
__device__ __forceinline__ void onehot_row_store(const MaskJoinArgs& a, u64* mine, int lane, int c, int64_t row, u64 w0, u64 w1) {
  typedef u64 u64x2 __attribute__((ext_vector_type(2)));
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");      // (the reads of the previous row are done)
  __builtin_amdgcn_wave_barrier();
  *reinterpret_cast<u64x2*>(mine + 2 * lane) = u64x2{w0, w1};
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // the row's mask now lies in LDS as the 16 G bytes of its lanes, in leaf order; piece P = 16 leaves = 2 of those bytes
  const unsigned short* bits16 = reinterpret_cast<const unsigned short*>(mine + 2 * (lane - c));
  const int pieces = (a.l + 15) >> 4;
  if (row >= a.n) return;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int P = i * G + c;
    if (P < pieces) {
      const unsigned int bits = bits16[P];
      v4u out;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const unsigned int b = (bits >> (4 * d)) & 0xfu;
        out[d] = (b & 1u) | ((b & 2u) << 7) | ((b & 4u) << 14) | ((b & 8u) << 21);
      }
      uint8_t* dst = a.onehot + row * a.l + 16 * P;
      if (a.onehot_vec) {
        *reinterpret_cast<v4u*>(dst) = out;
      } else if (16 * P + 16 <= a.l) {                    // rows that start at multiples of 4 bytes only
        *reinterpret_cast<Words4At4*>(dst) = Words4At4{{out[0], out[1], out[2], out[3]}};
      } else {                                            // the row's last, partial piece
#pragma unroll
        for (int d = 0; d < 4; ++d)
          if (16 * P + 4 * d < a.l) *reinterpret_cast<unsigned int*>(dst + 4 * d) = out[d];
      }
    }
  }
}

// Join for trees of more than 192 leaves (an even number of mask words, no fact-side nodes).
// A mask row of `words` words is contiguous (128 bytes for 1,024 leaves), so G = words / 2 lanes
// (rounded up to a power of two) read it as neighbouring 16-byte pieces: one load instruction then
// touches 64 / G rows of a table as whole runs instead of 64 unrelated pieces, which is what the
// address path of the vector memory unit is bound by in the kernel above.  A wavefront owns 64
// consecutive fact rows: their keys are read once, coalesced (lane = row), and handed to the lane
// groups through the cross-lane network; in pass t group g works on row (64 / G) t + g.  Each lane
// ANDs its two words over the tables, finds its lowest set bit, and a minimum over the group gives
// the leaf.  The gathers of four passes are requested before the first is consumed.
// OH: one-hot rows as well.
//   1  (l a multiple of 4, rows aligned likewise) through onehot_row_store, neighbouring 16-byte pieces of a row per
//      store instruction: 0.50 ms per 2.4e6 rows at 1,024 leaves (4.9 TB/s written); when every lane wrote the 128 bytes
//      of its own two words a line took eight instructions to fill: 1.04 ms
//   2  (any l) the rows were cleared beforehand and a lane sets the byte of each leaf reached, one per row for a tree:
//      0.80 ms at 1,024 leaves
template <int KT, int G, int OH>       // dimensions (1..4, 0 = any number); lanes per fact row (2..64)
__global__ __launch_bounds__(256) void fused_tree_mask_rows_kernel(MaskJoinArgs a) {
  constexpr int KK = KT > 0 ? KT : LQ_MAX_DIMS;
  constexpr int RPP = 64 / G;                 // rows per pass
  constexpr int PB = G < 4 ? G : 4;           // passes in flight together (G passes cover the 64 rows)
  typedef u64 u64x2 __attribute__((ext_vector_type(2)));
  __shared__ __align__(16) u64 swap[OH == 1 ? 4 * 64 * 2 : 2];     // per wavefront: the 16 bytes of every lane
  const int lane = threadIdx.x & 63, g = lane / G, c = lane % G;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t row0 = wave * 64;
  if (row0 >= a.n) return;
  int key[KK];
#pragma unroll
  for (int k = 0; k < KK; ++k) key[k] = (KT > 0 || k < a.K) ? a.fk[k][min(row0 + lane, a.n - 1)] : 0;
  const bool piece = 2 * c < a.words;         // (lanes past the last pair of words of a row stay idle)
  for (int t0 = 0; t0 < G; t0 += PB) {
    u64x2 m[PB];
#pragma unroll
    for (int e = 0; e < PB; ++e) {
      m[e] = u64x2{~0ull, ~0ull};
      const int src = (t0 + e) * RPP + g;     // the lane that holds this row's keys
#pragma unroll
      for (int k = 0; k < KK; ++k)
        if (KT > 0 || k < a.K) {
          const int j = __shfl(key[k], src, 64);
          if (piece) m[e] &= *reinterpret_cast<const u64x2*>(a.M[k] + static_cast<int64_t>(j) * a.words + 2 * c);
        }
    }
#pragma unroll
    for (int e = 0; e < PB; ++e) {
      int pos = 0x7fffffff;
      if (piece && a.K > 0) {
        if (m[e][0] != 0ull) pos = 128 * c + __builtin_ctzll(m[e][0]);
        else if (m[e][1] != 0ull) pos = 128 * c + 64 + __builtin_ctzll(m[e][1]);
      }
#pragma unroll
      for (int d = 1; d < G; d <<= 1) pos = min(pos, __shfl_xor(pos, d, 64));
      const int64_t row = row0 + (t0 + e) * RPP + g;
      if (a.leaf && c == 0 && row < a.n) a.leaf[row] = pos == 0x7fffffff ? -1 : pos;
      if constexpr (OH == 2) {
        if (piece && row < a.n && a.K > 0)
#pragma unroll
          for (int half = 0; half < 2; ++half)
            for (u64 w = m[e][half]; w != 0ull; w &= w - 1ull) a.onehot[row * a.l + 128 * c + 64 * half + __builtin_ctzll(w)] = 1;
      }
      if constexpr (OH == 1)
        onehot_row_store<G>(a, swap + (threadIdx.x >> 6) * 128, lane, c, row, (piece && a.K > 0) ? m[e][0] : 0ull,
                            (piece && a.K > 0) ? m[e][1] : 0ull);
    }
  }
}

// The same with nodes on fact-table columns (any number of dimensions), for trees whose per-leaf lists
// of such nodes did not fit (the call returns at once when they are there: the walk kernel below
// serves those).  A lane applies every such node to its two words of the row: the node's test is
// evaluated on the fact row of the lane's group, and the mask pair that applies is ANDed in.  The
// pairs of the first nodes sit in LDS (32 KB: 128 nodes at 1,024 leaves), those of further nodes are
// read from memory.  One-hot rows are cleared beforehand; a byte is set per leaf reached.
constexpr int ROWS_FACT_LDS = 32 * 1024;
template <int G>
__global__ __launch_bounds__(256) void fused_tree_mask_rows_fact_kernel(MaskJoinArgs a) {
  constexpr int KK = LQ_MAX_DIMS;
  constexpr int RPP = 64 / G;
  constexpr int PB = G < 4 ? G : 4;
  typedef u64 u64x2 __attribute__((ext_vector_type(2)));
  __shared__ __align__(16) u64 tf_lds[ROWS_FACT_LDS / 8];
  __shared__ u64 ft_lds[ROWS_FACT_LDS / 64];      // column and threshold of the nodes in LDS (at least 4 words per row)
  __shared__ __align__(16) u64 swap[4 * 64 * 2];  // per wavefront: the 16 bytes of every lane (onehot_row_store)
  if (a.f.cnt[1] != 0) return;                   // per-leaf lists of fact-side nodes are there
  const int fact_nodes = *a.f.cnt;
  const bool every = a.onehot != nullptr;
  const bool rows_whole = a.onehot_vec || a.onehot_w4;
  const int in_lds = min(fact_nodes, ROWS_FACT_LDS / (16 * a.words));
  for (int i = threadIdx.x; i < in_lds * a.words * 2; i += 256) tf_lds[i] = a.f.tf[i];
  for (int i = threadIdx.x; i < in_lds; i += 256)
    ft_lds[i] = static_cast<u64>(static_cast<unsigned int>(a.f.feat[i])) | (static_cast<u64>(__float_as_uint(a.f.thr[i])) << 32);
  __syncthreads();
  const int lane = threadIdx.x & 63, g = lane / G, c = lane % G;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t row0 = wave * 64;
  if (row0 >= a.n) return;
  int key[KK];
#pragma unroll
  for (int k = 0; k < KK; ++k) key[k] = k < a.K ? a.fk[k][min(row0 + lane, a.n - 1)] : 0;
  const bool piece = 2 * c < a.words;
  const int wc = piece ? 2 * c : 0;           // (idle lanes follow along on the first words and store nothing)
  for (int t0 = 0; t0 < G; t0 += PB) {
    u64 m0[PB], m1[PB];
    FactRows<PB> fr;
    int64_t rows[PB];
#pragma unroll
    for (int e = 0; e < PB; ++e) rows[e] = min(row0 + (t0 + e) * RPP + g, a.n - 1);
    fact_rows_load(a.f, rows, fr);
#pragma unroll
    for (int e = 0; e < PB; ++e) {
      u64x2 m = u64x2{~0ull, ~0ull};
      const int src = (t0 + e) * RPP + g;
#pragma unroll
      for (int k = 0; k < KK; ++k)
        if (k < a.K) {
          const int j = __shfl(key[k], src, 64);
          m &= *reinterpret_cast<const u64x2*>(a.M[k] + static_cast<int64_t>(j) * a.words + wc);
        }
      m0[e] = m[0]; m1[e] = m[1];
    }
    // (the data of node q + 1 is requested before node q is applied)
    auto node = [&](int q, u64& ft, u64x2& p0, u64x2& p1) {      // {test true, test false} for this lane's two words
      if (q < in_lds) {
        ft = ft_lds[q];
        const u64x2* src = reinterpret_cast<const u64x2*>(tf_lds) + q * a.words + wc;
        p0 = src[0]; p1 = src[1];
      } else {
        ft = static_cast<u64>(static_cast<unsigned int>(a.f.feat[q])) | (static_cast<u64>(__float_as_uint(a.f.thr[q])) << 32);
        const u64x2* src = reinterpret_cast<const u64x2*>(a.f.tf) + static_cast<int64_t>(q) * a.words + wc;
        p0 = src[0]; p1 = src[1];
      }
    };
    u64 ft = 0ull, nft = 0ull;
    u64x2 p0 = {0ull, 0ull}, p1 = {0ull, 0ull}, np0 = {0ull, 0ull}, np1 = {0ull, 0ull};
    if (fact_nodes > 0) node(0, ft, p0, p1);
    for (int q = 0; q < fact_nodes; ++q) {
      if (q + 1 < fact_nodes) node(q + 1, nft, np0, np1);
      const int f = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned int>(ft)));
      const float v = __uint_as_float(static_cast<unsigned int>(ft >> 32));
      fact_node_and(a.f, fr, f, v, p0[0], p0[1], m0);
      fact_node_and(a.f, fr, f, v, p1[0], p1[1], m1);
      ft = nft; p0 = np0; p1 = np1;
    }
#pragma unroll
    for (int e = 0; e < PB; ++e) {
      int pos = 0x7fffffff;
      const int64_t row = row0 + (t0 + e) * RPP + g;
      if (piece && (a.K > 0 || fact_nodes > 0)) {
        if (m0[e] != 0ull) pos = 128 * c + __builtin_ctzll(m0[e]);
        else if (m1[e] != 0ull) pos = 128 * c + 64 + __builtin_ctzll(m1[e]);
        if (every && !rows_whole && row < a.n)
#pragma unroll
          for (int half = 0; half < 2; ++half)
            for (u64 m = half ? m1[e] : m0[e]; m != 0ull; m &= m - 1ull) {
              const int j = 128 * c + 64 * half + __builtin_ctzll(m);
              if (j < a.l) a.onehot[row * a.l + j] = 1;
            }
      }
#pragma unroll
      for (int d = 1; d < G; d <<= 1) pos = min(pos, __shfl_xor(pos, d, 64));
      if (c == 0 && row < a.n && a.leaf) a.leaf[row] = pos == 0x7fffffff ? -1 : pos;
      if (every && rows_whole) {
        const bool any = piece && (a.K > 0 || fact_nodes > 0);
        onehot_row_store<G>(a, swap + (threadIdx.x >> 6) * 128, lane, c, row, any ? m0[e] : 0ull, any ? m1[e] : 0ull);
      }
    }
  }
}

// The same from the per-leaf lists of fact-side nodes (the call returns at once when they are not there).
// The tables have left few leaves possible.  The G lanes of a row take its lowest leaf still possible and
// check it against the fact-side nodes on its own path; the first test that comes out the other way takes
// that leaf out, and with it every leaf that wants the same outcome of that node (one AND with the node's
// mask row: in a tree, the subtree on that side), so a row needs about as many rounds as its path has
// fact-side nodes instead of one AND per fact-side node and mask word.  For the leaf number the walk stops
// at the first leaf that passes; for one-hot rows (cleared beforehand) it sets that leaf's byte and goes on:
// H need not be a tree.  A lane's four rows go through their rounds together, so that the loads of a round
// (list bounds, list entries, fact value, mask row: each waits for the one before) are in flight for all four.
constexpr int WALK_ROWS = 1;        // rows of a lane that go through their rounds together
// WPL: mask words per lane (1: trees of up to 64 leaves, one lane per row, G = 1).
// OH: 0 = leaf numbers only, 1 = one-hot rows written whole at the end (onehot_row_store), 2 = byte by byte.
template <int G, int WPL, int OH>
__global__ __launch_bounds__(256) void fused_tree_mask_rows_walk_kernel(MaskJoinArgs a) {
  constexpr int KK = LQ_MAX_DIMS;
  constexpr int RPP = 64 / G;
  constexpr int PB = G < WALK_ROWS ? G : WALK_ROWS;
  constexpr int NONE = 0x7fffffff;
  typedef u64 u64x2 __attribute__((ext_vector_type(2)));
  __shared__ __align__(16) u64 swap[OH == 1 ? 4 * 64 * 2 : 2];   // per wavefront: the 16 bytes of every lane (onehot_row_store)
  if (a.f.cnt[1] == 0) return;
  constexpr bool every = OH != 0;
  constexpr bool rows_whole = OH == 1;
  const int lane = threadIdx.x & 63, g = lane / G, c = lane % G;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t row0 = wave * 64;
  if (row0 >= a.n) return;
  int key[KK];
#pragma unroll
  for (int k = 0; k < KK; ++k) key[k] = k < a.K ? a.fk[k][min(row0 + lane, a.n - 1)] : 0;
  static_assert(WPL == 2 || G == 1, "one word per lane: one lane per row");
  const bool piece = WPL * c < a.words;
  const int wc = piece ? WPL * c : 0;         // (idle lanes follow along on the first words and store nothing)
  for (int t0 = 0; t0 < G; t0 += PB) {
    u64 w0[PB], w1[PB];
    const float* xr[PB];
    int64_t row[PB];                           // (the same for the G lanes of a row, and so is all control flow below)
    bool open[PB];
    int found[PB];
    u64 r0[rows_whole ? PB : 1], r1[rows_whole ? PB : 1];      // leaves reached (one-hot rows written whole)
#pragma unroll
    for (int e = 0; e < PB; ++e) {
      if constexpr (rows_whole) { r0[e] = 0ull; r1[e] = 0ull; }
      row[e] = row0 + (t0 + e) * RPP + g;
      xr[e] = a.f.X + min(row[e], a.n - 1) * a.f.ldx;
      u64x2 m = u64x2{~0ull, WPL == 2 ? ~0ull : 0ull};
      const int src = (t0 + e) * RPP + g;
#pragma unroll
      for (int k = 0; k < KK; ++k)
        if (k < a.K) {
          const int j = __shfl(key[k], src, 64);
          if constexpr (WPL == 2) m &= *reinterpret_cast<const u64x2*>(a.M[k] + static_cast<int64_t>(j) * a.words + wc);
          else m[0] &= a.M[k][static_cast<int64_t>(j) * a.words + wc];
        }
      const bool live = piece && row[e] < a.n;
      w0[e] = live ? m[0] : 0ull; w1[e] = live ? m[1] : 0ull;
      open[e] = true; found[e] = NONE;
    }
    for (;;) {
      int j[PB], i[PB], end[PB], bad[PB];
      bool outcome[PB];
      bool any = false;
#pragma unroll
      for (int e = 0; e < PB; ++e) {
        int lo = w0[e] != 0ull ? 128 * c + __builtin_ctzll(w0[e]) : (w1[e] != 0ull ? 128 * c + 64 + __builtin_ctzll(w1[e]) : NONE);
#pragma unroll
        for (int d = 1; d < G; d <<= 1) lo = min(lo, __shfl_xor(lo, d, 64));
        j[e] = lo;
        open[e] = open[e] && lo < a.l;          // none left (without tables the bits past the last leaf are still set)
        any = any || open[e];
      }
      if (!any) break;
#pragma unroll
      for (int e = 0; e < PB; ++e) {
        i[e] = open[e] ? a.f.leaf_off[j[e]] : 0;
        end[e] = open[e] ? a.f.leaf_off[j[e] + 1] : 0;
        bad[e] = -1; outcome[e] = false;
      }
      for (;;) {                                 // the lists of the four leaves, entry by entry
        uint4 en[PB];
        bool scan[PB], more = false;
#pragma unroll
        for (int e = 0; e < PB; ++e) {
          scan[e] = bad[e] < 0 && i[e] < end[e];
          if (scan[e]) en[e] = a.f.leaf_ent[i[e]];
          more = more || scan[e];
        }
        if (!more) break;
        float x[PB];
#pragma unroll
        for (int e = 0; e < PB; ++e) x[e] = scan[e] ? xr[e][en[e].x] : 0.0f;
#pragma unroll
        for (int e = 0; e < PB; ++e)
          if (scan[e]) {
            const bool test = x[e] > __uint_as_float(en[e].z);
            if (test == (en[e].y != 0u)) { bad[e] = static_cast<int>(en[e].w); outcome[e] = test; }
            ++i[e];
          }
      }
      u64x2 p0[PB], p1[PB];                      // {test true, test false} of this lane's two words
#pragma unroll
      for (int e = 0; e < PB; ++e)
        if (open[e] && bad[e] >= 0) {
          const u64x2* src = reinterpret_cast<const u64x2*>(a.f.tf) + static_cast<int64_t>(bad[e]) * a.words + wc;
          p0[e] = src[0];
          if constexpr (WPL == 2) p1[e] = src[1]; else p1[e] = u64x2{0ull, 0ull};
        }
#pragma unroll
      for (int e = 0; e < PB; ++e) {
        if (!open[e]) continue;
        if (bad[e] >= 0) {
          w0[e] &= outcome[e] ? p0[e][0] : p0[e][1];
          w1[e] &= outcome[e] ? p1[e][0] : p1[e][1];
        } else {
          if (found[e] == NONE) found[e] = j[e];
          if (!every) open[e] = false;
          else if (c == (j[e] >> 7)) {
            const u64 bit = 1ull << (j[e] & 63);
            if constexpr (!rows_whole) a.onehot[row[e] * a.l + j[e]] = 1;
            if (j[e] & 64) w1[e] &= ~bit; else w0[e] &= ~bit;
            if constexpr (rows_whole) { if (j[e] & 64) r1[e] |= bit; else r0[e] |= bit; }
          }
        }
      }
    }
#pragma unroll
    for (int e = 0; e < PB; ++e) {
      if (c == 0 && row[e] < a.n && a.leaf) a.leaf[row[e]] = found[e] == NONE ? -1 : found[e];
      if constexpr (rows_whole) onehot_row_store<G>(a, swap + (threadIdx.x >> 6) * 128, lane, c, row[e], r0[e], r1[e]);
    }
  }
}

// Clears `bytes` bytes from p on (any alignment): 16-byte stores between the first and the last 16-byte boundary.
__global__ __launch_bounds__(256) void zero_bytes_kernel(uint8_t* __restrict__ p, int64_t bytes) {
  typedef unsigned int v4u __attribute__((ext_vector_type(4)));
  const int64_t head = min(bytes, static_cast<int64_t>((16 - (reinterpret_cast<uintptr_t>(p) & 15)) & 15));
  const int64_t pieces = (bytes - head) / 16;
  const int64_t tail = bytes - head - 16 * pieces;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < pieces; i += stride)
    *reinterpret_cast<v4u*>(p + head + 16 * i) = v4u{0u, 0u, 0u, 0u};
  if (blockIdx.x == 0 && threadIdx.x < head) p[threadIdx.x] = 0;
  if (blockIdx.x == 0 && threadIdx.x < tail) p[head + 16 * pieces + threadIdx.x] = 0;
}

// The same join for trees of up to 64 leaves (one mask word) and leaf-only output, with the mask
// tables that fit kept in LDS: one persistent workgroup per compute unit stages them once, then its
// threads stride over the fact rows, four rows each per step.  Gathers from LDS do not go through the
// address path of the vector memory unit, which is what bounds the kernel above.
struct MaskLds {
  int32_t off[LQ_MAX_DIMS];     // position of the table in LDS in words, -1 = stays in memory
  int32_t rows[LQ_MAX_DIMS];
  int32_t vec;                  // key columns and leaf are 16-byte aligned: four rows per load / store
  int32_t fact_off;             // position of the fact-side nodes in LDS in words (three words per node)
};
constexpr int MLDS_THREADS = 1024;
constexpr int FACT_LDS_NODES = 128;    // fact-side nodes kept in LDS; further ones are read from memory per step
template <int KT, bool FACT>       // KT: number of dimensions, 1..4; FACT: the fact table has columns
__global__ __launch_bounds__(MLDS_THREADS) void fused_tree_mask_lds_kernel(MaskJoinArgs a, MaskLds L) {
  constexpr int KK = KT, R = 4;
  typedef u64 u64x2 __attribute__((ext_vector_type(2)));
  extern __shared__ __align__(16) u64 tab[];
  const int tid = threadIdx.x;
  // stage: 16 bytes per thread and load, four loads requested before the first is stored
  for (int k = 0; k < KK; ++k)
    if ((KT > 0 || k < a.K) && L.off[k] >= 0) {
      const int pairs = L.rows[k] / 2, half_off = L.off[k] / 2;      // (table offsets in LDS are even)
      const u64x2* src = reinterpret_cast<const u64x2*>(a.M[k]);
      for (int i0 = tid; i0 < pairs; i0 += 4 * MLDS_THREADS) {
        u64x2 v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i0 + e * MLDS_THREADS < pairs) v[e] = src[i0 + e * MLDS_THREADS];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (i0 + e * MLDS_THREADS < pairs) {
            tab[2 * (half_off + i0 + e * MLDS_THREADS)] = v[e][0];
            tab[2 * (half_off + i0 + e * MLDS_THREADS) + 1] = v[e][1];
          }
      }
      if (tid == 0 && (L.rows[k] & 1)) tab[L.off[k] + L.rows[k] - 1] = a.M[k][L.rows[k] - 1];
    }
  int fact_nodes = 0;
  if constexpr (FACT) {
    fact_nodes = *a.f.cnt;
    if (tid < min(fact_nodes, FACT_LDS_NODES)) {
      tab[L.fact_off + 3 * tid] = static_cast<u64>(static_cast<unsigned int>(a.f.feat[tid])) |
                                  (static_cast<u64>(__float_as_uint(a.f.thr[tid])) << 32);
      tab[L.fact_off + 3 * tid + 1] = a.f.tf[2 * tid];
      tab[L.fact_off + 3 * tid + 2] = a.f.tf[2 * tid + 1];
    }
  }
  __syncthreads();
  // Without fact columns every thread takes four consecutive fact rows per step: one 16-byte load per
  // key column, one 16-byte store of the four leaves (plain loads: streaming hints made this kernel
  // slower).  With fact columns its rows are 64 apart (row = 256 wavefront + 64 u + lane), so that the
  // lanes of a wavefront read neighbouring rows of X and every cache line of X is fetched once.
  typedef int v4i __attribute__((ext_vector_type(4)));
  constexpr int RS = FACT ? 64 : 1;                                   // distance between a thread's rows
  const int64_t step = static_cast<int64_t>(gridDim.x) * MLDS_THREADS * R;
  const int in_block = FACT ? 256 * (tid >> 6) + (tid & 63) : R * tid;
  int64_t base = static_cast<int64_t>(blockIdx.x) * MLDS_THREADS * R + in_block;
  if (base - in_block >= a.n) return;
  v4i key[KK];
  auto load_keys = [&](int64_t b, v4i (&out)[KK]) {
#pragma unroll
    for (int k = 0; k < KK; ++k) {
      out[k] = v4i{0, 0, 0, 0};
      if (KT > 0 || k < a.K) {
        if (!FACT && L.vec && b + R <= a.n) out[k] = *reinterpret_cast<const v4i*>(a.fk[k] + b);
        else {
#pragma unroll
          for (int u = 0; u < R; ++u) out[k][u] = a.fk[k][min(b + RS * u, a.n - 1)];
        }
      }
    }
  };
  load_keys(min(base, a.n - 1), key);
  for (;;) {
    const int64_t nbase = base + step;
    const bool more = nbase - in_block < a.n;            // (uniform over the workgroup)
    v4i nkey[KK];
    load_keys(min(more ? nbase : base, a.n - 1), nkey);   // keys of the next step are in flight during this one
    FactRows<R> fr;
    if (FACT && fact_nodes > 0) {                         // requested before the mask gathers, used after them
      int64_t rows[R];
#pragma unroll
      for (int u = 0; u < R; ++u) rows[u] = min(base + RS * u, a.n - 1);
      fact_rows_load(a.f, rows, fr);
    }
    u64 m[R];
#pragma unroll
    for (int u = 0; u < R; ++u) m[u] = ~0ull;
#pragma unroll
    for (int k = 0; k < KK; ++k)
      if (KT > 0 || k < a.K) {
        if (L.off[k] >= 0) {                       // (uniform: a table is in LDS for every row or for none)
#pragma unroll
          for (int u = 0; u < R; ++u) m[u] &= tab[L.off[k] + key[k][u]];
        } else {
          const u64* __restrict__ g = a.M[k];
#pragma unroll
          for (int u = 0; u < R; ++u) m[u] &= g[key[k][u]];
        }
      }
    if constexpr (FACT) {
      for (int q = 0; q < fact_nodes; ++q) {
        u64 ft, when_true, when_false;
        if (q < FACT_LDS_NODES) {
          ft = tab[L.fact_off + 3 * q]; when_true = tab[L.fact_off + 3 * q + 1]; when_false = tab[L.fact_off + 3 * q + 2];
        } else {
          ft = static_cast<u64>(static_cast<unsigned int>(a.f.feat[q])) | (static_cast<u64>(__float_as_uint(a.f.thr[q])) << 32);
          when_true = a.f.tf[2 * q]; when_false = a.f.tf[2 * q + 1];
        }
        const int f = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned int>(ft)));
        const float v = __uint_as_float(static_cast<unsigned int>(ft >> 32));
        fact_node_and(a.f, fr, f, v, when_true, when_false, m);
      }
    }
    v4i lf;
#pragma unroll
    for (int u = 0; u < R; ++u) lf[u] = m[u] != 0ull ? __builtin_ctzll(m[u]) : -1;
    if (!FACT && L.vec && base + R <= a.n) *reinterpret_cast<v4i*>(a.leaf + base) = lf;
    else {
#pragma unroll
      for (int u = 0; u < R; ++u)
        if (base + RS * u < a.n) a.leaf[base + RS * u] = lf[u];
    }
    if (!more) break;
    base = nbase;
    for (int k = 0; k < KK; ++k) key[k] = nkey[k];
  }
}

// LQ_CHECK_FKS for the tree calls: synchronous range check of the key columns against the row counts
// in star->dims; `flag` is a device word inside the caller's workspace.
int tree_check_fks(const lq_star* star, void* flag, size_t flag_bytes, hipStream_t s) {
  if (star->n_dims == 0 || star->n_fact == 0) return LQ_OK;
  if (!star->dims) return fail(LQ_ERR_NULL, "LQ_CHECK_FKS needs star->dims for the row counts");
  if (!flag || flag_bytes < 256 || !aligned(flag, 256))
    return fail(LQ_ERR_WORKSPACE, "LQ_CHECK_FKS needs a 256-byte aligned workspace of >= 256 bytes");
  int64_t rows[LQ_MAX_DIMS];
  for (int k = 0; k < star->n_dims; ++k) {
    if (!star->fks || !star->fks[k] || !aligned(star->fks[k], 4)) return fail(LQ_ERR_NULL, "fks[%d] is NULL or misaligned", k);
    rows[k] = star->dims[k].rows;
  }
  int rc = launch_check_fks(star->n_fact, star->n_dims, star->fks, rows, false, static_cast<int32_t*>(flag), s);
  if (rc) return rc;
  int32_t h = 0;
  LQ_HIP_TRY(hipMemcpyAsync(&h, flag, sizeof(h), hipMemcpyDeviceToHost, s));
  LQ_HIP_TRY(hipStreamSynchronize(s));
  if (h) return fail(LQ_ERR_FK_RANGE, "a foreign key lies outside its dimension table");
  return LQ_OK;
}

int check_tree(const lq_tree* tree, TreeArgs* t) {
  if (!tree) return fail(LQ_ERR_NULL, "tree is NULL");
  if (tree->n_nodes < 1 || tree->n_leaves < 1) return fail(LQ_ERR_SHAPE, "tree needs nodes and leaves");
  if (tree->n_leaves > 16384) return fail(LQ_ERR_UNSUPPORTED, "more than 16384 leaves");
  if (!tree->feature || !tree->threshold || !tree->H) return fail(LQ_ERR_NULL, "tree arrays are NULL");
  if (!aligned(tree->feature, 4) || !aligned(tree->threshold, 4))
    return fail(LQ_ERR_SHAPE, "tree arrays are misaligned");
  t->p = tree->n_nodes; t->l = tree->n_leaves;
  t->ld = static_cast<int64_t>(round_up(static_cast<size_t>(tree->n_leaves), 16));
  t->feature = tree->feature; t->thr = tree->threshold; t->H = tree->H;
  return LQ_OK;
}

int check_star_basic(const lq_star* star, bool need_dims) {
  if (!star) return fail(LQ_ERR_NULL, "star is NULL");
  if (star->n_fact < 0) return fail(LQ_ERR_SHAPE, "n_fact < 0");
  if (star->n_dims < 0 || star->n_dims > LQ_MAX_DIMS) return fail(LQ_ERR_SHAPE, "n_dims outside 0..%d", LQ_MAX_DIMS);
  if (star->fact.cols < 0) return fail(LQ_ERR_SHAPE, "fact.cols < 0");
  if (star->fact.cols > 0 && star->fact.dtype != LQ_F32) return fail(LQ_ERR_DTYPE, "tree paths take f32 tables");
  if (need_dims) {
    if (star->n_dims > 0 && !star->dims) return fail(LQ_ERR_NULL, "star->dims is NULL");
    for (int k = 0; k < star->n_dims; ++k) {
      const lq_mat& d = star->dims[k];
      if (d.dtype != LQ_F32) return fail(LQ_ERR_DTYPE, "tree paths take f32 tables");
      if (d.rows < 1 || d.cols < 1 || d.ld < d.cols || !d.data || !aligned(d.data, 4))
        return fail(LQ_ERR_SHAPE, "dims[%d] is malformed", k);
    }
  }
  return LQ_OK;
}

// Rows of one dimension table (all of them, or the slice an incremental refresh touches) with the
// place of their pre-fused rows.
struct DimSlice {
  const float* D; int64_t ldd, rows;
  int32_t col_off, cols;
  uint8_t* out;
};

int project_slices(const TreeArgs& t, const DimSlice* sl, int n, hipStream_t s) {
  if (n == 0) return LQ_OK;
  if (t.p <= 256) {
    // every wavefront builds the node masks of its 64 leaves once (p loads): give it at least p / 8
    // rows to spread that over
    ProjectArgs pa{};
    int64_t max_rows = 0;
    for (int k = 0; k < n; ++k) {
      pa.D[k] = sl[k].D; pa.out[k] = sl[k].out; pa.ldd[k] = sl[k].ldd; pa.rows[k] = sl[k].rows;
      pa.col_off[k] = sl[k].col_off; pa.cols[k] = sl[k].cols;
      max_rows = std::max<int64_t>(max_rows, sl[k].rows);
    }
    const int64_t rows_per_block = 4 * std::max<int64_t>(4, t.p / 8);
    const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>((max_rows + rows_per_block - 1) / rows_per_block,
                                                                  static_cast<int64_t>(num_cus()) * 8));
    const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>((t.ld + 63) / 64), static_cast<unsigned>(n)), block(256);
    if (t.p <= 64) hipLaunchKernelGGL(tree_project_bits_kernel<1>, grid, block, 0, s, t, pa);
    else if (t.p <= 128) hipLaunchKernelGGL(tree_project_bits_kernel<2>, grid, block, 0, s, t, pa);
    else hipLaunchKernelGGL(tree_project_bits_kernel<4>, grid, block, 0, s, t, pa);
    LQ_LAUNCH_CHECK("tree_project_bits_kernel");
    return LQ_OK;
  }
  for (int k = 0; k < n; ++k) {
    const DimSlice& d = sl[k];
    if (d.rows == 0) continue;
    if (t.p <= 0x7fff) {   // beyond 4 mask words per leaf the per-leaf node lists are as fast or faster (measured up to 16 words)
      const int64_t col_tiles = (t.ld + TP_COLS - 1) / TP_COLS;
      // enough row slices to fill the GPU, each long enough to amortise building the lists
      int64_t slices = std::max<int64_t>(1, std::min<int64_t>((static_cast<int64_t>(num_cus()) * 2 + col_tiles - 1) / col_tiles,
                                                              (d.rows + 255) / 256));
      slices = std::min<int64_t>(slices, 65535);
      const int64_t rpb = (d.rows + slices - 1) / slices;
      hipLaunchKernelGGL(tree_project_sparse_kernel, dim3(static_cast<unsigned>(col_tiles), static_cast<unsigned>(slices)),
                         dim3(TPS_THREADS), 0, s, t, d.D, d.ldd, d.rows, d.col_off, d.cols, d.out, rpb,
                         static_cast<int32_t>(col_tiles));
      LQ_LAUNCH_CHECK("tree_project_sparse_kernel");
    } else {
      const int64_t total = d.rows * t.ld;
      const int64_t blocks = std::min<int64_t>((total + 255) / 256, static_cast<int64_t>(num_cus()) * 32);
      hipLaunchKernelGGL(tree_project_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, t,
                         d.D, d.ldd, d.rows, d.col_off, d.cols, d.out);
      LQ_LAUNCH_CHECK("tree_project_kernel");
    }
  }
  return LQ_OK;
}

// Mask rows of the table rows in sl[k].out (sl[k].D is not read).
int compress_slices(const TreeArgs& t, const DimSlice* sl, u64* const* masks, int n, hipStream_t s) {
  if (n == 0) return LQ_OK;
  const int32_t words = static_cast<int32_t>(lq_tree_mask_words(t.l));
  CompressArgs ca{};
  int64_t max_rows = 0;
  for (int k = 0; k < n; ++k) {
    ca.table[k] = sl[k].out; ca.masks[k] = masks[k];
    ca.rows[k] = sl[k].rows; ca.col_off[k] = sl[k].col_off; ca.cols[k] = sl[k].cols;
    max_rows = std::max<int64_t>(max_rows, sl[k].rows);
  }
  const int64_t blocks = (max_rows + CMP_THREADS - 1) / CMP_THREADS;
  if (blocks < 1) return LQ_OK;
  if (blocks > 0x7fffffffLL || words > 65535) return fail(LQ_ERR_UNSUPPORTED, "too many rows or leaves for one launch");
  hipLaunchKernelGGL(tree_compress_kernel, dim3(static_cast<unsigned>(blocks), static_cast<unsigned>(words),
                                                static_cast<unsigned>(n)), dim3(CMP_THREADS), 0, s, t, ca, words);
  LQ_LAUNCH_CHECK("tree_compress_kernel");
  return LQ_OK;
}

}  // namespace
}  // namespace lq

using namespace lq;

extern "C" {

int64_t lq_tree_table_ld(int32_t n_leaves) {
  return n_leaves < 1 ? 0 : static_cast<int64_t>(round_up(static_cast<size_t>(n_leaves), 16));
}

int lq_tree_project_dims(const lq_star* star, const lq_tree* tree, void* const* tables, uint8_t* target,
                         void* hip_stream) {
  clear_error();
  TreeArgs t{};
  int rc = check_star_basic(star, true);
  if (rc) return rc;
  if ((rc = check_tree(tree, &t))) return rc;
  if (!target) return fail(LQ_ERR_NULL, "target is NULL");
  if (star->n_dims > 0 && !tables) return fail(LQ_ERR_NULL, "tables is NULL");
  for (int k = 0; k < star->n_dims; ++k)
    if (!tables[k] || !aligned(tables[k], 16)) return fail(LQ_ERR_NULL, "tables[%d] is NULL or not 16-byte aligned", k);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(tree_target_kernel, dim3(static_cast<unsigned>((t.ld + 63) / 64)), dim3(TT_THREADS), 0, s, t, target);
  LQ_LAUNCH_CHECK("tree_target_kernel");
  DimSlice sl[LQ_MAX_DIMS];
  int32_t off = star->fact.cols;
  for (int k = 0; k < star->n_dims; ++k) {
    const lq_mat& d = star->dims[k];
    sl[k] = DimSlice{static_cast<const float*>(d.data), d.ld, d.rows, off, d.cols, static_cast<uint8_t*>(tables[k])};
    off += d.cols;
  }
  return project_slices(t, sl, star->n_dims, s);
}

int lq_tree_project_dim_rows(const lq_star* star, const lq_tree* tree, void* const* tables, uint64_t* const* masks,
                             int32_t dim, int64_t first_row, int64_t n_rows, void* hip_stream) {
  clear_error();
  TreeArgs t{};
  int rc = check_star_basic(star, true);
  if (rc) return rc;
  if ((rc = check_tree(tree, &t))) return rc;
  if (dim < 0 || dim >= star->n_dims) return fail(LQ_ERR_SHAPE, "dim outside 0..%d", star->n_dims - 1);
  const lq_mat& d = star->dims[dim];
  if (first_row < 0 || n_rows < 0 || first_row > d.rows || n_rows > d.rows - first_row)
    return fail(LQ_ERR_SHAPE, "rows [%lld, +%lld) outside dims[%d]", static_cast<long long>(first_row),
                static_cast<long long>(n_rows), dim);
  if (!tables || !tables[dim] || !aligned(tables[dim], 16)) return fail(LQ_ERR_NULL, "tables[%d] is NULL or not 16-byte aligned", dim);
  if (masks && (!masks[dim] || !aligned(masks[dim], 8))) return fail(LQ_ERR_NULL, "masks[%d] is NULL or misaligned", dim);
  if (n_rows == 0) return LQ_OK;
  int32_t off = star->fact.cols;
  for (int k = 0; k < dim; ++k) off += star->dims[k].cols;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const DimSlice sl{static_cast<const float*>(d.data) + first_row * d.ld, d.ld, n_rows, off, d.cols,
                    static_cast<uint8_t*>(tables[dim]) + first_row * t.ld};
  if ((rc = project_slices(t, &sl, 1, s))) return rc;
  if (!masks) return LQ_OK;
  const int32_t words = static_cast<int32_t>(lq_tree_mask_words(t.l));
  u64* m = reinterpret_cast<u64*>(masks[dim]) + first_row * words;
  return compress_slices(t, &sl, &m, 1, s);
}

int lq_fused_join_tree(const lq_star* star, const lq_tree* tree, const void* const* tables,
                       const uint8_t* target, int32_t* leaf, uint8_t* onehot, uint32_t flags, void* ws,
                       size_t ws_bytes, void* hip_stream) {
  clear_error();
  FusedTreeArgs a{};
  int rc = check_star_basic(star, false);
  if (rc) return rc;
  if ((rc = check_tree(tree, &a.t))) return rc;
  if (!target || !aligned(target, 16)) return fail(LQ_ERR_NULL, "target is NULL or not 16-byte aligned");
  if (star->n_dims > 0 && (!tables || !star->fks)) return fail(LQ_ERR_NULL, "tables or fks is NULL");
  if (!leaf && !onehot) return fail(LQ_ERR_NULL, "neither leaf nor onehot requested");
  if (leaf && !aligned(leaf, 4)) return fail(LQ_ERR_SHAPE, "leaf is misaligned");
  a.n = star->n_fact; a.K = star->n_dims;
  for (int k = 0; k < a.K; ++k) {
    if (!tables[k] || !aligned(tables[k], 16)) return fail(LQ_ERR_NULL, "tables[%d] is NULL or not 16-byte aligned", k);
    if (a.n > 0 && (!star->fks[k] || !aligned(star->fks[k], 4))) return fail(LQ_ERR_NULL, "fks[%d] is NULL or misaligned", k);
    a.T[k] = static_cast<const uint8_t*>(tables[k]);
    a.fk[k] = star->fks[k];
  }
  a.chunks = static_cast<int32_t>(a.t.ld / 16);
  a.target = target; a.leaf = leaf; a.onehot = onehot;
  a.onehot_vec_ok = onehot && aligned(onehot, 16) && a.t.l % 16 == 0;
  a.c_f = star->fact.cols;
  a.has_fact_nodes = a.c_f > 0;      // nodes are only evaluated if their column index is < c_f
  if (a.c_f > 0) {
    if (a.n > 0 && (!star->fact.data || star->fact.ld < a.c_f)) return fail(LQ_ERR_NULL, "fact table is malformed");
    a.X = static_cast<const float*>(star->fact.data); a.ldx = star->fact.ld;
  }
  if (a.n == 0) return LQ_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (flags & LQ_CHECK_FKS)
    if ((rc = tree_check_fks(star, ws, ws_bytes, s))) return rc;
  int G = 1;
  while (G < a.chunks && G < 64) G <<= 1;
  if (!a.has_fact_nodes && a.chunks <= 256 && (!a.onehot || (a.onehot_vec_ok && a.t.l % 16 == 0))) {
    const int64_t bblocks = (a.n + 255) / 256;
    if (bblocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
    const dim3 grid(static_cast<unsigned>(bblocks)), block(256);
    if (a.chunks > 64) {                       // 1,025 to 4,096 leaves: two or four chunks per lane
#define LQ_TREE_C(KT_)                                                                                   \
  do {                                                                                                   \
    if (a.chunks <= 128) hipLaunchKernelGGL((fused_tree_batch_kernel<64, KT_, 2>), grid, block, 0, s, a); \
    else hipLaunchKernelGGL((fused_tree_batch_kernel<64, KT_, 4>), grid, block, 0, s, a);                 \
  } while (0)
      if (a.K == 1) LQ_TREE_C(1); else if (a.K == 2) LQ_TREE_C(2); else if (a.K == 3) LQ_TREE_C(3);
      else if (a.K == 4) LQ_TREE_C(4); else LQ_TREE_C(0);
#undef LQ_TREE_C
      LQ_LAUNCH_CHECK("fused_tree_batch_kernel");
      return LQ_OK;
    }
#define LQ_TREE_K(GG, KT_) hipLaunchKernelGGL((fused_tree_batch_kernel<GG, KT_>), grid, block, 0, s, a)
#define LQ_TREE_CASE(GG)                                                            \
  case GG:                                                                          \
    if (a.K == 1) LQ_TREE_K(GG, 1); else if (a.K == 2) LQ_TREE_K(GG, 2);            \
    else if (a.K == 3) LQ_TREE_K(GG, 3); else if (a.K == 4) LQ_TREE_K(GG, 4);       \
    else LQ_TREE_K(GG, 0);                                                          \
    break;
    switch (G) {
      LQ_TREE_CASE(1) LQ_TREE_CASE(2) LQ_TREE_CASE(4) LQ_TREE_CASE(8) LQ_TREE_CASE(16) LQ_TREE_CASE(32) LQ_TREE_CASE(64)
    }
#undef LQ_TREE_CASE
#undef LQ_TREE_K
    LQ_LAUNCH_CHECK("fused_tree_batch_kernel");
    return LQ_OK;
  }
  int64_t blocks = (a.n + 256 / G - 1) / (256 / G);
  size_t lds = 0;
  if (a.has_fact_nodes) {
    static_assert(16384 + 15 <= FT_NEED_MAX, "the table-only targets of the largest tree fit in LDS");
    a.lists = 16 * a.chunks <= FT_LISTS_MAX_L ? 1 : 0;
    lds = ft_lds_bytes(a.chunks, a.lists != 0);
    blocks = std::min<int64_t>(blocks, static_cast<int64_t>(num_cus()) * 8);    // (each workgroup prepares the tree once)
  }
  if (blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
  switch (G) {
#define LQ_TREE_CASE(GG) case GG: hipLaunchKernelGGL(fused_tree_kernel<GG>, dim3(static_cast<unsigned>(blocks)), dim3(256), lds, s, a); break;
    LQ_TREE_CASE(1) LQ_TREE_CASE(2) LQ_TREE_CASE(4) LQ_TREE_CASE(8) LQ_TREE_CASE(16) LQ_TREE_CASE(32) LQ_TREE_CASE(64)
#undef LQ_TREE_CASE
  }
  LQ_LAUNCH_CHECK("fused_tree_kernel");
  return LQ_OK;
}

// Workspace layout of the non-fused pipeline: [256 header | h fp32 | H bf16 | per chunk: T, B, R].
struct TreeWs { size_t fixed, per_row; int64_t ldt, ldb, ldh, ldr; int32_t p_pad; };
static bool tree_ws_layout(const lq_star* star, const lq_tree* tree, TreeWs* w) {
  if (!star || !tree || star->n_dims < 0 || star->n_dims > LQ_MAX_DIMS) return false;
  if (star->n_dims > 0 && !star->dims) return false;
  if (tree->n_nodes < 1 || tree->n_leaves < 1 || tree->n_leaves > 16384) return false;
  size_t kw = star->fact.cols > 0 ? star->fact.cols : 0;
  for (int k = 0; k < star->n_dims; ++k) kw += star->dims[k].cols;
  w->ldt = static_cast<int64_t>(round_up(kw, 4));
  w->p_pad = static_cast<int32_t>(round_up(static_cast<size_t>(tree->n_nodes), 8));
  w->ldb = w->p_pad;
  w->ldh = static_cast<int64_t>(round_up(static_cast<size_t>(tree->n_leaves), 8));
  w->ldr = w->ldh;
  w->fixed = 256 + round_up(static_cast<size_t>(tree->n_leaves) * 4, 256) +
             round_up(static_cast<size_t>(w->p_pad) * w->ldh * 2, 256);
  w->per_row = static_cast<size_t>(w->ldt) * 4 + static_cast<size_t>(w->ldb) * 2 + static_cast<size_t>(w->ldr) * 4;
  return true;
}

size_t lq_tree_workspace_bytes(const lq_star* star, const lq_tree* tree, int64_t chunk_rows) {
  TreeWs w;
  if (chunk_rows < 1 || !tree_ws_layout(star, tree, &w)) return 0;
  return w.fixed + round_up(static_cast<size_t>(chunk_rows), 256) * w.per_row + 3 * 256;
}

int lq_materialized_join_tree(const lq_star* star, const lq_tree* tree, int32_t* leaf, uint8_t* onehot,
                              void* ws, size_t ws_bytes, uint32_t flags, void* hip_stream) {
  clear_error();
  TreeArgs t{};
  int rc = check_star_basic(star, true);
  if (rc) return rc;
  if ((rc = check_tree(tree, &t))) return rc;
  if (!leaf && !onehot) return fail(LQ_ERR_NULL, "neither leaf nor onehot requested");
  if (star->n_dims > 0 && !star->fks) return fail(LQ_ERR_NULL, "fks is NULL");
  if (star->n_fact == 0) return LQ_OK;
  if (star->fact.cols > 0 && !star->fact.data) return fail(LQ_ERR_NULL, "fact data is NULL");
  for (int k = 0; k < star->n_dims; ++k)
    if (!star->fks[k]) return fail(LQ_ERR_NULL, "fks[%d] is NULL", k);
  if (!ws || !aligned(ws, 256)) return fail(LQ_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  TreeWs w;
  if (!tree_ws_layout(star, tree, &w)) return fail(LQ_ERR_SHAPE, "star or tree is malformed");
  if (ws_bytes < w.fixed + 3 * 256 + 256 * w.per_row)
    return fail(LQ_ERR_WORKSPACE, "workspace cannot hold one 256-row chunk (%zu bytes needed)",
                w.fixed + 3 * 256 + 256 * w.per_row);
  int64_t chunk = static_cast<int64_t>((ws_bytes - w.fixed - 3 * 256) / w.per_row) / 256 * 256;
  chunk = std::min<int64_t>(chunk, static_cast<int64_t>(round_up(static_cast<size_t>(star->n_fact), 256)));
  char* base = static_cast<char*>(ws) + 256;
  float* hplus = reinterpret_cast<float*>(base);
  bf16_t* Hb = reinterpret_cast<bf16_t*>(base + round_up(static_cast<size_t>(t.l) * 4, 256));
  char* per_chunk = static_cast<char*>(ws) + w.fixed;
  float* T = reinterpret_cast<float*>(per_chunk);
  bf16_t* B = reinterpret_cast<bf16_t*>(per_chunk + round_up(static_cast<size_t>(chunk) * w.ldt * 4, 256));
  float* R = reinterpret_cast<float*>(reinterpret_cast<char*>(B) + round_up(static_cast<size_t>(chunk) * w.ldb * 2, 256));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (flags & LQ_CHECK_FKS)      // the flag word takes the first bytes of the workspace, which are rewritten below
    if ((rc = tree_check_fks(star, ws, ws_bytes, s))) return rc;
  const int cus = num_cus();
  {
    const int64_t total = static_cast<int64_t>(w.p_pad) * w.ldh;
    const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>((total + 255) / 256, static_cast<int64_t>(cus) * 8));
    hipLaunchKernelGGL(tree_h_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, t, w.p_pad, Hb, w.ldh, hplus);
    LQ_LAUNCH_CHECK("tree_h_kernel");
  }
  for (int64_t r0 = 0; r0 < star->n_fact; r0 += chunk) {
    const int64_t m = std::min<int64_t>(chunk, star->n_fact - r0);
    if ((rc = launch_materialize(*star, T, w.ldt, r0, m, s))) return rc;
    const int64_t bit_blocks = std::min<int64_t>((m * w.ldb + 255) / 256, static_cast<int64_t>(cus) * 32);
    hipLaunchKernelGGL(tree_bits_kernel, dim3(static_cast<unsigned>(bit_blocks)), dim3(256), 0, s, t, T, w.ldt, m, B, w.ldb);
    LQ_LAUNCH_CHECK("tree_bits_kernel");
    if ((rc = launch_gemm(B, w.ldb, Hb, w.ldh, R, w.ldr, nullptr, m, t.l, w.p_pad, 0, LQ_BF16, LQ_F32, s))) return rc;
    const int64_t match_blocks = std::min<int64_t>((m + 3) / 4, static_cast<int64_t>(cus) * 16);
    hipLaunchKernelGGL(tree_match_kernel, dim3(static_cast<unsigned>(match_blocks)), dim3(256), 0, s, t.l, R, w.ldr, m, r0,
                       hplus, leaf, onehot);
    LQ_LAUNCH_CHECK("tree_match_kernel");
  }
  return LQ_OK;
}

// ceil(l / 64), rounded up to an even number from three words on: mask rows then start 16 bytes apart and the
// join reads them two words at a time (129 leaves: four words, the last all zero).
int64_t lq_tree_mask_words(int32_t n_leaves) {
  if (n_leaves < 1) return 0;
  const int64_t w = (static_cast<int64_t>(n_leaves) + 63) / 64;
  return (w >= 3 && (w & 1)) ? w + 1 : w;
}

int lq_tree_compress_tables(const lq_star* star, const lq_tree* tree, const void* const* tables,
                            uint64_t* const* masks, void* hip_stream) {
  clear_error();
  TreeArgs t{};
  int rc = check_star_basic(star, false);
  if (rc) return rc;
  if ((rc = check_tree(tree, &t))) return rc;
  if (star->n_dims > 0 && (!tables || !masks || !star->dims)) return fail(LQ_ERR_NULL, "tables, masks or star->dims is NULL");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (star->n_dims == 0) return LQ_OK;
  DimSlice sl[LQ_MAX_DIMS];
  u64* mk[LQ_MAX_DIMS];
  int32_t off = star->fact.cols;
  for (int k = 0; k < star->n_dims; ++k) {
    const lq_mat& d = star->dims[k];
    if (d.rows < 1 || d.cols < 1) return fail(LQ_ERR_SHAPE, "dims[%d] is malformed", k);
    if (!tables[k] || !masks[k] || !aligned(masks[k], 8) || !aligned(tables[k], 16))
      return fail(LQ_ERR_NULL, "tables[%d] or masks[%d] is NULL or misaligned", k, k);
    sl[k] = DimSlice{nullptr, 0, d.rows, off, d.cols, static_cast<uint8_t*>(const_cast<void*>(tables[k]))};
    mk[k] = reinterpret_cast<u64*>(masks[k]);
    off += d.cols;
  }
  return compress_slices(t, sl, mk, star->n_dims, s);
}

int64_t lq_tree_fact_mask_bytes(int32_t n_nodes, int32_t n_leaves) {
  if (n_nodes < 1 || n_leaves < 1) return 0;
  return static_cast<int64_t>(round_up(16 + 8 * static_cast<size_t>(n_nodes), 16)) +
         static_cast<int64_t>(n_nodes) * lq_tree_mask_words(n_leaves) * 16 +
         static_cast<int64_t>(round_up(4 * (static_cast<size_t>(n_leaves) + 1), 16)) +
         static_cast<int64_t>(FACT_LIST_PER_LEAF) * n_leaves * 16;
}

int lq_tree_fact_masks(int32_t c_f, const lq_tree* tree, void* fact_masks, void* hip_stream) {
  clear_error();
  TreeArgs t{};
  int rc = check_tree(tree, &t);
  if (rc) return rc;
  if (c_f < 0) return fail(LQ_ERR_SHAPE, "c_f < 0");
  if (!fact_masks || !aligned(fact_masks, 16)) return fail(LQ_ERR_NULL, "fact_masks is NULL or misaligned");
  const int32_t words = static_cast<int32_t>(lq_tree_mask_words(t.l));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const FactBuf fb = fact_buf(fact_masks, t.p, t.l);
  hipLaunchKernelGGL(tree_fact_masks_kernel, dim3(static_cast<unsigned>((t.p + 15) / 16)), dim3(256), 0, s, t, c_f, words, fb);
  LQ_LAUNCH_CHECK("tree_fact_masks_kernel");
  const unsigned leaf_blocks = static_cast<unsigned>((t.l + 63) / 64);
  hipLaunchKernelGGL(tree_fact_list_count_kernel, dim3(leaf_blocks), dim3(64 * FL_WAVES), 0, s, t, c_f, fb.leaf_off);
  LQ_LAUNCH_CHECK("tree_fact_list_count_kernel");
  hipLaunchKernelGGL(tree_fact_list_scan_kernel, dim3(1), dim3(1024), 0, s, fb.leaf_off, t.l, fb.cnt,
                     static_cast<int64_t>(FACT_LIST_PER_LEAF) * t.l);
  LQ_LAUNCH_CHECK("tree_fact_list_scan_kernel");
  hipLaunchKernelGGL(tree_fact_list_fill_kernel, dim3(leaf_blocks), dim3(64 * FL_WAVES), 0, s, t, c_f, fb.cnt, fb.leaf_off, fb.leaf_ent);
  LQ_LAUNCH_CHECK("tree_fact_list_fill_kernel");
  return LQ_OK;
}

int lq_fused_join_tree_masks(const lq_star* star, const lq_tree* tree, const uint64_t* const* masks,
                             const void* fact_masks, int32_t* leaf, uint8_t* onehot, uint32_t flags,
                             void* hip_stream) {
  clear_error();
  if (flags & LQ_CHECK_FKS)
    return fail(LQ_ERR_UNSUPPORTED, "this call has no workspace for LQ_CHECK_FKS: check the keys with lq_fused_join_tree or map them with the key map");
  TreeArgs t{};
  int rc = check_star_basic(star, false);
  if (rc) return rc;
  if ((rc = check_tree(tree, &t))) return rc;
  if (star->n_dims > 0 && (!masks || !star->fks)) return fail(LQ_ERR_NULL, "masks or fks is NULL");
  if (!leaf && !onehot) return fail(LQ_ERR_NULL, "neither leaf nor onehot requested");
  if (leaf && !aligned(leaf, 4)) return fail(LQ_ERR_SHAPE, "leaf is misaligned");
  MaskJoinArgs a{};
  a.n = star->n_fact; a.K = star->n_dims; a.l = t.l; a.words = static_cast<int32_t>(lq_tree_mask_words(t.l));
  for (int k = 0; k < a.K; ++k) {
    if (!masks[k] || !aligned(masks[k], 8)) return fail(LQ_ERR_NULL, "masks[%d] is NULL or misaligned", k);
    if (a.n > 0 && (!star->fks[k] || !aligned(star->fks[k], 4))) return fail(LQ_ERR_NULL, "fks[%d] is NULL or misaligned", k);
    a.M[k] = reinterpret_cast<const u64*>(masks[k]);
    a.fk[k] = star->fks[k];
  }
  a.leaf = leaf; a.onehot = onehot;
  a.onehot_vec = onehot && aligned(onehot, 16) && t.l % 16 == 0;
  a.onehot_w4 = onehot && aligned(onehot, 4) && t.l % 4 == 0;
  if (star->fact.cols > 0) {
    const lq_mat& x = star->fact;
    if (!fact_masks || !aligned(fact_masks, 16))
      return fail(LQ_ERR_NULL, "the fact table has columns: fact_masks (from lq_tree_fact_masks) is NULL or misaligned");
    if (x.ld < x.cols || (a.n > 0 && (!x.data || !aligned(x.data, 4)))) return fail(LQ_ERR_SHAPE, "fact is malformed");
    const FactBuf fb = fact_buf(const_cast<void*>(fact_masks), t.p, t.l);
    a.f.X = static_cast<const float*>(x.data); a.f.ldx = x.ld; a.f.c_f = x.cols;
    a.f.vec_x = (aligned(x.data, 16) && x.ld % 4 == 0 && x.cols % 4 == 0) ? 1 : 0;
    a.f.cnt = fb.cnt; a.f.feat = fb.feat; a.f.thr = fb.thr; a.f.tf = fb.tf;
    a.f.leaf_off = fb.leaf_off; a.f.leaf_ent = fb.leaf_ent;
  }
  if (a.n == 0) return LQ_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  bool wide_loads = a.words % 2 == 0;
  for (int k = 0; k < a.K; ++k) wide_loads = wide_loads && aligned(masks[k], 16);
  auto clear_onehot = [&]() {
    const int64_t pieces = (a.n * a.l + 15) / 16;
    const int64_t zb = std::max<int64_t>(1, std::min<int64_t>((pieces + 255) / 256, static_cast<int64_t>(num_cus()) * 32));
    hipLaunchKernelGGL(zero_bytes_kernel, dim3(static_cast<unsigned>(zb)), dim3(256), 0, s, onehot, a.n * a.l);
  };
  // Small trees on a fact table of more columns than the kernels below keep in registers: those re-read the row for
  // every fact-side node, the walk reads the few values the leaves still possible ask for.  (When the per-leaf lists
  // are not there the walk returns at once and the general kernel at the end of this function does the join.)
  if (a.f.X && a.f.c_f > FACT_REG_COLS && a.words <= 2 && (a.words == 1 || wide_loads) && aligned(a.f.tf, 16)) {
    const int64_t rb = (a.n + 255) / 256;
    if (rb > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
    if (onehot && !(a.onehot_vec || a.onehot_w4)) {
      clear_onehot();
      LQ_LAUNCH_CHECK("zero_bytes_kernel");
    }
    const dim3 rgrid(static_cast<unsigned>(rb)), rblock(256);
    const int oh = !onehot ? 0 : ((a.onehot_vec || a.onehot_w4) ? 1 : 2);
#define LQ_WALK1(WPL_)                                                                                          \
  do {                                                                                                          \
    if (oh == 0) hipLaunchKernelGGL((fused_tree_mask_rows_walk_kernel<1, WPL_, 0>), rgrid, rblock, 0, s, a);      \
    else if (oh == 1) hipLaunchKernelGGL((fused_tree_mask_rows_walk_kernel<1, WPL_, 1>), rgrid, rblock, 0, s, a); \
    else hipLaunchKernelGGL((fused_tree_mask_rows_walk_kernel<1, WPL_, 2>), rgrid, rblock, 0, s, a);              \
  } while (0)
    if (a.words == 1) LQ_WALK1(1); else LQ_WALK1(2);
#undef LQ_WALK1
    LQ_LAUNCH_CHECK("fused_tree_mask_rows_walk_kernel");
    a.skip_when_lists = 1;
  }
  if (!a.skip_when_lists && a.words == 1 && !onehot && star->dims && a.K >= 1 && a.K <= 4 && a.n >= (1 << 20)) {
    // small mask tables go to LDS (smallest first) as long as they fit next to each other
    MaskLds L{};
    int order[LQ_MAX_DIMS];
    bool ok = true;
    for (int k = 0; k < a.K; ++k) {
      order[k] = k;
      L.off[k] = -1;
      if (star->dims[k].rows < 1 || star->dims[k].rows > 0x7fffffffLL || !aligned(masks[k], 16)) ok = false;
      else L.rows[k] = static_cast<int32_t>(star->dims[k].rows);
    }
    if (ok) {
      std::stable_sort(order, order + a.K, [&](int x, int y) { return L.rows[x] < L.rows[y]; });
      int64_t used = 0;
      const int64_t budget = (156 * 1024) / 8;             // of the 160 KB of a compute unit; the fact-side nodes take 3 KB more
      for (int q = 0; q < a.K; ++q) {
        const int k = order[q];
        if (used + L.rows[k] > budget) break;
        L.off[k] = static_cast<int32_t>(used);
        used += (L.rows[k] + 1) / 2 * 2;
      }
      if (used > 0) {
        L.vec = aligned(leaf, 16) ? 1 : 0;
        for (int k = 0; k < a.K; ++k) L.vec = (L.vec && aligned(star->fks[k], 16)) ? 1 : 0;
        L.fact_off = static_cast<int32_t>(used);
        const size_t lds = (static_cast<size_t>(used) + (a.f.X ? 3 * FACT_LDS_NODES : 0)) * 8;
        const int64_t need = (a.n + MLDS_THREADS * 4 - 1) / (MLDS_THREADS * 4);
        const dim3 grid(static_cast<unsigned>(std::min<int64_t>(need, num_cus()))), block(MLDS_THREADS);
#define LQ_TML_F(KT_, F_)                                                                                 \
  do {                                                                                                    \
    if (lds > 64 * 1024)                                                                                  \
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_tree_mask_lds_kernel<KT_, F_>), \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
    hipLaunchKernelGGL((fused_tree_mask_lds_kernel<KT_, F_>), grid, block, lds, s, a, L);                 \
  } while (0)
#define LQ_TML(KT_)                                                                                       \
  do {                                                                                                    \
    if (a.f.X) LQ_TML_F(KT_, true); else LQ_TML_F(KT_, false);                                            \
  } while (0)
        if (a.K == 1) LQ_TML(1); else if (a.K == 2) LQ_TML(2); else if (a.K == 3) LQ_TML(3); else LQ_TML(4);
#undef LQ_TML
#undef LQ_TML_F
        LQ_LAUNCH_CHECK("fused_tree_mask_lds_kernel");
        return LQ_OK;
      }
    }
  }
  // (one-hot rows whose length is no multiple of 4 are cleared first and the join sets the byte of every leaf reached)
  if (wide_loads && a.f.X && a.words >= 4 && a.words <= 128 && aligned(a.f.tf, 16)) {
    const int64_t rb = (a.n + 255) / 256;
    if (rb > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
    if (onehot && !(a.onehot_vec || a.onehot_w4)) {
      clear_onehot();
      LQ_LAUNCH_CHECK("zero_bytes_kernel");
    }
    const dim3 rgrid(static_cast<unsigned>(rb)), rblock(256);
    int G = 2;
    while (2 * G < a.words) G *= 2;
    // (whether the tree's per-leaf lists are there is known on the device only: both kernels are launched and the one
    // whose form of the fact side is not there returns at once)
    const int oh = !onehot ? 0 : ((a.onehot_vec || a.onehot_w4) ? 1 : 2);
#define LQ_ROWS_FACT(G_)                                                                                         \
  do {                                                                                                           \
    if (oh == 0) hipLaunchKernelGGL((fused_tree_mask_rows_walk_kernel<G_, 2, 0>), rgrid, rblock, 0, s, a);        \
    else if (oh == 1) hipLaunchKernelGGL((fused_tree_mask_rows_walk_kernel<G_, 2, 1>), rgrid, rblock, 0, s, a);   \
    else hipLaunchKernelGGL((fused_tree_mask_rows_walk_kernel<G_, 2, 2>), rgrid, rblock, 0, s, a);                \
    hipLaunchKernelGGL(fused_tree_mask_rows_fact_kernel<G_>, rgrid, rblock, 0, s, a);                            \
  } while (0)
    switch (G) {
      case 2: LQ_ROWS_FACT(2); break;
      case 4: LQ_ROWS_FACT(4); break;
      case 8: LQ_ROWS_FACT(8); break;
      case 16: LQ_ROWS_FACT(16); break;
      case 32: LQ_ROWS_FACT(32); break;
      default: LQ_ROWS_FACT(64); break;
    }
#undef LQ_ROWS_FACT
    LQ_LAUNCH_CHECK("fused_tree_mask_rows_fact_kernel");
    return LQ_OK;
  }
  // (one-hot rows of up to four words are faster from the kernel below, which writes them 16 bytes per lane through the
  // cross-lane network when l is a multiple of 16: 0.14 ms per 2.4e6 rows at 256 leaves; larger ones are cleared first
  // and get a byte per leaf reached: 1.7 instead of 15.7 ms at 3,000 leaves)
  if (wide_loads && (!onehot || a.words > 4) && !a.f.X && a.words >= 4 && a.words <= 128) {
    const int64_t rb = (a.n + 255) / 256;
    if (rb > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
    const dim3 rgrid(static_cast<unsigned>(rb)), rblock(256);
    int G = 2;
    while (2 * G < a.words) G *= 2;
    const int oh = !onehot ? 0 : ((a.onehot_vec || a.onehot_w4) ? 1 : 2);
    if (oh == 2) {
      clear_onehot();
      LQ_LAUNCH_CHECK("zero_bytes_kernel");
    }
#define LQ_TR(KT_, G_)                                                                                \
  do {                                                                                                 \
    if (oh == 1) hipLaunchKernelGGL((fused_tree_mask_rows_kernel<KT_, G_, 1>), rgrid, rblock, 0, s, a);      \
    else if (oh == 2) hipLaunchKernelGGL((fused_tree_mask_rows_kernel<KT_, G_, 2>), rgrid, rblock, 0, s, a); \
    else hipLaunchKernelGGL((fused_tree_mask_rows_kernel<KT_, G_, 0>), rgrid, rblock, 0, s, a);              \
  } while (0)
#define LQ_TR_G(KT_)                                                                                   \
  do {                                                                                                 \
    switch (G) {                                                                                       \
      case 2: LQ_TR(KT_, 2); break;                                                                    \
      case 4: LQ_TR(KT_, 4); break;                                                                    \
      case 8: LQ_TR(KT_, 8); break;                                                                    \
      case 16: LQ_TR(KT_, 16); break;                                                                  \
      case 32: LQ_TR(KT_, 32); break;                                                                  \
      default: LQ_TR(KT_, 64); break;                                                                  \
    }                                                                                                  \
  } while (0)
    if (a.K == 1) LQ_TR_G(1); else if (a.K == 2) LQ_TR_G(2); else if (a.K == 3) LQ_TR_G(3); else if (a.K == 4) LQ_TR_G(4); else LQ_TR_G(0);
#undef LQ_TR_G
#undef LQ_TR
    LQ_LAUNCH_CHECK("fused_tree_mask_rows_kernel");
    return LQ_OK;
  }
  const int64_t blocks = (a.n + 1023) / 1024;
  if (blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "too many rows for one launch");
  const dim3 grid(static_cast<unsigned>(blocks)), block(256);
  const int wmax = (a.onehot_vec && a.words <= 4) ? (a.words <= 1 ? 1 : (a.words <= 2 ? 2 : 4)) : 0;
#define LQ_TM(KT_, W_)                                                                                \
  do {                                                                                                \
    if (wide_loads) hipLaunchKernelGGL((fused_tree_mask_kernel<KT_, W_, 2>), grid, block, 0, s, a);   \
    else hipLaunchKernelGGL((fused_tree_mask_kernel<KT_, W_, 1>), grid, block, 0, s, a);              \
  } while (0)
#define LQ_TM_W(KT_)                                                                                  \
  do {                                                                                                \
    if (wmax == 0) LQ_TM(KT_, 0); else if (wmax == 1) LQ_TM(KT_, 1); else if (wmax == 2) LQ_TM(KT_, 2); else LQ_TM(KT_, 4); \
  } while (0)
  if (a.K == 1) LQ_TM_W(1); else if (a.K == 2) LQ_TM_W(2); else if (a.K == 3) LQ_TM_W(3); else if (a.K == 4) LQ_TM_W(4); else LQ_TM_W(0);
#undef LQ_TM_W
#undef LQ_TM
  LQ_LAUNCH_CHECK("fused_tree_mask_kernel");
  return LQ_OK;
}

}  // extern "C"
