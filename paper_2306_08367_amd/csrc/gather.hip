// Materialisation of the joined table (first line of Eq. 1, T = X_f M_f + sum_k I_k D_k M_k),
// foreign-key validation, and the plain stream-copy yardstick.
#include "lq_common.h"

namespace lq {
namespace {

struct MatArgs {
  int64_t row0, rows;
  const void* X; int64_t ldx; int32_t c_f;
  int32_t K;
  const void* D[LQ_MAX_DIMS]; int64_t ldd[LQ_MAX_DIMS]; int32_t c[LQ_MAX_DIMS];
  int32_t off[LQ_MAX_DIMS];          // first column of dimension k in T
  const int32_t* fk[LQ_MAX_DIMS];
  void* T; int64_t ldt; int32_t kw;  // joined width
};

// One thread per (row, column) of the chunk, columns fastest: the writes to T are
// fully coalesced and the reads of one dimension row are contiguous across lanes.
template <typename E>
__global__ __launch_bounds__(256) void materialize_kernel(MatArgs a) {
  const int64_t total = a.rows * a.kw;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; idx < total;
       idx += stride) {
    const int64_t r = idx / a.kw;
    const int col = static_cast<int>(idx - r * a.kw);
    const int64_t row = a.row0 + r;
    E v;
    if (col < a.c_f) {
      v = static_cast<const E*>(a.X)[row * a.ldx + col];
    } else {
      int k = 0;
#pragma unroll
      for (int q = 1; q < LQ_MAX_DIMS; ++q)
        if (q < a.K && col >= a.off[q]) k = q;
      const int64_t j = a.fk[k][row];
      v = static_cast<const E*>(a.D[k])[j * a.ldd[k] + (col - a.off[k])];
    }
    static_cast<E*>(a.T)[r * a.ldt + col] = v;
  }
}

// 16-byte version: every segment of the joined row (fact columns, each dimension's columns) is a
// whole number of 16-byte chunks and every row start is 16-byte aligned.  A group of GROUP lanes
// copies one joined row, chunk by chunk; a dimension row is read as one contiguous run.
template <int GROUP>
__global__ __launch_bounds__(256) void materialize_vec_kernel(MatArgs a, int vec /*elements per chunk*/,
                                                              int chunks_per_row) {
  const int sub = threadIdx.x / GROUP, c0 = threadIdx.x % GROUP;
  constexpr int ROWS_PER_BLOCK = 256 / GROUP;
  const size_t es = 16 / vec;
  for (int64_t r = static_cast<int64_t>(blockIdx.x) * ROWS_PER_BLOCK + sub; r < a.rows;
       r += static_cast<int64_t>(gridDim.x) * ROWS_PER_BLOCK) {
    const int64_t row = a.row0 + r;
    for (int ch = c0; ch < chunks_per_row; ch += GROUP) {
      const int col = ch * vec;
      const char* src;
      if (col < a.c_f) {
        src = static_cast<const char*>(a.X) + (row * a.ldx + col) * es;
      } else {
        int k = 0;
#pragma unroll
        for (int q = 1; q < LQ_MAX_DIMS; ++q)
          if (q < a.K && col >= a.off[q]) k = q;
        const int64_t j = a.fk[k][row];
        src = static_cast<const char*>(a.D[k]) + (j * a.ldd[k] + (col - a.off[k])) * es;
      }
      const uint4 v = *reinterpret_cast<const uint4*>(src);
      *reinterpret_cast<uint4*>(static_cast<char*>(a.T) + (r * a.ldt + col) * es) = v;
    }
  }
}

struct CheckArgs {
  int64_t n; int32_t K;
  const int32_t* fk[LQ_MAX_DIMS];
  int64_t rows[LQ_MAX_DIMS];
  int negative_ok;
};

__global__ __launch_bounds__(256) void check_fks_kernel(CheckArgs a, int32_t* flag) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  int bad = 0;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < a.n; i += stride)
    for (int k = 0; k < a.K; ++k) {
      const int64_t j = a.fk[k][i];
      if (j >= a.rows[k] || (j < 0 && !a.negative_ok)) bad = 1;
    }
  if (bad) atomicOr(flag, 1);
}

// Group codes of the dimension side: bit 1 of the flag is raised for a code outside [0, card) on a
// dimension row whose mask lets it through (rows that are filtered out are never looked up).
struct CodeCheckArgs {
  int32_t K;
  const uint8_t* mask[LQ_MAX_DIMS];
  const int32_t* code[LQ_MAX_DIMS];
  int64_t rows[LQ_MAX_DIMS];
  int32_t card[LQ_MAX_DIMS];
};

__global__ __launch_bounds__(256) void check_codes_kernel(CodeCheckArgs a, int32_t* flag) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  int bad = 0;
  for (int k = 0; k < a.K; ++k) {
    if (!a.code[k]) continue;
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j < a.rows[k]; j += stride) {
      const int32_t v = a.code[k][j];
      if ((v < 0 || v >= a.card[k]) && (!a.mask[k] || a.mask[k][j])) bad = 1;
    }
  }
  if (bad) atomicOr(flag, 2);
}

__global__ __launch_bounds__(256) void zero_flag_kernel(int32_t* flag) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *flag = 0;
}

// One 16-byte element per thread: workgroups sweep memory in launch order, which keeps the
// set of open DRAM pages compact (measurably faster here than a grid-stride loop).
__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst,
                                                   const uint4* __restrict__ src, int64_t n16) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

}  // namespace

int launch_materialize(const lq_star& star, void* T, int64_t ldt, int64_t row0, int64_t rows,
                       hipStream_t s) {
  MatArgs a{};
  a.row0 = row0; a.rows = rows;
  a.X = star.fact.data; a.ldx = star.fact.ld; a.c_f = star.fact.cols;
  a.K = star.n_dims;
  int32_t off = a.c_f;
  for (int k = 0; k < a.K; ++k) {
    a.D[k] = star.dims[k].data; a.ldd[k] = star.dims[k].ld; a.c[k] = star.dims[k].cols;
    a.off[k] = off; off += a.c[k];
    a.fk[k] = star.fks[k];
  }
  a.T = T; a.ldt = ldt; a.kw = off;
  const int64_t total = rows * off;
  if (total <= 0) return LQ_OK;
  {
    const int32_t dt0 = a.c_f > 0 ? star.fact.dtype : star.dims[0].dtype;
    const int vec = dt0 == LQ_BF16 ? 8 : 4;
    const size_t es = dtype_size(dt0);
    bool ok = aligned(T, 16) && ldt % vec == 0 && a.c_f % vec == 0 &&
              (a.c_f == 0 || (aligned(a.X, 16) && a.ldx % vec == 0));
    for (int k = 0; k < a.K && ok; ++k)
      ok = a.c[k] % vec == 0 && a.ldd[k] % vec == 0 && aligned(a.D[k], 16);
    (void)es;
    if (ok) {
      const int cpr = off / vec;
      int group = 1;
      while (group < cpr && group < 64) group <<= 1;
      const int rpb = 256 / group;
      const int64_t blocks = std::min<int64_t>((rows + rpb - 1) / rpb, 0x7fffffffLL);
      switch (group) {
#define LQ_MAT_CASE(G) case G: hipLaunchKernelGGL(materialize_vec_kernel<G>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, a, vec, cpr); break;
        LQ_MAT_CASE(1) LQ_MAT_CASE(2) LQ_MAT_CASE(4) LQ_MAT_CASE(8) LQ_MAT_CASE(16) LQ_MAT_CASE(32) LQ_MAT_CASE(64)
#undef LQ_MAT_CASE
      }
      LQ_LAUNCH_CHECK("materialize_vec_kernel");
      return LQ_OK;
    }
  }
  const int64_t blocks = std::min<int64_t>((total + 255) / 256, static_cast<int64_t>(num_cus()) * 16);
  const int32_t dt = a.c_f > 0 ? star.fact.dtype : star.dims[0].dtype;
  if (dt == LQ_BF16)
    hipLaunchKernelGGL(materialize_kernel<uint16_t>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(materialize_kernel<float>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, a);
  LQ_LAUNCH_CHECK("materialize_kernel");
  return LQ_OK;
}

int launch_check_fks(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                     bool negative_ok, int32_t* d_flag, hipStream_t s) {
  CheckArgs a{};
  a.n = n; a.K = K; a.negative_ok = negative_ok ? 1 : 0;
  for (int k = 0; k < K; ++k) { a.fk[k] = fks[k]; a.rows[k] = rows[k]; }
  hipLaunchKernelGGL(zero_flag_kernel, dim3(1), dim3(64), 0, s, d_flag);
  LQ_LAUNCH_CHECK("zero_flag_kernel");
  if (n > 0 && K > 0) {
    const int64_t blocks = std::min<int64_t>((n + 255) / 256, static_cast<int64_t>(num_cus()) * 8);
    hipLaunchKernelGGL(check_fks_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, a, d_flag);
    LQ_LAUNCH_CHECK("check_fks_kernel");
  }
  return LQ_OK;
}

// Must follow launch_check_fks on the same stream (which clears the flag word).
int launch_check_codes(int32_t K, const int64_t* rows, const uint8_t* const* mask, const int32_t* const* code,
                       const int32_t* card, int32_t* d_flag, hipStream_t s) {
  CodeCheckArgs a{};
  a.K = K;
  int64_t most = 0;
  for (int k = 0; k < K; ++k) {
    a.mask[k] = mask ? mask[k] : nullptr;
    a.code[k] = code ? code[k] : nullptr;
    a.rows[k] = rows[k];
    a.card[k] = (code && code[k] && card) ? card[k] : 1;
    if (a.code[k]) most = std::max(most, rows[k]);
  }
  if (most == 0) return LQ_OK;
  const int64_t blocks = std::min<int64_t>((most + 255) / 256, static_cast<int64_t>(num_cus()) * 8);
  hipLaunchKernelGGL(check_codes_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, a, d_flag);
  LQ_LAUNCH_CHECK("check_codes_kernel");
  return LQ_OK;
}

int launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  int64_t n16 = static_cast<int64_t>(bytes / 16);
  const uint4* sp = static_cast<const uint4*>(src);
  uint4* dp = static_cast<uint4*>(dst);
  const int64_t per_launch = static_cast<int64_t>(1) << 37 >> 4;   // 128 GiB per launch keeps the grid below 2^31
  while (n16 > 0) {
    const int64_t m = std::min<int64_t>(n16, per_launch);
    hipLaunchKernelGGL(copy_kernel, dim3(static_cast<unsigned>((m + 255) / 256)), dim3(256), 0, s, dp, sp, m);
    LQ_LAUNCH_CHECK("copy_kernel");
    sp += m; dp += m; n16 -= m;
  }
  return LQ_OK;
}

}  // namespace lq
