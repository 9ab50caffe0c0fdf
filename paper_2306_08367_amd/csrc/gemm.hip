// Dense C = act(A * B + bias) on the matrix cores, fp32 accumulate.
//
// Used for the pre-fusion products P_k = D_k * (rows of L owned by dimension k)
// (underlined terms of Eq. 1) and for the layer-by-layer model evaluation of the
// non-fused pipeline (T * L, second line of Eq. 1).
//
// Tiling: a 256-thread workgroup (4 wavefronts) owns a 128 x 64 tile of C; each
// wavefront owns 32 rows x 64 columns as two 32x32 MFMA accumulators.  A and B
// tiles are staged through LDS k-major so that the 32 lanes reading one MFMA
// operand hit 32 consecutive words.
#include "lq_common.h"

namespace lq {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 64, BK = 16;
constexpr int PAD = 4;  // keeps rows of the k-major tiles on different banks for the staging stores

template <typename TA, typename TC>
__global__ __launch_bounds__(256) void gemm_kernel(const TA* __restrict__ A, int64_t lda,
                                                   const TA* __restrict__ B, int64_t ldb,
                                                   TC* __restrict__ C, int64_t ldc,
                                                   const TA* __restrict__ bias, int64_t M,
                                                   int32_t N, int32_t Kd, int relu,
                                                   int32_t tiles_n) {
  __shared__ float As[BK][BM + PAD];
  __shared__ float Bs[BK][BN + PAD];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t tile_m = static_cast<int64_t>(blockIdx.x) / tiles_n;
  const int tile_n = static_cast<int>(static_cast<int64_t>(blockIdx.x) % tiles_n);
  const int64_t m0 = tile_m * BM;
  const int n0 = tile_n * BN;

  v16f acc0 = {0}, acc1 = {0};

  for (int k0 = 0; k0 < Kd; k0 += BK) {
    // A tile: 128 rows x 16 k.  Thread t stages row t/2, k in [8*(t&1), +8).
    {
      const int r = tid >> 1;
      const int kb = (tid & 1) * 8;
      const int64_t row = m0 + r;
      const TA* src = A + row * lda + k0 + kb;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float v = 0.f;
        if (row < M && k0 + kb + q < Kd) v = Elem<TA>::load(src + q);
        As[kb + q][r] = v;
      }
    }
    // B tile: 16 k x 64 columns.  Thread t stages k = t/16, columns 4*(t%16) .. +4.
    {
      const int kk = tid >> 4;
      const int cb = (tid & 15) * 4;
      const TA* src = B + static_cast<int64_t>(k0 + kk) * ldb + n0 + cb;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v = 0.f;
        if (k0 + kk < Kd && n0 + cb + q < N) v = Elem<TA>::load(src + q);
        Bs[kk][cb + q] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int k = kk + (lane >> 5);
      const float a = As[k][wave * 32 + (lane & 31)];
      const float b0 = Bs[k][lane & 31];
      const float b1 = Bs[k][32 + (lane & 31)];
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc1, 0, 0, 0);
    }
    __syncthreads();
  }

  // 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
  const int col_in = lane & 31;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int col = n0 + half * 32 + col_in;
    if (col >= N) continue;
    const float bv = bias ? Elem<TA>::load(bias + col) : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = wave * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const int64_t row = m0 + r;
      if (row >= M) continue;
      float x = (half ? acc1[v] : acc0[v]) + bv;
      if (relu) x = fmaxf(x, 0.f);
      Elem<TC>::store(C + row * ldc + col, x);
    }
  }
}

template <typename TA, typename TC>
int launch_typed(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                 const void* bias, int64_t M, int32_t N, int32_t Kd, int relu, hipStream_t s) {
  const int64_t tiles_m = (M + BM - 1) / BM;
  const int32_t tiles_n = (N + BN - 1) / BN;
  const int64_t blocks = tiles_m * tiles_n;
  if (blocks <= 0) return LQ_OK;
  if (blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "gemm: %lld tiles exceed one grid", (long long)blocks);
  hipLaunchKernelGGL((gemm_kernel<TA, TC>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                     static_cast<const TA*>(A), lda, static_cast<const TA*>(B), ldb,
                     static_cast<TC*>(C), ldc, static_cast<const TA*>(bias), M, N, Kd, relu, tiles_n);
  LQ_LAUNCH_CHECK("gemm_kernel");
  return LQ_OK;
}

}  // namespace

// C[M x N] = act(A[M x Kd] * B[Kd x N] + bias).  A, B, bias share `in_dtype`.
int launch_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                const void* bias, int64_t M, int32_t N, int32_t Kd, int relu, int32_t in_dtype,
                int32_t out_dtype, hipStream_t s) {
  if (in_dtype == LQ_F32 && out_dtype == LQ_F32)
    return launch_typed<float, float>(A, lda, B, ldb, C, ldc, bias, M, N, Kd, relu, s);
  if (in_dtype == LQ_BF16 && out_dtype == LQ_F32)
    return launch_typed<bf16_t, float>(A, lda, B, ldb, C, ldc, bias, M, N, Kd, relu, s);
  if (in_dtype == LQ_BF16 && out_dtype == LQ_BF16)
    return launch_typed<bf16_t, bf16_t>(A, lda, B, ldb, C, ldc, bias, M, N, Kd, relu, s);
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
