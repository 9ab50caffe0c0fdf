// Internal helpers shared by the HIP sources of liblq (gfx950 only).
#ifndef LQ_COMMON_H_
#define LQ_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include <algorithm>

#include "lq.h"

namespace lq {

// ---- host side ---------------------------------------------------------------------------

// Records a formatted message for lq_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define LQ_HIP_TRY(expr)                                                              \
  do {                                                                                \
    hipError_t e_ = (expr);                                                           \
    if (e_ != hipSuccess)                                                             \
      return ::lq::fail(LQ_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));          \
  } while (0)

// Checks the launch that was just made.
#define LQ_LAUNCH_CHECK(what)                                                         \
  do {                                                                                \
    hipError_t e_ = hipGetLastError();                                                \
    if (e_ != hipSuccess)                                                             \
      return ::lq::fail(LQ_ERR_HIP, "launch of %s: %s", what, hipGetErrorString(e_)); \
  } while (0)

inline size_t dtype_size(int32_t dt) { return dt == LQ_BF16 ? 2 : 4; }
inline bool dtype_ok(int32_t dt) { return dt == LQ_F32 || dt == LQ_BF16; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
__host__ __device__ inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Number of compute units of the current device (cached per process).
int num_cus();

// Workgroups of `kernel` (of `threads` threads and `lds` bytes of dynamic LDS) that one compute unit of the
// current device holds at a time, by registers, LDS and wave slots; at least 1.  Cached per kernel and
// LDS size.  Grid-stride kernels size their grid as a whole multiple of this: the workgroups beyond
// one resident set only start when earlier ones end, at whatever occupancy is then left.
int resident_per_cu(const void* kernel, int threads, size_t lds);

// Everything a predict kernel needs, passed by value as the kernel argument.
struct PredictArgs {
  int64_t n;
  const void* X;            // [n x c_f], model dtype
  int64_t ldx;
  int32_t c_f;
  int32_t K;
  const void* P[LQ_MAX_DIMS];      // projected tables [r_k x l_1]
  int64_t ldp[LQ_MAX_DIMS];
  int64_t prows[LQ_MAX_DIMS];      // r_k
  const int32_t* fk[LQ_MAX_DIMS];
  int32_t n_layers;
  const void* W[LQ_MAX_LAYERS];    // W[0] only rows [0, c_f) are used by the fused kernels
  int64_t ldw[LQ_MAX_LAYERS];
  int32_t win[LQ_MAX_LAYERS];
  int32_t wout[LQ_MAX_LAYERS];
  const void* bias[LQ_MAX_LAYERS];
  void* Y;
  int64_t ldy;
  int32_t x_dtype;  // dtype of X, W, bias
  int32_t p_dtype;
  int32_t y_dtype;
  int32_t relu_linear;   // a one-layer call stores max(z, 0): the first layer of a model whose later layers run as dense
                         // products (honoured by the wide row-batch, column-tiled and shape-agnostic kernels only)
  int32_t accumulate_y;  // a one-layer call adds what Y already holds to z (x W_f + b_1 put there by a dense product when the
                         // fact table has more columns of its own than the kernel takes); same three kernels
  int32_t probe;         // a specialised kernel that would take the shape returns LQ_OK without launching
};

// Kernel launchers implemented in the .hip files.  Each returns an lq_status.
int launch_project_dims(const lq_mat& D, const lq_mat& W, int32_t row_off, const lq_mat& P,
                        hipStream_t s);
int launch_project_dims_all(int32_t K, const lq_mat* D, const lq_mat& W, int32_t first_off, const lq_mat* P,
                            hipStream_t s);
int launch_fused(const PredictArgs& a, hipStream_t s);
int launch_materialize(const lq_star& star, void* T, int64_t ldt, int64_t row0, int64_t rows,
                       hipStream_t s);
int launch_check_fks(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                     bool negative_ok, int32_t* d_flag, hipStream_t s);
int launch_check_codes(int32_t K, const int64_t* rows, const uint8_t* const* mask, const int32_t* const* code,
                       const int32_t* card, int32_t* d_flag, hipStream_t s);
int launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);

// ---- device side -------------------------------------------------------------------------
#ifdef __HIPCC__

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

// Round to nearest even; NaN stays NaN (quiet).
typedef __bf16 lq_bf16x2 __attribute__((ext_vector_type(2)));
typedef float lq_f32x2 __attribute__((ext_vector_type(2)));
// Two floats rounded to bf16 (to nearest, ties to even; NaN stays NaN), `lo` in bits 0..15 of the result:
// the hardware's packed conversion, one instruction.
__device__ __forceinline__ unsigned int f32x2_to_bf16x2(float lo, float hi) {
  return __builtin_bit_cast(unsigned int, __builtin_convertvector((lq_f32x2){lo, hi}, lq_bf16x2));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return static_cast<bf16_t>(f32x2_to_bf16x2(f, 0.f) & 0xffffu);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Load element i of an array whose element type is only known at run time.
__device__ __forceinline__ float load_as_f32(const void* base, int64_t i, int32_t dtype) {
  return dtype == LQ_BF16 ? bf16_to_f32(static_cast<const bf16_t*>(base)[i])
                          : static_cast<const float*>(base)[i];
}
__device__ __forceinline__ void store_from_f32(void* base, int64_t i, int32_t dtype, float v) {
  if (dtype == LQ_BF16) static_cast<bf16_t*>(base)[i] = f32_to_bf16(v);
  else static_cast<float*>(base)[i] = v;
}

#endif  // __HIPCC__
}  // namespace lq
#endif  // LQ_COMMON_H_
