// Yardsticks for the benchmarks: what this GPU delivers for the two access patterns the join stage is made
// of, measured without any of the method's arithmetic.  Not part of the method.
//   yard_stream_kernel  reads a buffer several times in one launch (a buffer that fits the 256 MB Infinity
//                       Cache gives that cache's rate, a large one the plain HBM read rate) and, in the same
//                       launch, writes another one: a pure stream with the read : write mix of a kernel
//   yard_gather_kernel  random row gathers from a table (row = 16 .. 1024 bytes, fetched by adjacent lanes as
//                       one contiguous run, eight rows in flight per lane), row numbers either hashed from
//                       the gather's index (no other traffic at all) or read from a key column
// Both fold what they read into a register and store it only under a condition that never holds, so that
// the loads cannot be removed and nothing is written.
#include "lq_common.h"

namespace lq {
namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix32(uint32_t x) {   // integer finaliser: spreads consecutive indices
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// One workgroup reads one 16 KB chunk (four 16-byte pieces per thread, the workgroup's loads contiguous), or
// writes one when its number lies past the read chunks; workgroups sweep memory in launch order.  Pass r reads
// chunk (c + 5 r) mod chunks from the workgroup that read chunk c in pass 0: workgroups are dealt to the eight
// XCDs in turn, so from pass to pass every chunk moves to another XCD and a buffer larger than one L2 is not
// served by the L2 that happened to keep its eighth of it.
constexpr int YARD_CHUNK16 = 1024;   // 16-byte pieces per chunk

__global__ __launch_bounds__(256) void yard_stream_kernel(const v4u* __restrict__ buf, int64_t n16, int64_t chunks,
                                                          int64_t read_blocks, v4u* __restrict__ wbuf, int64_t w16, v4u* sink) {
  const int64_t b = blockIdx.x;
  if (b >= read_blocks) {                                    // write part: zeros
    const int64_t base = (b - read_blocks) * YARD_CHUNK16 + threadIdx.x;
    const v4u z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < w16) __builtin_nontemporal_store(z, wbuf + base + u * 256);
    return;
  }
  const int64_t pass = b / chunks, c = (b % chunks + 5 * pass) % chunks;
  const int64_t base = c * YARD_CHUNK16 + threadIdx.x;
  v4u acc = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (base + u * 256 < n16) acc ^= buf[base + u * 256];
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0xf39cc060u && acc[3] == 0x5cedc834u) sink[0] = acc;
}

// LPR lanes fetch one row; a wavefront step gathers 64 / LPR rows per load instruction, 8 instructions in flight.
template <int LPR>
__global__ __launch_bounds__(256) void yard_gather_kernel(const v4u* __restrict__ table, uint32_t rows, int64_t n,
                                                          const int32_t* __restrict__ keys, uint32_t seed, v4u* sink) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, c = lane % LPR, sub = lane / LPR;
  const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = (static_cast<int64_t>(gridDim.x) * blockDim.x) >> 6;
  v4u acc = {0u, 0u, 0u, 0u};
  for (int64_t g0 = wave * (8 * RPW); g0 < n; g0 += nwaves * (8 * RPW)) {
    v4u p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int64_t g = g0 + u * RPW + sub;
      if (g >= n) g = n - 1;
      uint32_t row;
      if (keys) row = static_cast<uint32_t>(keys[g]);
      else row = static_cast<uint32_t>((static_cast<uint64_t>(mix32(static_cast<uint32_t>(g) + seed)) * rows) >> 32);
      p[u] = table[static_cast<int64_t>(row) * LPR + c];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= p[u];
  }
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0xf39cc060u && acc[3] == 0x5cedc834u) sink[0] = acc;
}

}  // namespace

typedef float v4f_y __attribute__((ext_vector_type(4)));

// Per iteration: 16 fp32 16x16x4 matrix instructions on four accumulators, then NV independent vector
// multiply-adds on eight registers.  Timed for NV = 0 and NV > 0 at the same occupancy, it shows how much
// of the vector work the matrix instructions of the same and of the other wavefronts of a SIMD hide.
template <int NV>
__global__ __launch_bounds__(256) void yard_matrix_kernel(float* sink, int iters, float a0, float b0) {
  v4f_y acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = v4f_y{0.f, 0.f, 0.f, 0.f};
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = a0 * i + threadIdx.x;
  const float a = a0 + threadIdx.x, b = b0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r & 3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[r & 3], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int v = 0; v < NV; ++v) x[v & 7] = fmaf(x[v & 7], b, a);
    __builtin_amdgcn_sched_barrier(0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) t += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
#pragma unroll
  for (int i = 0; i < 8; ++i) t += x[i];
  sink[static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x] = t;
}

}  // namespace lq

using namespace lq;

extern "C" {

int lq_yardstick_stream(const void* buf, size_t bytes, int32_t repeats, void* wbuf, size_t wbytes, void* sink,
                        void* hip_stream) {
  clear_error();
  if (!sink || (bytes && !buf) || (wbytes && !wbuf)) return fail(LQ_ERR_NULL, "a buffer or sink is NULL");
  if (!aligned(buf, 16) || !aligned(wbuf, 16) || !aligned(sink, 16) || bytes % 16 || wbytes % 16 || repeats < 1)
    return fail(LQ_ERR_SHAPE, "stream yardstick needs 16-byte aligned pointers, sizes that are multiples of 16 and repeats >= 1");
  const int64_t n16 = static_cast<int64_t>(bytes / 16), w16 = static_cast<int64_t>(wbytes / 16);
  const int64_t chunks = (n16 + YARD_CHUNK16 - 1) / YARD_CHUNK16;
  const int64_t read_blocks = chunks * repeats, write_blocks = (w16 + YARD_CHUNK16 - 1) / YARD_CHUNK16;
  if (read_blocks + write_blocks == 0) return LQ_OK;
  if (read_blocks + write_blocks > 0x7fffffffLL) return fail(LQ_ERR_UNSUPPORTED, "stream yardstick: too many chunks for one launch");
  hipLaunchKernelGGL(yard_stream_kernel, dim3(static_cast<unsigned>(read_blocks + write_blocks)), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const v4u*>(buf), n16, std::max<int64_t>(chunks, 1),
                     read_blocks, static_cast<v4u*>(wbuf), w16, static_cast<v4u*>(sink));
  LQ_LAUNCH_CHECK("yard_stream_kernel");
  return LQ_OK;
}

int lq_yardstick_read(const void* buf, size_t bytes, int32_t repeats, void* sink, void* hip_stream) {
  if (bytes == 0) { clear_error(); return fail(LQ_ERR_SHAPE, "read yardstick needs a non-empty buffer"); }
  return lq_yardstick_stream(buf, bytes, repeats, nullptr, 0, sink, hip_stream);
}

int lq_yardstick_gather(const void* table, int64_t rows, int32_t row_bytes, int64_t n_gathers, const int32_t* keys,
                        uint32_t seed, void* sink, void* hip_stream) {
  clear_error();
  if (!table || !sink) return fail(LQ_ERR_NULL, "table or sink is NULL");
  if (!aligned(table, 16) || !aligned(sink, 16) || !aligned(keys, 4)) return fail(LQ_ERR_SHAPE, "misaligned pointer");
  if (rows < 1 || rows > 0x7fffffffLL || n_gathers < 1) return fail(LQ_ERR_SHAPE, "rows or n_gathers out of range");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t blocks = static_cast<int64_t>(num_cus()) * 16;
  const v4u* t = static_cast<const v4u*>(table);
  v4u* k = static_cast<v4u*>(sink);
  const uint32_t r = static_cast<uint32_t>(rows);
#define LQ_YG(L) hipLaunchKernelGGL(yard_gather_kernel<L>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, t, r, n_gathers, keys, seed, k)
  switch (row_bytes) {
    case 16: LQ_YG(1); break;
    case 32: LQ_YG(2); break;
    case 64: LQ_YG(4); break;
    case 128: LQ_YG(8); break;
    case 256: LQ_YG(16); break;
    case 512: LQ_YG(32); break;
    case 1024: LQ_YG(64); break;
    default: return fail(LQ_ERR_SHAPE, "row_bytes must be a power of two from 16 to 1024");
  }
#undef LQ_YG
  LQ_LAUNCH_CHECK("yard_gather_kernel");
  return LQ_OK;
}

int lq_yardstick_matrix(int32_t vector_ops, int32_t waves_per_simd, int32_t iters, void* sink, size_t sink_bytes,
                        void* hip_stream) {
  clear_error();
  if (!sink) return fail(LQ_ERR_NULL, "sink is NULL");
  if (waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) return fail(LQ_ERR_SHAPE, "waves_per_simd must be 1..8, iters >= 1");
  const int64_t blocks = static_cast<int64_t>(num_cus()) * waves_per_simd;     // 256 threads: one wavefront per SIMD
  if (sink_bytes < static_cast<size_t>(blocks) * 256 * sizeof(float))
    return fail(LQ_ERR_SHAPE, "matrix yardstick: sink needs %lld bytes", (long long)(blocks * 256 * sizeof(float)));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
#define LQ_YM(NV) hipLaunchKernelGGL(yard_matrix_kernel<NV>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, \
                                     static_cast<float*>(sink), iters, 1.0f, 0.5f)
  switch (vector_ops) {
    case 0: LQ_YM(0); break;
    case 32: LQ_YM(32); break;
    case 64: LQ_YM(64); break;
    case 128: LQ_YM(128); break;
    default: return fail(LQ_ERR_SHAPE, "vector_ops must be 0, 32, 64 or 128");
  }
#undef LQ_YM
  LQ_LAUNCH_CHECK("yard_matrix_kernel");
  return LQ_OK;
}

}  // extern "C"
