// Join-computation stage (last line of Eq. 1) for wide bf16 models: hidden width a multiple of
// 32, up to 16 fact-owned columns, optional second layer of at most 16 outputs on the matrix cores.
//
// A wavefront handles 16 fact rows per pass.  Lane (g = lane / 16, j = lane % 16) works on row j
// and, in each 32-wide block kb of hidden units, owns units 32 kb + 8 g .. + 7 - exactly the
// eight bf16 values one lane supplies as the K-slice of the B operand of the 16x16x32 bf16 MFMA.
// So the gathered rows are summed in fp32 in place, rectified, rounded to bf16 once and fed to the
// MFMA without any cross-lane movement:  Y^T[16 outputs x 16 rows] = W_2^T [16 x l_1] * H^T.
// The four lanes of a row read 64 contiguous bytes of each projected row per load.
#include "lq_common.h"

namespace lq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int BF_THREADS = 256;

__device__ __forceinline__ void unpack_add(const v4u& w, float (&acc)[8]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    acc[2 * q] += __uint_as_float(w[q] << 16);
    acc[2 * q + 1] += __uint_as_float(w[q] & 0xffff0000u);
  }
}
__device__ __forceinline__ unsigned int pack2(float lo, float hi) {
  return f32x2_to_bf16x2(lo, hi);
}

// KB = l_1 / 32.  NL = 1: Y = z (TY = bf16 or float).  NL = 2: Y = W_2^T relu(z) + b_2, l_2 <= 16.
// HAS_X: the fact table has columns of its own.
template <int KB, int NL, typename TY, bool HAS_X>
__global__ __launch_bounds__(BF_THREADS) void fused_bf16_kernel(PredictArgs a) {
  const int lane = threadIdx.x & 63, g = lane >> 4, j = lane & 15;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (BF_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (BF_THREADS / 64);
  const int64_t npass = (a.n + 15) / 16;
  const int l2 = NL == 2 ? a.wout[1] : 0;
  // The fact term's rows of W_0 (up to 16 of them) are staged in LDS once: read from memory in every pass they went
  // through the address path the gathers need (linear 256 with 12 fact columns: 0.64 ms per 1e6 rows against 0.21 without).
  __shared__ __align__(16) bf16_t wf_lds[HAS_X ? 16 * 32 * KB : 8];
  if constexpr (HAS_X) {
    for (int i = threadIdx.x; i < a.c_f * 32 * KB; i += BF_THREADS)
      wf_lds[i] = static_cast<const bf16_t*>(a.W[0])[static_cast<int64_t>(i / (32 * KB)) * a.ldw[0] + i % (32 * KB)];
    __syncthreads();
  }

  // A operand of the second layer: lane (g, i = j) holds W_2[32 kb + 8 g + t][i], t = 0..7.
  v4u afrag[NL == 2 ? KB : 1];
  float b2[4] = {0.f, 0.f, 0.f, 0.f};
  if constexpr (NL == 2) {
    const bf16_t* W1 = static_cast<const bf16_t*>(a.W[1]);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      unsigned int h[8];
#pragma unroll
      for (int t = 0; t < 8; ++t)
        h[t] = j < l2 ? W1[static_cast<int64_t>(32 * kb + 8 * g + t) * a.ldw[1] + j] : 0u;
      afrag[kb] = (v4u){h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    }
    if (a.bias[1])
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (4 * g + v < l2) b2[v] = bf16_to_f32(static_cast<const bf16_t*>(a.bias[1])[4 * g + v]);
  }

  for (int64_t pass = wave; pass < npass; pass += nwaves) {
    const int64_t row = pass * 16 + j;
    const bool live = row < a.n;
    const int64_t rr = live ? row : a.n - 1;

    float acc[KB][8];
    if (a.bias[0]) {
      const bf16_t* b1 = static_cast<const bf16_t*>(a.bias[0]);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[kb][t] = bf16_to_f32(b1[32 * kb + 8 * g + t]);
    } else {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[kb][t] = 0.f;
    }
    if constexpr (HAS_X) {                 // the fact table's own columns: z += x W_f, weights from LDS
      const bf16_t* xr = static_cast<const bf16_t*>(a.X) + rr * a.ldx;
      const bf16_t* wf = wf_lds + 8 * g;
      for (int q = 0; q < a.c_f; ++q) {
        const float x = bf16_to_f32(xr[q]);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const v4u t = *reinterpret_cast<const v4u*>(wf + (q * KB + kb) * 32);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[kb][2 * e] = fmaf(x, __uint_as_float(t[e] << 16), acc[kb][2 * e]);
            acc[kb][2 * e + 1] = fmaf(x, __uint_as_float(t[e] & 0xffff0000u), acc[kb][2 * e + 1]);
          }
        }
      }
    }
    for (int k = 0; k < a.K; ++k) {
      const int64_t f = a.fk[k][rr];
      const bf16_t* p = static_cast<const bf16_t*>(a.P[k]) + f * a.ldp[k] + 8 * g;
      v4u w[KB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) w[kb] = *reinterpret_cast<const v4u*>(p + 32 * kb);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) unpack_add(w[kb], acc[kb]);
    }

    if constexpr (NL == 1) {
      if (live) {
        TY* yr = static_cast<TY*>(a.Y) + row * a.ldy + 8 * g;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          if constexpr (sizeof(TY) == 2) {
            const v4u o = {pack2(acc[kb][0], acc[kb][1]), pack2(acc[kb][2], acc[kb][3]),
                           pack2(acc[kb][4], acc[kb][5]), pack2(acc[kb][6], acc[kb][7])};
            *reinterpret_cast<v4u*>(yr + 32 * kb) = o;
          } else {
            *reinterpret_cast<v4f*>(yr + 32 * kb) = (v4f){acc[kb][0], acc[kb][1], acc[kb][2], acc[kb][3]};
            *reinterpret_cast<v4f*>(yr + 32 * kb + 4) = (v4f){acc[kb][4], acc[kb][5], acc[kb][6], acc[kb][7]};
          }
        }
      }
    } else {
      v4f out = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const v4u hb = {pack2(fmaxf(acc[kb][0], 0.f), fmaxf(acc[kb][1], 0.f)),
                        pack2(fmaxf(acc[kb][2], 0.f), fmaxf(acc[kb][3], 0.f)),
                        pack2(fmaxf(acc[kb][4], 0.f), fmaxf(acc[kb][5], 0.f)),
                        pack2(fmaxf(acc[kb][6], 0.f), fmaxf(acc[kb][7], 0.f))};
        out = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, afrag[kb]),
                                                      __builtin_bit_cast(bf16x8, hb), out, 0, 0, 0);
      }
      // register v of lane (g, j) is output 4 g + v of row j
      if (live) {
        TY* yr = static_cast<TY*>(a.Y) + row * a.ldy;
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (4 * g + v < l2) Elem<TY>::store(yr + 4 * g + v, out[v] + b2[v]);
      }
    }
  }
}

template <int KB, int NL, typename TY>
int launch_inst(const PredictArgs& a, hipStream_t s) {
  const int64_t npass = (a.n + 15) / 16;
  const int64_t blocks = std::min<int64_t>((npass + 3) / 4, static_cast<int64_t>(num_cus()) * 8);
  const dim3 grid(static_cast<unsigned>(blocks)), block(BF_THREADS);
  if (a.probe) return LQ_OK;
  if (a.c_f > 0) hipLaunchKernelGGL((fused_bf16_kernel<KB, NL, TY, true>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((fused_bf16_kernel<KB, NL, TY, false>), grid, block, 0, s, a);
  LQ_LAUNCH_CHECK("fused_bf16_kernel");
  return LQ_OK;
}

template <int KB>
int pick(const PredictArgs& a, hipStream_t s) {
  if (a.n_layers == 1)
    return a.y_dtype == LQ_BF16 ? launch_inst<KB, 1, bf16_t>(a, s) : launch_inst<KB, 1, float>(a, s);
  return a.y_dtype == LQ_BF16 ? launch_inst<KB, 2, bf16_t>(a, s) : launch_inst<KB, 2, float>(a, s);
}

}  // namespace

// Returns -1 when the shape is not one this kernel covers.
int try_fused_bf16(const PredictArgs& a, hipStream_t s) {
  if (a.x_dtype != LQ_BF16 || a.p_dtype != LQ_BF16) return -1;
  if (a.c_f > 16 || a.K < 1 || a.n_layers > 2) return -1;
  const int l1 = a.wout[0];
  if (l1 % 32 || l1 > 256) return -1;
  if (a.n_layers == 2 && a.wout[1] > 16) return -1;
  if (a.n_layers == 2 && a.wout[1] > 4 && a.c_f > 0) {
    // With fact columns the kernel for deeper bf16 models, which is tried next and keeps the fact term's weights in LDS,
    // is 1.3 to 1.8 times faster on these (256 -> 16 with 4 fact columns 0.44 -> 0.25 ms per 1e6 rows); it counts the
    // 16-byte pieces of a table in 32 bits.
    bool deep_takes = true;
    for (int k = 0; k < a.K; ++k) deep_takes = deep_takes && a.prows[k] * (a.ldp[k] / 8) <= 0xffffffffLL;
    if (deep_takes) return -1;
  }
  for (int k = 0; k < a.K; ++k)
    if (!aligned(a.P[k], 16) || a.ldp[k] % 8) return -1;
  if (a.n_layers == 1) {
    const size_t ys = dtype_size(a.y_dtype);
    if (!aligned(a.Y, 16) || (a.ldy * ys) % 16) return -1;
  }
  switch (l1 / 32) {
    case 1: return pick<1>(a, s);
    case 2: return pick<2>(a, s);
    case 4: return pick<4>(a, s);
    case 8: return pick<8>(a, s);
    default: return -1;
  }
}

}  // namespace lq
