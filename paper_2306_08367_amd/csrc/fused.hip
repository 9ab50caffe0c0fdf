// Join-computation stage with the model fused in (last line of Eq. 1):
//   z_i = x_i W_f + sum_k P_k[fk_k[i], :] + b_1,  then ReLU / later layers.
// The joined table is never formed; each fact row gathers one l_1-wide row from
// every projected dimension table and adds them up.
//
// Two kernels live here:
//   fused_vec_kernel      - the fast path.  A fact row is owned by a group of LPR
//                           adjacent lanes, each holding VEC consecutive hidden
//                           columns, so every gather is one 16-byte (or 4-byte)
//                           load per lane and a row of P_k is read as one
//                           contiguous run by its lane group.  W_f, b_1 and the
//                           lane's slice of W_2 sit in registers.
//   fused_generic_kernel  - any shape: a workgroup stages R rows of z in LDS and
//                           walks the remaining layers there.
#include "lq_common.h"

namespace lq {
namespace {

// ------------------------------------------------------------------ generic ------------

constexpr int GEN_THREADS = 256;

__global__ __launch_bounds__(GEN_THREADS) void fused_generic_kernel(PredictArgs a, int R, int maxw) {
  extern __shared__ float lds[];
  float* cur = lds;
  float* nxt = lds + static_cast<size_t>(R) * maxw;
  const int tid = threadIdx.x;
  const int l1 = a.wout[0];
  const int64_t n_tiles = (a.n + R - 1) / R;
  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int64_t base = tile * R;
    const int rows = static_cast<int>(min(static_cast<int64_t>(R), a.n - base));
    const bool last0 = a.n_layers == 1;
    for (int idx = tid; idx < rows * l1; idx += GEN_THREADS) {
      const int r = idx / l1, j = idx - r * l1;
      const int64_t row = base + r;
      float acc = 0.f;
      for (int q = 0; q < a.c_f; ++q)
        acc += load_as_f32(a.X, row * a.ldx + q, a.x_dtype) *
               load_as_f32(a.W[0], static_cast<int64_t>(q) * a.ldw[0] + j, a.x_dtype);
      for (int k = 0; k < a.K; ++k)
        acc += load_as_f32(a.P[k], static_cast<int64_t>(a.fk[k][row]) * a.ldp[k] + j, a.p_dtype);
      if (a.bias[0]) acc += load_as_f32(a.bias[0], j, a.x_dtype);
      if (last0) {
        if (a.accumulate_y) acc += load_as_f32(a.Y, row * a.ldy + j, a.y_dtype);
        store_from_f32(a.Y, row * a.ldy + j, a.y_dtype, a.relu_linear ? fmaxf(acc, 0.f) : acc);
      }
      else cur[r * maxw + j] = fmaxf(acc, 0.f);
    }
    for (int layer = 1; layer < a.n_layers; ++layer) {
      __syncthreads();
      const int win = a.win[layer], wout = a.wout[layer];
      const bool last = layer == a.n_layers - 1;
      for (int idx = tid; idx < rows * wout; idx += GEN_THREADS) {
        const int r = idx / wout, o = idx - r * wout;
        float acc = 0.f;
        for (int q = 0; q < win; ++q)
          acc += cur[r * maxw + q] *
                 load_as_f32(a.W[layer], static_cast<int64_t>(q) * a.ldw[layer] + o, a.x_dtype);
        if (a.bias[layer]) acc += load_as_f32(a.bias[layer], o, a.x_dtype);
        if (last) store_from_f32(a.Y, (base + r) * a.ldy + o, a.y_dtype, acc);
        else nxt[r * maxw + o] = fmaxf(acc, 0.f);
      }
      float* t = cur; cur = nxt; nxt = t;
    }
    __syncthreads();
  }
}

int launch_generic(const PredictArgs& a, hipStream_t s) {
  int maxw = 1;
  for (int j = 0; j + 1 < a.n_layers; ++j) maxw = std::max(maxw, a.wout[j]);
  int R = 16;
  while (R > 1 && static_cast<size_t>(2) * R * maxw * sizeof(float) > 64 * 1024) R >>= 1;
  const size_t lds = static_cast<size_t>(2) * R * maxw * sizeof(float);
  if (lds > 64 * 1024)
    return fail(LQ_ERR_UNSUPPORTED, "hidden width %d is too wide for the generic kernel", maxw);
  const int64_t n_tiles = (a.n + R - 1) / R;
  const int64_t blocks = std::min<int64_t>(n_tiles, static_cast<int64_t>(num_cus()) * 8);
  if (blocks <= 0) return LQ_OK;
  hipLaunchKernelGGL(fused_generic_kernel, dim3(static_cast<unsigned>(blocks)), dim3(GEN_THREADS),
                     lds, s, a, R, maxw);
  LQ_LAUNCH_CHECK("fused_generic_kernel");
  return LQ_OK;
}

// ------------------------------------------------------------------ vectorised ----------

// VEC consecutive elements of type T as one load.
template <typename T, int VEC> struct Chunk;
template <> struct Chunk<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    typedef float v4f_ __attribute__((ext_vector_type(4)));
    const v4f_ t = {v[0], v[1], v[2], v[3]};
    __builtin_nontemporal_store(t, reinterpret_cast<v4f_*>(p));   // written once, never re-read here
  }
};
template <> struct Chunk<float, 2> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[2]) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[2]) {
    *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
  }
};
template <> struct Chunk<float, 1> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[1]) { v[0] = *p; }
  static __device__ __forceinline__ void store(float* p, const float (&v)[1]) { *p = v[0]; }
};
template <> struct Chunk<bf16_t, 8> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v[2 * q] = __uint_as_float(w[q] << 16);
      v[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
      w[q] = f32x2_to_bf16x2(v[2 * q], v[2 * q + 1]);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};
template <> struct Chunk<bf16_t, 1> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[1]) { v[0] = bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[1]) { *p = f32_to_bf16(v[0]); }
};

constexpr int VEC_THREADS = 256;

template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over groups of LPR adjacent lanes (LPR a power of two), result in every lane of the group.
// Steps inside a 16-lane DPP row are DPP adds (quad permutes, half-row and row mirrors); only the
// steps across DPP rows go through the cross-lane network.
template <int LPR> __device__ __forceinline__ float group_allreduce(float y) {
  if (LPR >= 2) y += dpp_f<0xB1>(y);     // quad_perm [1,0,3,2]
  if (LPR >= 4) y += dpp_f<0x4E>(y);     // quad_perm [2,3,0,1]
  if (LPR >= 8) y += dpp_f<0x141>(y);    // row_half_mirror
  if (LPR >= 16) y += dpp_f<0x140>(y);   // row_mirror
  if (LPR >= 32) y += __shfl_xor(y, 16, 64);
  if (LPR >= 64) y += __shfl_xor(y, 32, 64);
  return y;
}

// TX: dtype of X / W / bias, TP: dtype of P, TY: dtype of Y.
// LPR lanes per fact row (power of two, <= 64), VEC hidden columns per lane: l_1 <= LPR * VEC, l_1 a
// multiple of VEC; lanes whose slice starts at or beyond l_1 idle (zero weights, no loads, no stores).
// CF: compile-time bound on c_f (fact columns beyond the real c_f count as zero).
// NL: 1 (linear) or 2 (ReLU then W_2 with L2 outputs).
template <typename TX, typename TP, typename TY, int VEC, int LPR, int CF, int NL, int L2, bool XV>
__global__ __launch_bounds__(VEC_THREADS) void fused_vec_kernel(PredictArgs a) {
  constexpr int RPW = 64 / LPR;                 // fact rows per wavefront pass
  constexpr int RPB = RPW * (VEC_THREADS / 64); // per workgroup pass
  const int tid = threadIdx.x;
  const int sub = tid / LPR;                    // which row of the workgroup pass
  const int c = tid % LPR;                      // which VEC-wide column slice
  const int col0 = c * VEC;
  const bool active = col0 < a.wout[0];

  const TX* __restrict__ X = static_cast<const TX*>(a.X);
  const TX* __restrict__ W0 = static_cast<const TX*>(a.W[0]);

  float wf[CF > 0 ? CF : 1][VEC];
#pragma unroll
  for (int q = 0; q < CF; ++q)
#pragma unroll
    for (int v = 0; v < VEC; ++v)
      wf[q][v] = (active && q < a.c_f) ? Elem<TX>::load(W0 + static_cast<int64_t>(q) * a.ldw[0] + col0 + v) : 0.f;
  float b1[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v)
    b1[v] = (active && a.bias[0]) ? Elem<TX>::load(static_cast<const TX*>(a.bias[0]) + col0 + v) : 0.f;

  float w2[NL == 2 ? VEC : 1][NL == 2 ? L2 : 1];
  float b2[NL == 2 ? L2 : 1];
  if (NL == 2) {
    const TX* __restrict__ W1 = static_cast<const TX*>(a.W[1]);
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int o = 0; o < L2; ++o)
        w2[v][o] = active ? Elem<TX>::load(W1 + static_cast<int64_t>(col0 + v) * a.ldw[1] + o) : 0.f;
#pragma unroll
    for (int o = 0; o < L2; ++o)
      b2[o] = a.bias[1] ? Elem<TX>::load(static_cast<const TX*>(a.bias[1]) + o) : 0.f;
  }

  const int64_t n_pass = (a.n + RPB - 1) / RPB;
  for (int64_t pass = blockIdx.x; pass < n_pass; pass += gridDim.x) {
    const int64_t row = pass * RPB + sub;
    const bool live = row < a.n;
    const int64_t rr = live ? row : a.n - 1;    // dead lanes redo the last row, store nothing

    float z[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) z[v] = b1[v];
    if (CF > 0) {
      const TX* xr = X + rr * a.ldx;
      float xq[CF > 0 ? CF : 1];
      if constexpr (XV) {   // fp32 fact columns in 16-byte pieces
#pragma unroll
        for (int q = 0; q < CF; q += 4) {
          const float4 t = *reinterpret_cast<const float4*>(xr + q);
          xq[q] = t.x; xq[q + 1] = t.y; xq[q + 2] = t.z; xq[q + 3] = t.w;
        }
      } else {
#pragma unroll
        for (int q = 0; q < CF; ++q) xq[q] = q < a.c_f ? Elem<TX>::load(xr + q) : 0.f;
      }
#pragma unroll
      for (int q = 0; q < CF; ++q)
#pragma unroll
        for (int v = 0; v < VEC; ++v) z[v] = fmaf(xq[q], wf[q][v], z[v]);
    }
    for (int k = 0; k < a.K; ++k) {
      const int64_t j = __builtin_nontemporal_load(a.fk[k] + rr);   // keys are read once: do not let them displace table rows in cache
      if (active) {
        float p[VEC];
        Chunk<TP, VEC>::load(static_cast<const TP*>(a.P[k]) + j * a.ldp[k] + col0, p);
#pragma unroll
        for (int v = 0; v < VEC; ++v) z[v] += p[v];
      }
    }

    if (NL == 1) {
      if (live && active) Chunk<TY, VEC>::store(static_cast<TY*>(a.Y) + row * a.ldy + col0, z);
    } else {
      float y[L2];
#pragma unroll
      for (int o = 0; o < L2; ++o) y[o] = 0.f;
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const float h = fmaxf(z[v], 0.f);
#pragma unroll
        for (int o = 0; o < L2; ++o) y[o] = fmaf(h, w2[v][o], y[o]);
      }
#pragma unroll
      for (int o = 0; o < L2; ++o) y[o] = group_allreduce<LPR>(y[o]);
      if (live && c == 0) {
        TY* yr = static_cast<TY*>(a.Y) + row * a.ldy;
#pragma unroll
        for (int o = 0; o < L2; ++o) Elem<TY>::store(yr + o, y[o] + b2[o]);
      }
    }
  }
}

template <typename TX, typename TP, typename TY, int VEC, int LPR, int CF, int NL, int L2>
int launch_vec_inst(const PredictArgs& a, hipStream_t s) {
  constexpr int RPB = (64 / LPR) * (VEC_THREADS / 64);
  const int64_t n_pass = (a.n + RPB - 1) / RPB;
  // One pass per workgroup: workgroups then sweep the fact table in launch order, which streams
  // from HBM measurably faster than a strided persistent loop.
  const int64_t blocks = std::min<int64_t>(n_pass, 0x7fffffffLL);
  if (blocks <= 0 || a.probe) return LQ_OK;
  constexpr bool can_xv = sizeof(TX) == 4 && CF > 0 && CF % 4 == 0;
  if (can_xv && a.c_f == CF && aligned(a.X, 16) && a.ldx % 4 == 0)
    hipLaunchKernelGGL((fused_vec_kernel<TX, TP, TY, VEC, LPR, CF, NL, L2, can_xv>),
                       dim3(static_cast<unsigned>(blocks)), dim3(VEC_THREADS), 0, s, a);
  else
    hipLaunchKernelGGL((fused_vec_kernel<TX, TP, TY, VEC, LPR, CF, NL, L2, false>),
                       dim3(static_cast<unsigned>(blocks)), dim3(VEC_THREADS), 0, s, a);
  LQ_LAUNCH_CHECK("fused_vec_kernel");
  return LQ_OK;
}

// Run-time -> compile-time dispatch.  Returns -1 when no instantiation fits.
template <typename TX, typename TP, typename TY, int VEC, int LPR, int CF>
int pick_layers(const PredictArgs& a, hipStream_t s) {
  if (a.n_layers == 1) return launch_vec_inst<TX, TP, TY, VEC, LPR, CF, 1, 1>(a, s);
  if (a.n_layers == 2) {
    switch (a.wout[1]) {
      case 1: return launch_vec_inst<TX, TP, TY, VEC, LPR, CF, 2, 1>(a, s);
      case 2: return launch_vec_inst<TX, TP, TY, VEC, LPR, CF, 2, 2>(a, s);
      case 4: return launch_vec_inst<TX, TP, TY, VEC, LPR, CF, 2, 4>(a, s);
      default: return -1;
    }
  }
  return -1;
}

template <typename TX, typename TP, typename TY, int VEC, int LPR>
int pick_cf(const PredictArgs& a, hipStream_t s) {
  if (a.c_f == 0) return pick_layers<TX, TP, TY, VEC, LPR, 0>(a, s);
  if (a.c_f <= 4) return pick_layers<TX, TP, TY, VEC, LPR, 4>(a, s);
  if (a.c_f <= 8) return pick_layers<TX, TP, TY, VEC, LPR, 8>(a, s);
  if (a.c_f <= 16) return pick_layers<TX, TP, TY, VEC, LPR, 16>(a, s);
  return -1;
}

template <typename TX, typename TP, typename TY, int VEC>
int pick_lpr(const PredictArgs& a, hipStream_t s) {
  const int l1 = a.wout[0];
  if (l1 % VEC) return -1;
  const int chunks = l1 / VEC;
  if (chunks <= 1) return pick_cf<TX, TP, TY, VEC, 1>(a, s);
  if (chunks <= 2) return pick_cf<TX, TP, TY, VEC, 2>(a, s);
  if (chunks <= 4) return pick_cf<TX, TP, TY, VEC, 4>(a, s);
  if (chunks <= 8) return pick_cf<TX, TP, TY, VEC, 8>(a, s);
  if (chunks <= 16) return pick_cf<TX, TP, TY, VEC, 16>(a, s);
  if (chunks <= 32) return pick_cf<TX, TP, TY, VEC, 32>(a, s);
  if (chunks <= 64) return pick_cf<TX, TP, TY, VEC, 64>(a, s);
  return -1;
}

// Are vec-element chunk accesses to P and Y legal?
bool chunks_aligned(const PredictArgs& a, int vec_p, int vec_y) {
  const size_t ps = dtype_size(a.p_dtype), ys = dtype_size(a.y_dtype);
  for (int k = 0; k < a.K; ++k)
    if (!aligned(a.P[k], vec_p * ps) || a.ldp[k] % vec_p) return false;
  if (a.n_layers == 1 && (!aligned(a.Y, vec_y * ys) || a.ldy % vec_y)) return false;
  return true;
}

int try_vec(const PredictArgs& a, hipStream_t s) {
  const int l1 = a.wout[0];
  if (a.x_dtype == LQ_F32 && a.p_dtype == LQ_F32 && a.y_dtype == LQ_F32) {
    if (l1 % 4 == 0 && l1 <= 256 && chunks_aligned(a, 4, 4)) return pick_lpr<float, float, float, 4>(a, s);
    if (l1 % 2 == 0 && l1 <= 128 && chunks_aligned(a, 2, 2)) return pick_lpr<float, float, float, 2>(a, s);
    if (l1 <= 64) return pick_lpr<float, float, float, 1>(a, s);
    return -1;
  }
  if (a.x_dtype == LQ_BF16 && a.p_dtype == LQ_BF16 && a.y_dtype == LQ_BF16) {
    if (l1 % 8 == 0 && l1 <= 512 && chunks_aligned(a, 8, 8)) return pick_lpr<bf16_t, bf16_t, bf16_t, 8>(a, s);
    return -1;
  }
  return -1;
}

}  // namespace

int try_rowbatch64(const PredictArgs& a, hipStream_t s);
int try_rowbatch_wide(const PredictArgs& a, hipStream_t s);
int try_fused_bf16(const PredictArgs& a, hipStream_t s);
int try_fused_tile(const PredictArgs& a, hipStream_t s);
int try_fused_deep(const PredictArgs& a, hipStream_t s);
int try_fused_deep_bf16(const PredictArgs& a, hipStream_t s);
int try_fused_lds(const PredictArgs& a, hipStream_t s);
int try_fused_coltile(const PredictArgs& a, hipStream_t s);

int launch_linear_stage(const PredictArgs& f, hipStream_t s);
int launch_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, const void* bias, int64_t M,
                int32_t N, int32_t Kd, int relu, int32_t in_dtype, int32_t out_dtype, hipStream_t s);

int launch_fused(const PredictArgs& a, hipStream_t s) {
  if (a.n == 0) return LQ_OK;
  int rc = try_rowbatch64(a, s);
  if (rc >= 0) return rc;
  rc = try_fused_deep(a, s);          // three to eight layers, or a second layer of 5..128 outputs
  if (rc >= 0) return rc;
  rc = try_rowbatch_wide(a, s);
  if (rc >= 0) return rc;
  rc = try_fused_bf16(a, s);
  if (rc >= 0) return rc;
  rc = try_fused_deep_bf16(a, s);     // bf16: three to eight layers, a second layer of 17..256 outputs, or what the kernel above left
  if (rc >= 0) return rc;
  rc = try_fused_lds(a, s);           // linear models with 1 / 2 / 4 outputs whose small projected tables fit LDS
  if (rc >= 0) return rc;
  if (a.n_layers == 1 && a.wout[0] > 128) return launch_linear_stage(a, s);   // wide linear operators: in passes if need be
  rc = try_vec(a, s);
  if (rc >= 0) return rc;
  rc = try_fused_coltile(a, s);       // first layers wider than 256 (fp32) / 512 (bf16) columns, one or two layers
  if (rc >= 0) return rc;
  if (a.n_layers == 1) return launch_linear_stage(a, s);   // (a wide linear operator with many fact columns)
  rc = try_fused_tile(a, s);
  if (rc >= 0) return rc;
  return launch_generic(a, s);
}

// Does one of the specialised kernels take this shape?  (The per-wavefront tile kernel and the shape-agnostic
// kernel, which take anything, do not count.)  Nothing is launched.
bool fused_kernel_covers(const PredictArgs& a0) {
  PredictArgs a = a0;
  a.probe = 1;
  hipStream_t s = nullptr;
  // (the lane-group kernel does not count for first layers wider than 128: it is latency-bound there, 10.6 ms per
  // 1e6 rows at bf16 512 -> 4 with 12 fact columns against 1.5 ms in passes)
  return try_rowbatch64(a, s) >= 0 || try_fused_deep(a, s) >= 0 || try_rowbatch_wide(a, s) >= 0 || try_fused_bf16(a, s) >= 0 ||
         try_fused_deep_bf16(a, s) >= 0 || try_fused_lds(a, s) >= 0 || (a.wout[0] <= 128 && try_vec(a, s) >= 0) ||
         try_fused_coltile(a, s) >= 0;
}

int launch_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, const void* bias, int64_t M,
                int32_t N, int32_t Kd, int relu, int32_t in_dtype, int32_t out_dtype, hipStream_t s);

// Workspace bytes per 256 fact rows of the layered form below (two activation buffers as wide as the widest
// hidden layer, rows 16 bytes apart at the least).
size_t fused_layered_bytes_per_256(const PredictArgs& a) {
  const size_t es = dtype_size(a.x_dtype);
  size_t widest = 0;
  for (int j = 0; j + 1 < a.n_layers; ++j) widest = std::max(widest, round_up(static_cast<size_t>(a.wout[j]) * es, 16));
  return 2 * 256 * widest;
}

// The join stage as a linear operator (one layer, optionally with the ReLU in its store) on the kernels that take any
// width.  When the fact table has more columns of its own, or the star more tables, than they take in one go, the
// stage is cut into passes over Y: x W_f + b_1 by a dense product, then up to four tables at a time added to what Y
// holds (accumulate_y), the ReLU in the last pass only.
int launch_linear_stage(const PredictArgs& f, hipStream_t s) {
  auto wide_kernels = [&](const PredictArgs& g) {
    int rc = try_rowbatch_wide(g, s);
    if (rc < 0) rc = try_fused_coltile(g, s);
    return rc;
  };
  int rc = wide_kernels(f);
  if (rc >= 0) return rc;
  if (f.K > 0 && f.x_dtype == f.y_dtype && f.x_dtype == f.p_dtype) {
    constexpr int GROUP = 4;
    const int n_groups = (f.K + GROUP - 1) / GROUP;
    // pass p takes tables [GROUP p, GROUP p + GROUP); the fact term goes with the first pass if that pass takes it,
    // else ahead of it as a dense product
    auto pass = [&](int p, bool fact_here, bool probe) {
      PredictArgs g = f;
      g.K = std::min(GROUP, f.K - GROUP * p);
      for (int k = 0; k < g.K; ++k) {
        g.P[k] = f.P[GROUP * p + k]; g.ldp[k] = f.ldp[GROUP * p + k]; g.prows[k] = f.prows[GROUP * p + k];
        g.fk[k] = f.fk[GROUP * p + k];
      }
      const bool first = p == 0 && fact_here;
      if (!first) { g.c_f = 0; g.X = nullptr; g.bias[0] = nullptr; g.accumulate_y = 1; }
      g.relu_linear = (p == n_groups - 1) ? f.relu_linear : 0;
      g.probe = probe ? 1 : 0;
      return g;
    };
    bool fact_here = wide_kernels(pass(0, true, true)) >= 0;
    bool ok = fact_here || wide_kernels(pass(0, false, true)) >= 0;
    for (int p = 1; p < n_groups && ok; ++p) ok = wide_kernels(pass(p, fact_here, true)) >= 0;
    if (ok) {
      if (!fact_here) {
        if (f.c_f > 0) {
          rc = launch_gemm(f.X, f.ldx, f.W[0], f.ldw[0], f.Y, f.ldy, f.bias[0], f.n, f.wout[0], f.c_f, 0, f.x_dtype, f.y_dtype, s);
          if (rc) return rc;
        } else {
          fact_here = true;       // (no fact columns: the first pass carries the bias and starts Y)
        }
      }
      for (int p = 0; p < n_groups; ++p)
        if ((rc = wide_kernels(pass(p, fact_here, false)))) return rc < 0 ? fail(LQ_ERR_UNSUPPORTED, "linear stage: a pass lost its kernel") : rc;
      return LQ_OK;
    }
  }
  if (!f.relu_linear && !f.accumulate_y) {       // (the lane-group and the per-wavefront tile kernel know neither)
    rc = try_vec(f, s);
    if (rc < 0) rc = try_fused_tile(f, s);
    if (rc >= 0) return rc;
  }
  return launch_generic(f, s);
}

// Models that none of the specialised kernels takes (a wide first layer followed by a wide or a third layer, say
// 1,024 -> 1,024 or 512 -> 64 -> 1): the join stage runs as a linear operator with the ReLU in its store
// (z = x W_f + sum_k P_k[fk_k] + b_1 written once, in chunks of rows that fit the workspace), the later layers as
// dense products on the matrix cores.  Still no joined table, and the first layer's k x l_1 product stays pre-fused.
int launch_fused_layered(const PredictArgs& a, void* ws, size_t ws_bytes, hipStream_t s) {
  const size_t es = dtype_size(a.x_dtype);
  const size_t per256 = fused_layered_bytes_per_256(a);
  int64_t chunk = static_cast<int64_t>(ws_bytes / per256) * 256;
  chunk = std::min<int64_t>(chunk, static_cast<int64_t>(round_up(static_cast<size_t>(a.n), 256)));
  if (chunk < 256) return fail(LQ_ERR_WORKSPACE, "workspace too small for one 256-row chunk of the layered form");
  const size_t half = static_cast<size_t>(chunk) / 256 * (per256 / 2);
  uint8_t* buf[2] = {static_cast<uint8_t*>(ws), static_cast<uint8_t*>(ws) + half};
  for (int64_t r0 = 0; r0 < a.n; r0 += chunk) {
    const int64_t m = std::min<int64_t>(chunk, a.n - r0);
    PredictArgs f = a;
    f.n = m;
    f.X = a.X ? static_cast<const uint8_t*>(a.X) + static_cast<size_t>(r0) * a.ldx * es : nullptr;
    for (int k = 0; k < a.K; ++k) f.fk[k] = a.fk[k] + r0;
    f.n_layers = 1;
    f.relu_linear = 1;
    f.y_dtype = a.x_dtype;
    int64_t ld = static_cast<int64_t>(round_up(static_cast<size_t>(a.wout[0]) * es, 16) / es);
    f.Y = buf[0]; f.ldy = ld;
    int rc = launch_linear_stage(f, s);
    if (rc) return rc;
    int cur = 0;
    for (int j = 1; j < a.n_layers; ++j) {
      const bool last = j == a.n_layers - 1;
      void* C = last ? static_cast<void*>(static_cast<uint8_t*>(a.Y) + static_cast<size_t>(r0) * a.ldy * dtype_size(a.y_dtype))
                     : static_cast<void*>(buf[cur ^ 1]);
      const int64_t ldc = last ? a.ldy : static_cast<int64_t>(round_up(static_cast<size_t>(a.wout[j]) * es, 16) / es);
      rc = launch_gemm(buf[cur], ld, a.W[j], a.ldw[j], C, ldc, a.bias[j], m, a.wout[j], a.win[j], last ? 0 : 1, a.x_dtype,
                       last ? a.y_dtype : a.x_dtype, s);
      if (rc) return rc;
      ld = ldc;
      cur ^= 1;
    }
  }
  return LQ_OK;
}

// The tile kernel alone (testing / tuning aid), generic kernel if it does not cover the shape.
int launch_fused_tile(const PredictArgs& a, hipStream_t s) {
  if (a.n == 0) return LQ_OK;
  const int rc = try_fused_tile(a, s);
  if (rc >= 0) return rc;
  return launch_generic(a, s);
}

// The generic kernel alone (used to cross-check the fast path from the tests via a flag).
int launch_fused_generic(const PredictArgs& a, hipStream_t s) {
  if (a.n == 0) return LQ_OK;
  return launch_generic(a, s);
}

}  // namespace lq
