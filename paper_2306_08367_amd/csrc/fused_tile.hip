// Join-computation stage (last line of Eq. 1) followed by an MLP of any depth, for shapes the
// specialised kernels do not cover (wider second layers, three or more layers, hidden widths up
// to 512, fact columns with bf16 models).
//
// Every wavefront works on its own 16 fact rows at a time, with no workgroup barrier in the loop
// (measured here: many independent wavefronts hide the key -> gather latency chain better than larger
// cooperative tiles).
//   phase 1  z = x W_f + sum_k P_k[fk_k] + b_1 for the 16 rows, one 4-column piece per lane and
//            step (a projected row is read as a contiguous run by neighbouring lanes), ReLU,
//            result to the wavefront's LDS buffer in fp32.  W_f and b_1 are staged in LDS once.
//   phase 2  every further layer is a [16 x l_j] * [l_j x l_(j+1)] product on the matrix cores
//            (16x16x4 fp32 MFMA; A operand from LDS, B operand = the weights straight from cache),
//            ping-ponging between two LDS buffers when there are more than two layers; the last
//            layer is written to Y.
// bf16 inputs are widened to fp32 on load; accumulation is fp32 throughout.
#include "lq_common.h"

namespace lq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TILE_THREADS = 256;
constexpr int WAVES = TILE_THREADS / 64;
constexpr int WROWS = 16;               // fact rows per wavefront step

// Makes the LDS writes of this wavefront visible to all of its lanes.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// P4: projected tables can be read in 4-element pieces (l_1 % 4 == 0, aligned).
// XB / PB: the model (X, W, bias) / the projected tables are bf16 (else fp32).
// PIECES, KT (fp32 only): l_1 = 16 PIECES and the number of dimensions as compile-time constants, so
// that phase 1 unrolls and requests all keys, then all gathers of a step at once; 0 = run-time loops.
template <bool P4, bool XB, bool PB, int PIECES, int KT>
__global__ __launch_bounds__(TILE_THREADS) void fused_tile_kernel(PredictArgs a, int maxw, int wf_ld, int nbuf, int wl_floats) {
  constexpr int32_t XD = XB ? LQ_BF16 : LQ_F32, PD = PB ? LQ_BF16 : LQ_F32;
  extern __shared__ __align__(16) float lds_f[];
  float* wf = lds_f;                                     // [c_f + 1][wf_ld]: W_f rows, then b_1, in fp32
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* wl = lds_f + (a.c_f + 1) * wf_ld;               // weights of layers 2.., [l_j][l_(j+1)] each, in fp32 (if they fit)
  float* bufA = wl + wl_floats + wave * nbuf * WROWS * maxw;   // [16][maxw], private to the wavefront
  float* bufB = bufA + (nbuf - 1) * WROWS * maxw;
  const int l1 = a.wout[0];
  for (int i = tid; i < (a.c_f + 1) * wf_ld; i += TILE_THREADS) {
    const int q = i / wf_ld, c = i - q * wf_ld;
    float v = 0.f;
    if (c < l1) {
      if (q < a.c_f) v = load_as_f32(a.W[0], static_cast<int64_t>(q) * a.ldw[0] + c, XD);
      else if (a.bias[0]) v = load_as_f32(a.bias[0], c, XD);
    }
    wf[i] = v;
  }
  if (wl_floats > 0) {
    int off = 0;
    for (int layer = 1; layer < a.n_layers; ++layer) {
      const int cnt = a.win[layer] * a.wout[layer];
      for (int i = tid; i < cnt; i += TILE_THREADS) {
        const int k = i / a.wout[layer], c = i - k * a.wout[layer];
        wl[off + i] = load_as_f32(a.W[layer], static_cast<int64_t>(k) * a.ldw[layer] + c, XD);
      }
      off += cnt;
    }
  }
  __syncthreads();

  const bool single = a.n_layers == 1;
  const int64_t n_steps = (a.n + WROWS - 1) / WROWS;
  for (int64_t step = static_cast<int64_t>(blockIdx.x) * WAVES + wave; step < n_steps;
       step += static_cast<int64_t>(gridDim.x) * WAVES) {
    const int64_t base = step * WROWS;
    const int rows = static_cast<int>(min<int64_t>(WROWS, a.n - base));

    // ---- phase 1
    const int per_row = P4 ? l1 / 4 : l1;
    if constexpr (PIECES > 0) {
      constexpr int PER_ROW = 4 * PIECES;                  // 16-byte pieces per row; lane handles pieces lane + 64 u
      int64_t rowu[PIECES];
      int keyu[PIECES][KT];
#pragma unroll
      for (int u = 0; u < PIECES; ++u) {
        const int r = (lane + 64 * u) / PER_ROW;
        rowu[u] = base + min(r, rows - 1);
#pragma unroll
        for (int k = 0; k < KT; ++k) keyu[u][k] = a.fk[k][rowu[u]];
      }
      v4f pu[PIECES][KT];
#pragma unroll
      for (int u = 0; u < PIECES; ++u) {
        const int c0 = ((lane + 64 * u) % PER_ROW) * 4;
#pragma unroll
        for (int k = 0; k < KT; ++k)
          pu[u][k] = *reinterpret_cast<const v4f*>(static_cast<const float*>(a.P[k]) +
                                                   static_cast<int64_t>(keyu[u][k]) * a.ldp[k] + c0);
      }
#pragma unroll
      for (int u = 0; u < PIECES; ++u) {
        const int i = lane + 64 * u;
        const int r = i / PER_ROW, c0 = (i % PER_ROW) * 4;
        v4f z = *reinterpret_cast<const v4f*>(wf + a.c_f * wf_ld + c0);
        for (int q = 0; q < a.c_f; ++q) {
          const float x = static_cast<const float*>(a.X)[rowu[u] * a.ldx + q];
          const v4f w = *reinterpret_cast<const v4f*>(wf + q * wf_ld + c0);
#pragma unroll
          for (int v = 0; v < 4; ++v) z[v] = fmaf(x, w[v], z[v]);
        }
#pragma unroll
        for (int k = 0; k < KT; ++k)
#pragma unroll
          for (int v = 0; v < 4; ++v) z[v] += pu[u][k][v];
#pragma unroll
        for (int v = 0; v < 4; ++v) bufA[r * maxw + c0 + v] = fmaxf(z[v], 0.f);
      }
    } else
    for (int i = lane; i < WROWS * per_row; i += 64) {
      const int r = i / per_row, c0 = (i - r * per_row) * (P4 ? 4 : 1);
      const int64_t row = base + min(r, rows - 1);         // rows past the end repeat the last one
      float z[4] = {0.f, 0.f, 0.f, 0.f};
      if (P4) {
        const v4f b = *reinterpret_cast<const v4f*>(wf + a.c_f * wf_ld + c0);
#pragma unroll
        for (int v = 0; v < 4; ++v) z[v] = b[v];
        for (int q = 0; q < a.c_f; ++q) {
          const float x = load_as_f32(a.X, row * a.ldx + q, XD);
          const v4f w = *reinterpret_cast<const v4f*>(wf + q * wf_ld + c0);
#pragma unroll
          for (int v = 0; v < 4; ++v) z[v] = fmaf(x, w[v], z[v]);
        }
        for (int k = 0; k < a.K; ++k) {
          const int64_t off = static_cast<int64_t>(a.fk[k][row]) * a.ldp[k] + c0;
          if (!PB) {
            const v4f p = *reinterpret_cast<const v4f*>(static_cast<const float*>(a.P[k]) + off);
#pragma unroll
            for (int v = 0; v < 4; ++v) z[v] += p[v];
          } else {
            const uint2 p = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(a.P[k]) + off);
            z[0] += __uint_as_float(p.x << 16); z[1] += __uint_as_float(p.x & 0xffff0000u);
            z[2] += __uint_as_float(p.y << 16); z[3] += __uint_as_float(p.y & 0xffff0000u);
          }
        }
      } else {
        z[0] = wf[a.c_f * wf_ld + c0];
        for (int q = 0; q < a.c_f; ++q)
          z[0] = fmaf(load_as_f32(a.X, row * a.ldx + q, XD), wf[q * wf_ld + c0], z[0]);
        for (int k = 0; k < a.K; ++k)
          z[0] += load_as_f32(a.P[k], static_cast<int64_t>(a.fk[k][row]) * a.ldp[k] + c0, PD);
      }
#pragma unroll
      for (int v = 0; v < (P4 ? 4 : 1); ++v) {
        if (single) { if (r < rows) store_from_f32(a.Y, (base + r) * a.ldy + c0 + v, a.y_dtype, z[v]); }
        else bufA[r * maxw + c0 + v] = fmaxf(z[v], 0.f);
      }
    }
    if (single) continue;
    wave_sync();

    // ---- phase 2: remaining layers on the matrix cores
    float* in = bufA;
    float* out = bufB;
    const int arow = lane & 15, kk = lane >> 4;            // A operand: row, k = 4 s + lane / 16
    int woff = 0;
    for (int layer = 1; layer < a.n_layers; ++layer) {
      const int win = a.win[layer], wout = a.wout[layer];
      const bool last = layer == a.n_layers - 1;
      // fp32 weights: from the LDS copy if there is one, else from memory (through the same pointer)
      const float* wsrc = wl_floats > 0 ? wl + woff : static_cast<const float*>(a.W[layer]);
      const int64_t wstride = wl_floats > 0 ? wout : a.ldw[layer];
      woff += win * wout;
      // four 16-column tiles at a time: one read of the A operand feeds four independent accumulators
      for (int tc0 = 0; tc0 * 16 < wout; tc0 += 4) {
        v4f acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
        const int ntile = min(4, (wout - 16 * tc0 + 15) / 16);   // column tiles that exist
        for (int s4 = 0; s4 < win; s4 += 4) {
          const int k = s4 + kk;
          const float av = k < win ? in[arow * maxw + k] : 0.f;
          float bv[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int bcol = 16 * (tc0 + j) + (lane & 15);  // B operand: column, same k
            bv[j] = 0.f;
            if (k < win && bcol < wout) {
              if (XB && wl_floats == 0) bv[j] = load_as_f32(a.W[layer], static_cast<int64_t>(k) * a.ldw[layer] + bcol, XD);
              else bv[j] = wsrc[static_cast<int64_t>(k) * wstride + bcol];
            }
          }
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (j < ntile) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv[j], acc[j], 0, 0, 0);
        }
        // register v of lane l: row 4 (l / 16) + v, column 16 tc + l % 16
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int bcol = 16 * (tc0 + j) + (lane & 15);
          if (bcol < wout) {
            const float bb = a.bias[layer] ? load_as_f32(a.bias[layer], bcol, XD) : 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int r = 4 * kk + v;
              const float y = acc[j][v] + bb;
              if (last) { if (r < rows) store_from_f32(a.Y, (base + r) * a.ldy + bcol, a.y_dtype, y); }
              else out[r * maxw + bcol] = fmaxf(y, 0.f);
            }
          }
        }
      }
      wave_sync();
      float* t = in; in = out; out = t;
    }
  }
}

size_t tile_lds_bytes(const PredictArgs& a, int maxw, int wf_ld, int nbuf, int wl_floats) {
  return static_cast<size_t>(a.c_f + 1) * wf_ld * 4 + static_cast<size_t>(wl_floats) * 4 +
         static_cast<size_t>(WAVES) * nbuf * WROWS * maxw * 4;
}

}  // namespace

// Returns -1 when the shape is not one this kernel covers.
int try_fused_tile(const PredictArgs& a, hipStream_t s) {
  int maxw = 4;
  for (int j = 0; j + 1 < a.n_layers; ++j) maxw = std::max(maxw, a.wout[j]);   // widths that live in LDS
  if (maxw > 512 || a.wout[0] > 512 || a.c_f > 64) return -1;
  maxw = static_cast<int>(round_up(static_cast<size_t>(maxw), 4)) + 4;          // +4 staggers rows over LDS banks
  const int wf_ld = static_cast<int>(round_up(static_cast<size_t>(a.wout[0]), 4));
  const int nbuf = a.n_layers > 2 ? 2 : 1;
  int wl_floats = 0;                                     // weights of the later layers go to LDS when they fit next to the tiles
  for (int j = 1; j < a.n_layers; ++j) wl_floats += a.win[j] * a.wout[j];
  if (wl_floats > 5 * 1024) wl_floats = 0;                 // (more than 20 KB costs more in resident workgroups than the LDS reads gain)
  const size_t lds = tile_lds_bytes(a, maxw, wf_ld, nbuf, wl_floats);
  if (lds > 150 * 1024) return -1;
  bool p4 = a.wout[0] % 4 == 0;
  const size_t ps = dtype_size(a.p_dtype);
  for (int k = 0; k < a.K && p4; ++k) p4 = aligned(a.P[k], 4 * ps) && a.ldp[k] % 4 == 0;
  const int64_t n_steps = (a.n + WROWS - 1) / WROWS;
  const int per_cu = static_cast<int>(std::max<size_t>(1, std::min<size_t>(8, (160 * 1024) / lds)));
  const int64_t blocks = std::min<int64_t>((n_steps + WAVES - 1) / WAVES, static_cast<int64_t>(num_cus()) * per_cu * 2);
  if (blocks <= 0) return LQ_OK;
#define LQ_TILE_INST(P4_, XB_, PB_, PC_, KT_)                                                                   \
  do {                                                                                                          \
    if (lds > 64 * 1024)                                                                                        \
      LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_tile_kernel<P4_, XB_, PB_, PC_, KT_>), \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));       \
    hipLaunchKernelGGL((fused_tile_kernel<P4_, XB_, PB_, PC_, KT_>), dim3(static_cast<unsigned>(blocks)),       \
                       dim3(TILE_THREADS), lds, s, a, maxw, wf_ld, nbuf, wl_floats);                                       \
  } while (0)
#define LQ_TILE(P4_, XB_, PB_) LQ_TILE_INST(P4_, XB_, PB_, 0, 0)
#define LQ_TILE_K(PC_)                                                                      \
  switch (a.K) {                                                                            \
    case 1: LQ_TILE_INST(true, false, false, PC_, 1); break;                                \
    case 2: LQ_TILE_INST(true, false, false, PC_, 2); break;                                \
    case 3: LQ_TILE_INST(true, false, false, PC_, 3); break;                                \
    default: LQ_TILE_INST(true, false, false, PC_, 4); break;                               \
  }
  const bool xb = a.x_dtype == LQ_BF16, pb = a.p_dtype == LQ_BF16;
  const int l1w = a.wout[0];
  const bool unrolled = p4 && !xb && !pb && a.n_layers > 1 && a.K >= 1 && a.K <= 4 &&
                        (l1w == 32 || l1w == 64 || l1w == 128 || l1w == 256);
  if (unrolled) {
    if (l1w == 32) { LQ_TILE_K(2) } else if (l1w == 64) { LQ_TILE_K(4) } else if (l1w == 128) { LQ_TILE_K(8) } else { LQ_TILE_K(16) }
  } else if (p4) {
    if (!xb && !pb) LQ_TILE(true, false, false);
    else if (xb && pb) LQ_TILE(true, true, true);
    else if (xb) LQ_TILE(true, true, false);
    else return -1;
  } else {
    if (!xb && !pb) LQ_TILE(false, false, false);
    else if (xb && pb) LQ_TILE(false, true, true);
    else if (xb) LQ_TILE(false, true, false);
    else return -1;
  }
#undef LQ_TILE_K
#undef LQ_TILE_INST
#undef LQ_TILE
  LQ_LAUNCH_CHECK("fused_tile_kernel");
  return LQ_OK;
}

}  // namespace lq
