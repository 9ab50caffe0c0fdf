// The C boundary of liblq: argument validation, error reporting and dispatch.
// Every entry point validates on the host, enqueues on the caller's stream and returns.
#include <string.h>

#include <mutex>
#include <vector>

#include "lq_common.h"

namespace lq {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = 0; }

int num_cus() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cached[dev] = v;
  }
  return cached[dev];
}

int resident_per_cu(const void* kernel, int threads, size_t lds) {
  struct Entry { int dev; const void* kernel; int threads; size_t lds; int value; };
  static std::mutex mu;
  static std::vector<Entry> cache;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) dev = 0;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : cache)
    if (e.dev == dev && e.kernel == kernel && e.threads == threads && e.lds == lds) return e.value;
  int v = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, kernel, threads, lds) != hipSuccess || v < 1) {
    (void)hipGetLastError();
    v = 1;
  }
  cache.push_back({dev, kernel, threads, lds, v});
  return v;
}

int launch_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                const void* bias, int64_t M, int32_t N, int32_t Kd, int relu, int32_t in_dtype,
                int32_t out_dtype, hipStream_t s);
int launch_fused_generic(const PredictArgs& a, hipStream_t s);
bool fused_kernel_covers(const PredictArgs& a);
size_t fused_layered_bytes_per_256(const PredictArgs& a);
int launch_fused_layered(const PredictArgs& a, void* ws, size_t ws_bytes, hipStream_t s);
int launch_fused_tile(const PredictArgs& a, hipStream_t s);
int launch_groupby(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                   const uint8_t* const* mask, const int32_t* const* code, const int32_t* card,
                   const uint8_t* fact_mask, int32_t M, const int32_t* const* meas, int64_t* sums,
                   int64_t* counts, int32_t G, void* ws, size_t ws_bytes, bool reuse_tables, hipStream_t s);
size_t groupby_ws_bytes(int32_t K, const int64_t* rows, int64_t n_acc);
size_t groupby_bucket_ws_bytes(int64_t n, int32_t K, const int64_t* rows, int64_t G, int32_t M);
int launch_group_diff(int64_t G, const int64_t* two, int64_t* sums, hipStream_t s);
int launch_groupby_agg(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                       const uint8_t* const* mask, const int32_t* const* code, const int32_t* card,
                       int32_t n_preds, const lq_range_pred* preds, int32_t M, const lq_measure* meas,
                       int64_t* sums, int64_t* mins, int64_t* maxs, int64_t* counts, int32_t G, void* ws,
                       bool reuse_tables, hipStream_t s);
size_t groupby_tables_bytes(int32_t K, const int64_t* rows);
int launch_group_avg(int32_t M, int64_t G, const int64_t* sums, const int64_t* counts, double* avgs, hipStream_t s);

namespace {

int check_mat(const lq_mat& m, const char* what, bool need_data) {
  if (m.rows < 0 || m.cols < 0) return fail(LQ_ERR_SHAPE, "%s: negative size", what);
  if (!dtype_ok(m.dtype)) return fail(LQ_ERR_DTYPE, "%s: unknown dtype %d", what, m.dtype);
  if (m.rows > 0 && m.cols > 0) {
    if (m.ld < m.cols) return fail(LQ_ERR_SHAPE, "%s: ld %lld < cols %d", what, (long long)m.ld, m.cols);
    if (need_data && !m.data) return fail(LQ_ERR_NULL, "%s: data is NULL", what);
    if (m.data && !aligned(m.data, dtype_size(m.dtype)))
      return fail(LQ_ERR_SHAPE, "%s: data is not aligned to its element size", what);
  }
  return LQ_OK;
}

// Validates star + model (+ optional P) and works out the common dtype and the joined width.
struct Checked {
  int32_t dtype = LQ_F32;
  int32_t kw = 0;      // joined width k
  int32_t l1 = 0, l_out = 0;
};

int check_star_model(const lq_star* star, const lq_model* model, bool need_dims, Checked* out) {
  if (!star || !model) return fail(LQ_ERR_NULL, "star or model is NULL");
  if (star->n_fact < 0) return fail(LQ_ERR_SHAPE, "n_fact < 0");
  if (star->n_dims < 0 || star->n_dims > LQ_MAX_DIMS)
    return fail(LQ_ERR_SHAPE, "n_dims %d outside 0..%d", star->n_dims, LQ_MAX_DIMS);
  if (model->n_layers < 1 || model->n_layers > LQ_MAX_LAYERS)
    return fail(LQ_ERR_SHAPE, "n_layers %d outside 1..%d", model->n_layers, LQ_MAX_LAYERS);
  if (!model->W) return fail(LQ_ERR_NULL, "model->W is NULL");
  if (star->n_dims > 0 && !star->fks) return fail(LQ_ERR_NULL, "star->fks is NULL");
  if (star->n_dims > 0 && need_dims && !star->dims) return fail(LQ_ERR_NULL, "star->dims is NULL");

  const int32_t dt = model->W[0].dtype;
  int rc = LQ_OK;
  int32_t kw = 0;
  if (star->fact.cols > 0) {
    if ((rc = check_mat(star->fact, "fact", star->n_fact > 0))) return rc;
    if (star->fact.rows != star->n_fact) return fail(LQ_ERR_SHAPE, "fact.rows != n_fact");
    if (star->fact.dtype != dt) return fail(LQ_ERR_DTYPE, "fact and W[0] differ in dtype");
    kw = star->fact.cols;
  } else if (star->fact.cols < 0) {
    return fail(LQ_ERR_SHAPE, "fact.cols < 0");
  }
  for (int k = 0; k < star->n_dims; ++k) {
    if (star->n_fact > 0 && !star->fks[k]) return fail(LQ_ERR_NULL, "fks[%d] is NULL", k);
    if (star->fks[k] && !aligned(star->fks[k], 4)) return fail(LQ_ERR_SHAPE, "fks[%d] is not 4-byte aligned", k);
    if (need_dims || star->dims) {
      char name[32];
      snprintf(name, sizeof(name), "dims[%d]", k);
      if ((rc = check_mat(star->dims[k], name, true))) return rc;
      if (star->dims[k].dtype != dt) return fail(LQ_ERR_DTYPE, "%s and W[0] differ in dtype", name);
      if (star->dims[k].rows < 1 && star->n_fact > 0) return fail(LQ_ERR_SHAPE, "%s has no rows", name);
      kw += star->dims[k].cols;
    }
  }
  for (int j = 0; j < model->n_layers; ++j) {
    char name[32];
    snprintf(name, sizeof(name), "W[%d]", j);
    if ((rc = check_mat(model->W[j], name, true))) return rc;
    if (model->W[j].dtype != dt) return fail(LQ_ERR_DTYPE, "all layers must share one dtype");
    if (model->W[j].cols < 1) return fail(LQ_ERR_SHAPE, "%s has no columns", name);
    if (j > 0 && model->W[j].rows != model->W[j - 1].cols)
      return fail(LQ_ERR_SHAPE, "%s has %lld rows but the previous layer has %d outputs", name,
                  (long long)model->W[j].rows, model->W[j - 1].cols);
    if (model->bias && model->bias[j] && !aligned(model->bias[j], dtype_size(dt)))
      return fail(LQ_ERR_SHAPE, "bias[%d] is misaligned", j);
  }
  if ((need_dims || star->dims || star->n_dims == 0) && model->W[0].rows != kw)
    return fail(LQ_ERR_SHAPE, "W[0] has %lld rows but the joined width is %d",
                (long long)model->W[0].rows, kw);
  out->dtype = dt;
  out->kw = static_cast<int32_t>(model->W[0].rows);
  out->l1 = model->W[0].cols;
  out->l_out = model->W[model->n_layers - 1].cols;
  return LQ_OK;
}

int check_Y(const lq_mat* Y, int64_t n, int32_t l_out, int32_t model_dtype) {
  if (!Y) return fail(LQ_ERR_NULL, "Y is NULL");
  int rc = check_mat(*Y, "Y", n > 0);
  if (rc) return rc;
  if (Y->rows != n || Y->cols != l_out)
    return fail(LQ_ERR_SHAPE, "Y is %lld x %d, expected %lld x %d", (long long)Y->rows, Y->cols,
                (long long)n, l_out);
  if (Y->dtype == LQ_BF16 && model_dtype != LQ_BF16)
    return fail(LQ_ERR_DTYPE, "bf16 output needs a bf16 model");
  return LQ_OK;
}

void fill_layers(PredictArgs* a, const lq_model* model) {
  a->n_layers = model->n_layers;
  for (int j = 0; j < model->n_layers; ++j) {
    a->W[j] = model->W[j].data;
    a->ldw[j] = model->W[j].ld;
    a->win[j] = static_cast<int32_t>(model->W[j].rows);
    a->wout[j] = model->W[j].cols;
    a->bias[j] = model->bias ? model->bias[j] : nullptr;
  }
}

// Synchronous range check of the foreign keys; ws must hold one int32.
int run_fk_check(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                 bool negative_ok, void* ws, size_t ws_bytes, hipStream_t s) {
  if (!ws || ws_bytes < 256 || !aligned(ws, 256))
    return fail(LQ_ERR_WORKSPACE, "LQ_CHECK_FKS needs a 256-byte aligned workspace of >= 256 bytes");
  int32_t* flag = static_cast<int32_t*>(ws);
  int rc = launch_check_fks(n, K, fks, rows, negative_ok, flag, s);
  if (rc) return rc;
  int32_t h = 0;
  LQ_HIP_TRY(hipMemcpyAsync(&h, flag, sizeof(h), hipMemcpyDeviceToHost, s));
  LQ_HIP_TRY(hipStreamSynchronize(s));
  if (h) return fail(LQ_ERR_FK_RANGE, "a foreign key lies outside its dimension table");
  return LQ_OK;
}

// Group-by calls keep the packed side tables at the start of their workspace (and may be asked to
// reuse them), so the check's flag word goes behind them, into the partial-sum area that the scan
// overwrites afterwards.  Besides the keys, the check covers the group codes of the dimension side:
// a code outside [0, group_card) on a row that passes its mask would address an accumulator that
// does not exist.
int check_groupby_fks(int64_t n, int32_t K, const int32_t* const* fks, const int64_t* rows,
                      const uint8_t* const* mask, const int32_t* const* code, const int32_t* card, void* ws,
                      size_t ws_bytes, hipStream_t s) {
  const size_t off = groupby_tables_bytes(K, rows);
  if (!ws || ws_bytes < off + 256 || !aligned(ws, 256))
    return fail(LQ_ERR_WORKSPACE, "LQ_CHECK_FKS needs a 256-byte aligned workspace of >= 256 bytes");
  int32_t* flag = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(ws) + off);
  int rc = launch_check_fks(n, K, fks, rows, true, flag, s);
  if (rc) return rc;
  if ((rc = launch_check_codes(K, rows, mask, code, card, flag, s))) return rc;
  int32_t h = 0;
  LQ_HIP_TRY(hipMemcpyAsync(&h, flag, sizeof(h), hipMemcpyDeviceToHost, s));
  LQ_HIP_TRY(hipStreamSynchronize(s));
  if (h & 1) return fail(LQ_ERR_FK_RANGE, "a foreign key lies outside its dimension table");
  if (h & 2) return fail(LQ_ERR_SHAPE, "a group code lies outside [0, group_card) on a dimension row that passes its mask");
  return LQ_OK;
}

constexpr uint32_t FLAG_FORCE_GENERIC = 0x100u;   // testing aid, see lq_fused_join_predict

}  // namespace
}  // namespace lq

using namespace lq;

extern "C" {

const char* lq_last_error(void) { return g_err; }
const char* lq_version(void) { return "lq 0.1 (gfx950)"; }

int lq_project_dims(const lq_star* star, const lq_model* model, lq_mat* P, void* hip_stream) {
  clear_error();
  Checked c;
  int rc = check_star_model(star, model, true, &c);
  if (rc) return rc;
  if (star->n_dims > 0 && !P) return fail(LQ_ERR_NULL, "P is NULL");
  for (int k = 0; k < star->n_dims; ++k) {
    char name[32];
    snprintf(name, sizeof(name), "P[%d]", k);
    if ((rc = check_mat(P[k], name, true))) return rc;
    if (P[k].rows != star->dims[k].rows || P[k].cols != c.l1)
      return fail(LQ_ERR_SHAPE, "%s is %lld x %d, expected %lld x %d", name, (long long)P[k].rows,
                  P[k].cols, (long long)star->dims[k].rows, c.l1);
    if (P[k].dtype == LQ_BF16 && c.dtype != LQ_BF16)
      return fail(LQ_ERR_DTYPE, "%s: bf16 projected tables need a bf16 model", name);
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int32_t off = star->fact.cols > 0 ? star->fact.cols : 0;
  return launch_project_dims_all(star->n_dims, star->dims, model->W[0], off, P, s);
}

int lq_project_dim_rows(const lq_star* star, const lq_model* model, lq_mat* P, int32_t dim,
                        int64_t first_row, int64_t n_rows, void* hip_stream) {
  clear_error();
  Checked c;
  int rc = check_star_model(star, model, true, &c);
  if (rc) return rc;
  if (!P) return fail(LQ_ERR_NULL, "P is NULL");
  if (dim < 0 || dim >= star->n_dims) return fail(LQ_ERR_SHAPE, "dimension %d outside 0..%d", dim, star->n_dims - 1);
  if ((rc = check_mat(P[dim], "P[dim]", true))) return rc;
  const lq_mat& D = star->dims[dim];
  if (P[dim].rows != D.rows || P[dim].cols != c.l1) return fail(LQ_ERR_SHAPE, "P[dim] does not match its dimension table");
  if (P[dim].dtype == LQ_BF16 && c.dtype != LQ_BF16) return fail(LQ_ERR_DTYPE, "bf16 projected tables need a bf16 model");
  if (first_row < 0 || n_rows < 0 || first_row + n_rows > D.rows)
    return fail(LQ_ERR_SHAPE, "rows %lld .. +%lld outside the dimension table", (long long)first_row, (long long)n_rows);
  if (n_rows == 0) return LQ_OK;
  int32_t off = star->fact.cols > 0 ? star->fact.cols : 0;
  for (int k = 0; k < dim; ++k) off += star->dims[k].cols;
  lq_mat Ds = D, Ps = P[dim];
  Ds.data = static_cast<char*>(D.data) + static_cast<size_t>(first_row) * D.ld * dtype_size(D.dtype);
  Ds.rows = n_rows;
  Ps.data = static_cast<char*>(P[dim].data) + static_cast<size_t>(first_row) * P[dim].ld * dtype_size(P[dim].dtype);
  Ps.rows = n_rows;
  return launch_project_dims(Ds, model->W[0], off, Ps, static_cast<hipStream_t>(hip_stream));
}

int lq_fusion_advice(const lq_star* star, const lq_model* model, double queries_per_update, lq_advice* out) {
  clear_error();
  Checked c;
  int rc = check_star_model(star, model, true, &c);
  if (rc) return rc;
  if (!out) return fail(LQ_ERR_NULL, "out is NULL");
  if (!(queries_per_update > 0.0)) return fail(LQ_ERR_SHAPE, "queries_per_update must be positive");
  const double n = static_cast<double>(star->n_fact), k = c.kw, l = c.l1;
  double sum_r = 0, mm_dims = 0, prefuse = 0, dim_elems = 0, p_elems = 0;
  for (int j = 0; j < star->n_dims; ++j) {
    const double r = static_cast<double>(star->dims[j].rows), cj = star->dims[j].cols;
    sum_r += r;
    mm_dims += cj * k * r;          // D_j M_j            (the c k sum r_j term of the complexity analysis)
    prefuse += r * cj * l;          // D_j M_j L, done once per update of the dimensions or the model
    dim_elems += r * cj;
    p_elems += r * l;
  }
  out->cost_no_fusion = mm_dims + n * k * sum_r + n * k * l;
  out->cost_fusion = n * l * sum_r;
  out->cost_prefusion = prefuse;
  out->ratio = out->cost_fusion > 0 ? out->cost_no_fusion / out->cost_fusion : 0.0;
  out->ratio_leading_term = l > 0 ? k / l : 0.0;
  out->memory_growth = dim_elems > 0 ? p_elems / dim_elems : 0.0;
  // What the kernels here actually move per fact row (one nonzero per row of I_k, not the dense model):
  const double es = static_cast<double>(dtype_size(c.dtype));
  out->bytes_per_row_fused = es * (star->fact.cols > 0 ? star->fact.cols : 0) + 4.0 * star->n_dims +
                             es * l * star->n_dims + es * c.l_out;
  out->bytes_per_row_no_fusion = es * (star->fact.cols > 0 ? star->fact.cols : 0) + 4.0 * star->n_dims +
                                 es * (k - (star->fact.cols > 0 ? star->fact.cols : 0)) + 2.0 * es * k + es * c.l_out;
  // The decision.  The dense model above prices I_k as an n x r_k matrix; here I_k is one key per
  // fact row, so what decides is what the two pipelines of this library move and multiply per fact
  // row, at the rates they sustain on an MI355X (measured with this library's own kernels):
  //   streamed bytes (fact columns, keys, outputs, T written and read back)   ~5 TB/s
  //   gathered bytes (rows of P_k or D_k; from L2 / the 256 MB Infinity Cache while the tables fit
  //   in half of it, else whole 128-byte lines from memory)                    ~14 TB/s / ~3 TB/s
  //   dense products                                                           ~60 TFLOP/s fp32, ~400 bf16
  //   a kernel launch                                                          ~4 us
  const double c_f = star->fact.cols > 0 ? star->fact.cols : 0;
  const double K = star->n_dims;
  constexpr double STREAM = 5.0e12, CACHE_GATHER = 14.0e12, MEMORY_GATHER = 3.0e12, LAUNCH = 4.0e-6;
  constexpr double CACHE_BYTES = 128.0 * 1024 * 1024;
  const double dense = c.dtype == LQ_BF16 ? 400.0e12 : 60.0e12;
  double later_flops = 0, later_bytes = 0;     // layers after the first: same products in both pipelines,
  for (int j = 1; j < model->n_layers; ++j) {  // but the non-fused one moves every activation through memory
    later_flops += 2.0 * static_cast<double>(model->W[j].rows) * model->W[j].cols;
    later_bytes += 2.0 * es * static_cast<double>(model->W[j].rows);
  }
  auto gather_seconds = [&](double row_bytes, double table_bytes) {
    if (table_bytes <= CACHE_BYTES) return row_bytes / CACHE_GATHER;
    return std::max(row_bytes, 128.0) / MEMORY_GATHER;
  };
  double gather_f = 0, gather_n = 0;           // one row of P_j / of D_j per dimension and fact row
  for (int j = 0; j < star->n_dims; ++j) {
    gather_f += gather_seconds(es * l, p_elems * es);
    gather_n += gather_seconds(es * star->dims[j].cols, dim_elems * es);
  }
  const double stream_f = es * c_f + 4.0 * K + es * c.l_out;
  const double stream_n = es * c_f + 4.0 * K + 2.0 * es * k + later_bytes + es * c.l_out;
  out->seconds_fused = n * (stream_f / STREAM + gather_f + later_flops / dense) + LAUNCH;
  out->seconds_no_fusion = n * (stream_n / STREAM + gather_n + (2.0 * k * l + later_flops) / dense) +
                           (1.0 + model->n_layers) * LAUNCH;
  out->seconds_prefusion = (dim_elems + p_elems) * es / STREAM + 2.0 * prefuse / dense + LAUNCH;
  out->fuse = queries_per_update * (out->seconds_no_fusion - out->seconds_fused) > out->seconds_prefusion ? 1 : 0;
  return LQ_OK;
}

int lq_fused_join_predict(const lq_star* star, const lq_model* model, const lq_mat* P, lq_mat* Y,
                          void* ws, size_t ws_bytes, uint32_t flags, void* hip_stream) {
  clear_error();
  Checked c;
  int rc = check_star_model(star, model, false, &c);
  if (rc) return rc;
  if (star->n_dims > 0 && !P) return fail(LQ_ERR_NULL, "P is NULL");
  if ((rc = check_Y(Y, star->n_fact, c.l_out, c.dtype))) return rc;
  PredictArgs a{};
  a.n = star->n_fact;
  a.c_f = star->fact.cols > 0 ? star->fact.cols : 0;
  a.X = a.c_f ? star->fact.data : nullptr;
  a.ldx = star->fact.ld;
  a.K = star->n_dims;
  int64_t rows[LQ_MAX_DIMS];
  for (int k = 0; k < a.K; ++k) {
    char name[32];
    snprintf(name, sizeof(name), "P[%d]", k);
    if ((rc = check_mat(P[k], name, true))) return rc;
    if (P[k].cols != c.l1 || P[k].rows < 1)
      return fail(LQ_ERR_SHAPE, "%s is %lld x %d, expected r_k x %d", name, (long long)P[k].rows,
                  P[k].cols, c.l1);
    if (P[k].dtype != P[0].dtype) return fail(LQ_ERR_DTYPE, "projected tables differ in dtype");
    if (P[k].dtype == LQ_BF16 && c.dtype != LQ_BF16)
      return fail(LQ_ERR_DTYPE, "%s: bf16 projected tables need a bf16 model", name);
    if (star->dims) {
      if (star->dims[k].rows != P[k].rows)
        return fail(LQ_ERR_SHAPE, "%s has %lld rows, dims[%d] has %lld", name, (long long)P[k].rows, k,
                    (long long)star->dims[k].rows);
    }
    a.P[k] = P[k].data;
    a.ldp[k] = P[k].ld;
    a.prows[k] = P[k].rows;
    a.fk[k] = star->fks[k];
    rows[k] = P[k].rows;
  }
  if (!star->dims && a.K > 0 && model->W[0].rows < a.c_f)
    return fail(LQ_ERR_SHAPE, "W[0] has fewer rows than the fact table has columns");
  fill_layers(&a, model);
  a.Y = Y->data; a.ldy = Y->ld;
  a.x_dtype = c.dtype;
  a.p_dtype = a.K ? P[0].dtype : c.dtype;
  a.y_dtype = Y->dtype;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if ((flags & LQ_CHECK_FKS) && a.K > 0 && a.n > 0)
    if ((rc = run_fk_check(a.n, a.K, star->fks, rows, false, ws, ws_bytes, s))) return rc;
  if (flags & FLAG_FORCE_GENERIC) return launch_fused_generic(a, s);
  if (flags & LQ_FORCE_TILE) return launch_fused_tile(a, s);
  // A model of two or more layers that no specialised kernel takes, and a workspace with room for a chunk of
  // activations behind its first 256 bytes: the join stage as a linear operator, then dense products.
  // (Only for models with a layer wider than 128 or more than 16 fact columns: narrow models that no specialised
  // kernel takes are better off in one pass of the per-wavefront tile kernel than in a dense product per layer.)
  int widest = 0;
  for (int j = 0; j < a.n_layers; ++j) widest = std::max(widest, a.wout[j]);
  if (a.n_layers >= 2 && (widest > 128 || a.c_f > 16) && a.n > 0 && ws && aligned(ws, 256) &&
      ws_bytes >= 256 + fused_layered_bytes_per_256(a) && !fused_kernel_covers(a))
    return launch_fused_layered(a, static_cast<uint8_t*>(ws) + 256, ws_bytes - 256, s);
  return launch_fused(a, s);
}

size_t lq_workspace_bytes(int which_call, const lq_star* star, const lq_model* model,
                          int64_t chunk_rows) {
  if (which_call == LQ_CALL_FUSED) {
    // 256 bytes for the checked call; with chunk_rows > 0 and a model of two or more layers also two activation
    // buffers of that many rows, which the layered form of the join stage uses when no specialised kernel takes
    // the model (see lq_fused_join_predict)
    if (chunk_rows < 1 || !model || !model->W || model->n_layers < 2 || model->n_layers > LQ_MAX_LAYERS) return 256;
    const size_t es = dtype_size(model->W[0].dtype);
    size_t widest = 0;
    for (int j = 0; j + 1 < model->n_layers; ++j)
      widest = std::max(widest, round_up(static_cast<size_t>(model->W[j].cols) * es, 16));
    return 256 + 2 * round_up(static_cast<size_t>(chunk_rows), 256) * widest;
  }
  if (which_call != LQ_CALL_MATERIALIZED || !star || !model || !model->W || chunk_rows < 1) return 0;
  if (model->n_layers < 1 || model->n_layers > LQ_MAX_LAYERS) return 0;
  const size_t es = dtype_size(model->W[0].dtype);
  size_t widest = 0;
  for (int j = 0; j + 1 < model->n_layers; ++j)
    widest = std::max(widest, static_cast<size_t>(model->W[j].cols));
  const size_t rows = round_up(static_cast<size_t>(chunk_rows), 256);
  const size_t t_bytes = round_up(rows * static_cast<size_t>(model->W[0].rows) * es, 256);
  const size_t act_bytes = round_up(rows * widest * es, 256);
  return 256 + t_bytes + 2 * act_bytes;
}

int lq_materialized_join_predict(const lq_star* star, const lq_model* model, lq_mat* Y, void* ws,
                                 size_t ws_bytes, uint32_t flags, void* hip_stream) {
  clear_error();
  Checked c;
  int rc = check_star_model(star, model, true, &c);
  if (rc) return rc;
  if ((rc = check_Y(Y, star->n_fact, c.l_out, c.dtype))) return rc;
  if (star->n_fact == 0) return LQ_OK;
  if (!ws || !aligned(ws, 256)) return fail(LQ_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  // Largest chunk (multiple of 256 rows) whose buffers fit.
  const size_t per256 = lq_workspace_bytes(LQ_CALL_MATERIALIZED, star, model, 256) - 256;
  if (ws_bytes < 256 + per256)
    return fail(LQ_ERR_WORKSPACE, "workspace of %zu bytes cannot hold one 256-row chunk (%zu needed)",
                ws_bytes, 256 + per256);
  int64_t chunk = static_cast<int64_t>((ws_bytes - 256) / per256) * 256;
  while (chunk > 256 && lq_workspace_bytes(LQ_CALL_MATERIALIZED, star, model, chunk) > ws_bytes) chunk -= 256;
  chunk = std::min<int64_t>(chunk, static_cast<int64_t>(round_up(static_cast<size_t>(star->n_fact), 256)));

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int64_t rows[LQ_MAX_DIMS];
  for (int k = 0; k < star->n_dims; ++k) rows[k] = star->dims[k].rows;
  if ((flags & LQ_CHECK_FKS) && star->n_dims > 0)
    if ((rc = run_fk_check(star->n_fact, star->n_dims, star->fks, rows, false, ws, ws_bytes, s))) return rc;

  const size_t es = dtype_size(c.dtype);
  size_t widest = 0;
  for (int j = 0; j + 1 < model->n_layers; ++j) widest = std::max(widest, static_cast<size_t>(model->W[j].cols));
  char* base = static_cast<char*>(ws) + 256;
  void* T = base;
  const size_t t_bytes = round_up(static_cast<size_t>(chunk) * c.kw * es, 256);
  const size_t act_bytes = round_up(static_cast<size_t>(chunk) * widest * es, 256);
  void* act[2] = {base + t_bytes, base + t_bytes + act_bytes};

  for (int64_t r0 = 0; r0 < star->n_fact; r0 += chunk) {
    const int64_t m = std::min<int64_t>(chunk, star->n_fact - r0);
    if ((rc = launch_materialize(*star, T, c.kw, r0, m, s))) return rc;
    const void* in = T;
    int64_t ldin = c.kw;
    for (int j = 0; j < model->n_layers; ++j) {
      const bool last = j == model->n_layers - 1;
      void* out = last ? static_cast<void*>(static_cast<char*>(Y->data) +
                                            static_cast<size_t>(r0) * Y->ld * dtype_size(Y->dtype))
                       : act[j & 1];
      const int64_t ldout = last ? Y->ld : model->W[j].cols;
      rc = launch_gemm(in, ldin, model->W[j].data, model->W[j].ld, out, ldout,
                       model->bias ? model->bias[j] : nullptr, m, model->W[j].cols,
                       static_cast<int32_t>(model->W[j].rows), last ? 0 : 1, c.dtype,
                       last ? Y->dtype : c.dtype, s);
      if (rc) return rc;
      in = out;
      ldin = ldout;
    }
  }
  return LQ_OK;
}

size_t lq_groupby_workspace_bytes(int32_t n_dims, const int64_t* dim_rows, const int32_t* group_card,
                                  int32_t n_measures) {
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS || (n_dims > 0 && !dim_rows)) return 0;
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES) return 0;
  int64_t G = 1;
  for (int k = 0; k < n_dims; ++k) {
    if (dim_rows[k] < 0) return 0;
    if (group_card) {
      if (group_card[k] < 1 || group_card[k] > 65535) return 0;
      G *= group_card[k];
      if (G > LQ_MAX_GROUPS) return 0;
    }
  }
  return groupby_ws_bytes(n_dims, dim_rows, G * (n_measures + 1));
}

size_t lq_groupby_bucket_workspace_bytes(int64_t n_fact, int32_t n_dims, const int64_t* dim_rows, const int32_t* group_card,
                                         int32_t n_measures) {
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS || (n_dims > 0 && !dim_rows) || !group_card) return 0;
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES) return 0;
  int64_t G = 1;
  for (int k = 0; k < n_dims; ++k) {
    if (dim_rows[k] < 0 || group_card[k] < 1 || group_card[k] > 65535) return 0;
    G *= group_card[k];
    if (G > LQ_MAX_GROUPS) return 0;
  }
  return groupby_bucket_ws_bytes(n_fact, n_dims, dim_rows, G, n_measures);
}

// Validation and launch shared by lq_masked_groupby_sum and its allocation-free variant.
static int groupby_sum_checked(int64_t n_fact, int32_t n_dims, const int32_t* const* fks,
                               const int64_t* dim_rows, const uint8_t* const* dim_mask,
                               const int32_t* const* dim_code, const int32_t* group_card,
                               const uint8_t* fact_mask, int32_t n_measures,
                               const int32_t* const* measures, int64_t* sums, int64_t* counts, void* ws,
                               size_t ws_bytes, uint32_t flags, void* hip_stream) {
  if (n_fact < 0) return fail(LQ_ERR_SHAPE, "n_fact < 0");
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS) return fail(LQ_ERR_SHAPE, "n_dims %d outside 0..%d", n_dims, LQ_MAX_DIMS);
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES)
    return fail(LQ_ERR_SHAPE, "n_measures %d outside 1..%d", n_measures, LQ_MAX_MEASURES);
  if (n_dims > 0 && (!fks || !dim_rows)) return fail(LQ_ERR_NULL, "fks or dim_rows is NULL");
  if (!measures || !sums) return fail(LQ_ERR_NULL, "measures or sums is NULL");
  if (!aligned(sums, 8) || !aligned(counts, 8)) return fail(LQ_ERR_SHAPE, "sums / counts are not 8-byte aligned");
  int64_t G = 1;
  for (int k = 0; k < n_dims; ++k) {
    if (n_fact > 0 && !fks[k]) return fail(LQ_ERR_NULL, "fks[%d] is NULL", k);
    if (!aligned(fks[k], 4)) return fail(LQ_ERR_SHAPE, "fks[%d] is not 4-byte aligned", k);
    if (dim_rows[k] < 0 || dim_rows[k] > 0x7fffffffLL) return fail(LQ_ERR_SHAPE, "dim_rows[%d] out of range", k);
    if (dim_code && dim_code[k]) {
      if (!group_card) return fail(LQ_ERR_NULL, "group_card is NULL");
      if (group_card[k] < 1 || group_card[k] > 65535)
        return fail(LQ_ERR_SHAPE, "group_card[%d] = %d outside 1..65535", k, group_card[k]);
      if (!aligned(dim_code[k], 4)) return fail(LQ_ERR_SHAPE, "dim_code[%d] is not 4-byte aligned", k);
      G *= group_card[k];
      if (G > LQ_MAX_GROUPS) return fail(LQ_ERR_UNSUPPORTED, "more than 2^30 groups");
    }
    if (dim_rows[k] == 0 && n_fact > 0 && ((dim_code && dim_code[k]) || (dim_mask && dim_mask[k])))
      return fail(LQ_ERR_SHAPE, "dimension %d has no rows", k);
  }
  for (int m = 0; m < n_measures; ++m) {
    if (n_fact > 0 && !measures[m]) return fail(LQ_ERR_NULL, "measures[%d] is NULL", m);
    if (!aligned(measures[m], 4)) return fail(LQ_ERR_SHAPE, "measures[%d] is not 4-byte aligned", m);
  }
  const size_t need = groupby_ws_bytes(n_dims, dim_rows, G * (n_measures + 1));
  if (!ws || !aligned(ws, 256) || ws_bytes < need)
    return fail(LQ_ERR_WORKSPACE, "group-by needs a 256-byte aligned workspace of %zu bytes", need);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc;
  if ((flags & LQ_CHECK_FKS) && n_dims > 0 && n_fact > 0)
    if ((rc = check_groupby_fks(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, ws, ws_bytes, s))) return rc;
  // Three or four measures over more accumulators than LDS holds: the bucketed form takes two measures a call, so with a
  // workspace that has room for it the call runs as two of them (the counts with the first, the side tables encoded
  // once); far fewer device-wide atomics than one pass of the generic scan.
  const bool reuse = (flags & LQ_REUSE_SIDE_TABLES) != 0;
  if (n_measures > 2 && G * 3 > 8192 && aligned(fact_mask, 4) && n_fact > 0) {
    const size_t big = groupby_bucket_ws_bytes(n_fact, n_dims, dim_rows, G, 2);
    if (big > 0 && ws_bytes >= big) {
      for (int m0 = 0; m0 < n_measures; m0 += 2) {
        const int mm = std::min(2, n_measures - m0);
        if ((rc = launch_groupby(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, fact_mask, mm, measures + m0,
                                 sums + static_cast<int64_t>(m0) * G, m0 == 0 ? counts : nullptr, static_cast<int32_t>(G), ws,
                                 ws_bytes, reuse || m0 > 0, s)))
          return rc;
      }
      return LQ_OK;
    }
  }
  return launch_groupby(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, fact_mask,
                        n_measures, measures, sums, counts, static_cast<int32_t>(G), ws, ws_bytes, reuse, s);
}

int lq_masked_groupby_sum(int64_t n_fact, int32_t n_dims, const int32_t* const* fks,
                          const int64_t* dim_rows, const uint8_t* const* dim_mask,
                          const int32_t* const* dim_code, const int32_t* group_card,
                          const uint8_t* fact_mask, int32_t n_measures,
                          const int32_t* const* measures, int64_t* sums, int64_t* counts, void* ws,
                          size_t ws_bytes, uint32_t flags, void* hip_stream) {
  clear_error();
  return groupby_sum_checked(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, fact_mask,
                             n_measures, measures, sums, counts, ws, ws_bytes, flags, hip_stream);
}

// ---- the same call for callers that cannot allocate --------------------------------------------
// The side tables and the per-workgroup partial rows live in this array instead of a caller
// workspace.  Every GPU holds its own copy at its own address; host code reaches it only through
// the address hipGetSymbolAddress returns for the current device (the array's name is a host-side
// stand-in, not a device address).
static __device__ __align__(256) unsigned char scratch[LQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  int dev = 0;
  LQ_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(LQ_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    LQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || !aligned(p, 256)) return fail(LQ_ERR_HIP, "static scratch array has no usable device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LQ_OK;
}
}  // namespace

size_t lq_static_scratch_bytes(void) { return LQ_STATIC_SCRATCH_BYTES; }

int lq_masked_groupby_sum_static(int64_t n_fact, int32_t n_dims, const int32_t* const* fks,
                                 const int64_t* dim_rows, const uint8_t* const* dim_mask,
                                 const int32_t* const* dim_code, const int32_t* group_card,
                                 const uint8_t* fact_mask, int32_t n_measures,
                                 const int32_t* const* measures, int64_t* sums, int64_t* counts,
                                 uint32_t flags, void* hip_stream) {
  clear_error();
  if (flags != 0) return fail(LQ_ERR_UNSUPPORTED, "the allocation-free group-by takes no flags");
  // Size the request before touching the device, so that an oversized one is refused by name.
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS) return fail(LQ_ERR_SHAPE, "n_dims %d outside 0..%d", n_dims, LQ_MAX_DIMS);
  if (n_dims > 0 && !dim_rows) return fail(LQ_ERR_NULL, "fks or dim_rows is NULL");
  int32_t cards[LQ_MAX_DIMS];
  for (int k = 0; k < n_dims; ++k) cards[k] = (dim_code && dim_code[k] && group_card) ? group_card[k] : 1;
  const size_t need = lq_groupby_workspace_bytes(n_dims, dim_rows, cards, n_measures);
  if (need > LQ_STATIC_SCRATCH_BYTES)
    return fail(LQ_ERR_WORKSPACE,
                "this query needs %zu bytes of scratch, the allocation-free entry point holds %u: use "
                "lq_masked_groupby_sum with a workspace", need, (unsigned)LQ_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  int rc = static_scratch(&ws);
  if (rc) return rc;
  // need == 0 means invalid sizes: the shared validation below names the argument.
  return groupby_sum_checked(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, fact_mask,
                             n_measures, measures, sums, counts, ws, LQ_STATIC_SCRATCH_BYTES, 0u, hip_stream);
}

size_t lq_groupby_agg_workspace_bytes(int32_t n_dims, const int64_t* dim_rows, const int32_t* group_card,
                                      int32_t n_measures) {
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS || (n_dims > 0 && !dim_rows)) return 0;
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES) return 0;
  int64_t G = 1;
  for (int k = 0; k < n_dims; ++k) {
    if (dim_rows[k] < 0) return 0;
    if (group_card) {
      if (group_card[k] < 1 || group_card[k] > 65535) return 0;
      G *= group_card[k];
      if (G > LQ_MAX_GROUPS) return 0;
    }
  }
  return groupby_ws_bytes(n_dims, dim_rows, G * (3 * n_measures + 1));
}

// Aggregates that the plain group-by can compute: one measure that is a column or a difference of two, or two
// columns.  cols: the fact columns to sum; *sub: the result is the first sum minus the second.
static bool agg_as_plain_sums(int32_t n_measures, const lq_measure* measures, const int32_t** cols, int* n_cols, bool* sub) {
  *sub = false;
  *n_cols = 0;
  if (n_measures == 1 && measures[0].op == 2) {
    cols[0] = measures[0].a; cols[1] = measures[0].b; *n_cols = 2; *sub = true;
    return true;
  }
  if (n_measures > 2) return false;
  for (int m = 0; m < n_measures; ++m) {
    if (measures[m].op != 0) return false;
    cols[(*n_cols)++] = measures[m].a;
  }
  return true;
}

size_t lq_groupby_agg_bucket_workspace_bytes(int64_t n_fact, int32_t n_dims, const int64_t* dim_rows,
                                             const int32_t* group_card, int32_t n_measures, const lq_measure* measures) {
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS || (n_dims > 0 && !dim_rows) || !group_card || !measures) return 0;
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES) return 0;
  const int32_t* cols[2];
  int n_cols = 0;
  bool sub = false;
  if (!agg_as_plain_sums(n_measures, measures, cols, &n_cols, &sub)) return 0;
  int64_t G = 1;
  for (int k = 0; k < n_dims; ++k) {
    if (dim_rows[k] < 0 || group_card[k] < 1 || group_card[k] > 65535) return 0;
    G *= group_card[k];
    if (G > LQ_MAX_GROUPS) return 0;
  }
  const size_t big = groupby_bucket_ws_bytes(n_fact, n_dims, dim_rows, G, n_cols);
  if (big == 0) return 0;
  return round_up(big, 256) + (sub ? static_cast<size_t>(G) * 16 : 0);
}

int lq_groupby_agg(int64_t n_fact, int32_t n_dims, const int32_t* const* fks, const int64_t* dim_rows,
                   const uint8_t* const* dim_mask, const int32_t* const* dim_code, const int32_t* group_card,
                   int32_t n_preds, const lq_range_pred* preds, int32_t n_measures, const lq_measure* measures,
                   int64_t* sums, int64_t* mins, int64_t* maxs, int64_t* counts, void* ws, size_t ws_bytes,
                   uint32_t flags, void* hip_stream) {
  clear_error();
  if (n_fact < 0) return fail(LQ_ERR_SHAPE, "n_fact < 0");
  if (n_dims < 0 || n_dims > LQ_MAX_DIMS) return fail(LQ_ERR_SHAPE, "n_dims %d outside 0..%d", n_dims, LQ_MAX_DIMS);
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES) return fail(LQ_ERR_SHAPE, "n_measures %d outside 1..%d", n_measures, LQ_MAX_MEASURES);
  if (n_preds < 0 || n_preds > 4) return fail(LQ_ERR_SHAPE, "n_preds %d outside 0..4", n_preds);
  if (n_dims > 0 && (!fks || !dim_rows)) return fail(LQ_ERR_NULL, "fks or dim_rows is NULL");
  if (!measures || (n_preds > 0 && !preds)) return fail(LQ_ERR_NULL, "measures or preds is NULL");
  if (!sums && !mins && !maxs && !counts) return fail(LQ_ERR_NULL, "no output requested");
  if (!aligned(sums, 8) || !aligned(mins, 8) || !aligned(maxs, 8) || !aligned(counts, 8))
    return fail(LQ_ERR_SHAPE, "outputs are not 8-byte aligned");
  int64_t G = 1;
  for (int k = 0; k < n_dims; ++k) {
    if (n_fact > 0 && !fks[k]) return fail(LQ_ERR_NULL, "fks[%d] is NULL", k);
    if (!aligned(fks[k], 4)) return fail(LQ_ERR_SHAPE, "fks[%d] is not 4-byte aligned", k);
    if (dim_rows[k] < 0 || dim_rows[k] > 0x7fffffffLL) return fail(LQ_ERR_SHAPE, "dim_rows[%d] out of range", k);
    if (dim_code && dim_code[k]) {
      if (!group_card) return fail(LQ_ERR_NULL, "group_card is NULL");
      if (group_card[k] < 1 || group_card[k] > 65535) return fail(LQ_ERR_SHAPE, "group_card[%d] outside 1..65535", k);
      G *= group_card[k];
      if (G > LQ_MAX_GROUPS) return fail(LQ_ERR_UNSUPPORTED, "more than 2^30 groups");
    }
    if (dim_rows[k] == 0 && n_fact > 0 && ((dim_code && dim_code[k]) || (dim_mask && dim_mask[k])))
      return fail(LQ_ERR_SHAPE, "dimension %d has no rows", k);
  }
  for (int m = 0; m < n_measures; ++m) {
    if (measures[m].op < 0 || measures[m].op > 2) return fail(LQ_ERR_SHAPE, "measures[%d].op is unknown", m);
    if (n_fact > 0 && (!measures[m].a || (measures[m].op != 0 && !measures[m].b))) return fail(LQ_ERR_NULL, "measures[%d] lacks a column", m);
    if (!aligned(measures[m].a, 4) || !aligned(measures[m].b, 4)) return fail(LQ_ERR_SHAPE, "measures[%d] is misaligned", m);
  }
  for (int q = 0; q < n_preds; ++q)
    if ((n_fact > 0 && !preds[q].col) || !aligned(preds[q].col, 4)) return fail(LQ_ERR_NULL, "preds[%d].col is NULL or misaligned", q);
  const size_t need = groupby_ws_bytes(n_dims, dim_rows, G * (3 * n_measures + 1));
  if (!ws || !aligned(ws, 256) || ws_bytes < need) return fail(LQ_ERR_WORKSPACE, "aggregate needs a 256-byte aligned workspace of %zu bytes", need);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc;
  if ((flags & LQ_CHECK_FKS) && n_dims > 0 && n_fact > 0)
    if ((rc = check_groupby_fks(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, ws, ws_bytes, s))) return rc;
  // Sums and counts without fact predicates over more groups than LDS holds, given the large workspace: the plain
  // group-by computes them in its bucketed form (SUM(a - b) as SUM(a) - SUM(b), exact in int64).
  if (n_preds == 0 && !mins && !maxs && sums && n_fact > 0) {
    const int32_t* cols[2];
    int n_cols = 0;
    bool sub = false;
    if (agg_as_plain_sums(n_measures, measures, cols, &n_cols, &sub)) {
      const size_t big = round_up(groupby_bucket_ws_bytes(n_fact, n_dims, dim_rows, G, n_cols), 256);
      if (big > 0 && ws_bytes >= big + (sub ? static_cast<size_t>(G) * 16 : 0)) {
        const bool reuse = (flags & LQ_REUSE_SIDE_TABLES) != 0;
        if (!sub)
          return launch_groupby(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, nullptr, n_cols, cols, sums,
                                counts, static_cast<int32_t>(G), ws, big, reuse, s);
        int64_t* two = reinterpret_cast<int64_t*>(static_cast<uint8_t*>(ws) + big);
        if ((rc = launch_groupby(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, nullptr, 2, cols, two, counts,
                                 static_cast<int32_t>(G), ws, big, reuse, s)))
          return rc;
        return launch_group_diff(G, two, sums, s);
      }
    }
  }
  return launch_groupby_agg(n_fact, n_dims, fks, dim_rows, dim_mask, dim_code, group_card, n_preds, preds,
                            n_measures, measures, sums, mins, maxs, counts, static_cast<int32_t>(G), ws,
                            (flags & LQ_REUSE_SIDE_TABLES) != 0, s);
}

int lq_group_avg(int32_t n_measures, int64_t n_groups, const int64_t* sums, const int64_t* counts, double* avgs,
                 void* hip_stream) {
  clear_error();
  if (n_measures < 1 || n_measures > LQ_MAX_MEASURES) return fail(LQ_ERR_SHAPE, "n_measures %d outside 1..%d", n_measures, LQ_MAX_MEASURES);
  if (n_groups < 0 || n_groups > LQ_MAX_GROUPS) return fail(LQ_ERR_SHAPE, "n_groups outside 0..2^30");
  if (n_groups == 0) return LQ_OK;
  if (!sums || !counts || !avgs) return fail(LQ_ERR_NULL, "sums, counts or avgs is NULL");
  if (!aligned(sums, 8) || !aligned(counts, 8) || !aligned(avgs, 8)) return fail(LQ_ERR_SHAPE, "arrays are not 8-byte aligned");
  return launch_group_avg(n_measures, n_groups, sums, counts, avgs, static_cast<hipStream_t>(hip_stream));
}

int lq_stream_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  clear_error();
  if (bytes == 0) return LQ_OK;
  if (!dst || !src) return fail(LQ_ERR_NULL, "dst or src is NULL");
  if (!aligned(dst, 16) || !aligned(src, 16) || bytes % 16)
    return fail(LQ_ERR_SHAPE, "stream copy needs 16-byte aligned pointers and size");
  return launch_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
