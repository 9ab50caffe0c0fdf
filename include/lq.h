/*
 * lq - star-schema joins as foreign-key indicator products, fused with model
 * prediction, and relational aggregates as linear algebra, for AMD gfx950.
 *
 * The calls follow "Accelerating Machine Learning Queries with Linear Algebra
 * Query Processing" (SSDBM 2023).  Notation (Table 1 of the paper): n fact
 * rows (the paper's i), K dimension tables, D_k of r_k rows and c_k columns,
 * c_f feature columns owned by the fact table, k = c_f + sum c_k the joined
 * width, L (here W[0]) the first linear operator of the model with l outputs,
 * I_k in {0,1}^(n x r_k) the row-mapping matrix of dimension k.
 *
 * Conventions shared by every call
 *   - Every `data` / array pointer is a DEVICE pointer unless the comment says
 *     host.  Descriptor structs and the small pointer arrays inside them live
 *     on the host.  All matrices are row-major with leading dimension `ld` in
 *     elements (ld >= cols).
 *   - I_k is never stored as a matrix: because a fact row matches exactly one
 *     row of each dimension (Section 2.3.3: one 1 per materialised row),
 *     I_k is the int32 column fks[k][i] in [0, r_k), already mapped from key
 *     values to 0-based dimension row numbers.
 *   - The library owns no memory.  Inputs are read-only, outputs and
 *     workspaces are caller-allocated, and nothing is kept between calls.
 *   - Calls validate on the host, enqueue kernels on `hip_stream` (a
 *     hipStream_t passed as void*, NULL = the default stream) and return
 *     without waiting; outputs are valid once the stream has been
 *     synchronised.  Calls on one stream run in order.
 *   - Return value: LQ_OK or an lq_status; on an error nothing has been
 *     enqueued and lq_last_error() (thread-local, host) describes it.  No C++
 *     exception crosses this boundary.
 *   - With LQ_CHECK_FKS a call first verifies on the device that every foreign
 *     key is in range, waits for that check, and returns LQ_ERR_FK_RANGE
 *     without touching the outputs if one is not.  Without the flag, keys are
 *     trusted (referential integrity of the star schema, Section 3.1) and an
 *     out-of-range key is undefined behaviour.
 */
#ifndef LQ_H_
#define LQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LQ_OK = 0,
  LQ_ERR_NULL = 1,        /* a required pointer is NULL */
  LQ_ERR_SHAPE = 2,       /* sizes do not fit together */
  LQ_ERR_DTYPE = 3,       /* unsupported element type or mix of types */
  LQ_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small */
  LQ_ERR_FK_RANGE = 5,    /* LQ_CHECK_FKS found a key outside its table */
  LQ_ERR_UNSUPPORTED = 6, /* valid request this build cannot run */
  LQ_ERR_HIP = 7,         /* the HIP runtime reported an error */
  LQ_ERR_DUPLICATE_KEY = 8 /* LQ_CHECK_KEYS found a dimension key twice */
} lq_status;

typedef enum { LQ_F32 = 0, LQ_BF16 = 1 } lq_dtype;

/* flags */
#define LQ_CHECK_FKS 1u
#define LQ_CHECK_KEYS 2u
/* lq_masked_groupby_sum / lq_groupby_agg: the caller states that the previous call of the same
 * entry point with this workspace had the same dim_rows, dim_mask, dim_code and group_card (same
 * pointers, unchanged contents) and the same n_measures, and that nothing else wrote to the
 * workspace since.  The call then skips re-encoding the dimension side tables (the pushed-down
 * selection vectors and group codes of Sections 2.2-2.4) and goes straight to the fact scan: a
 * dashboard that re-runs a query over new fact rows, or with another fact_mask or other measures
 * columns, pays for the dimension side once.  Results are undefined if the statement is false. */
#define LQ_REUSE_SIDE_TABLES 4u
/* Testing aid for lq_fused_join_predict: run the shape-agnostic kernel even where a
 * specialised one exists, so that the two can be compared. */
#define LQ_FORCE_GENERIC 0x100u
/* Likewise: run the LDS-tiled matrix-core MLP kernel where it covers the shape. */
#define LQ_FORCE_TILE 0x200u

/* which_call values of lq_workspace_bytes */
#define LQ_CALL_FUSED 1
#define LQ_CALL_MATERIALIZED 2

#define LQ_MAX_DIMS 8
#define LQ_MAX_LAYERS 8
#define LQ_MAX_MEASURES 4
#define LQ_MAX_GROUPS (1 << 30)

/* A row-major matrix on the device. */
typedef struct {
  void*   data;   /* device; may be NULL only when rows*cols == 0 */
  int64_t rows;
  int32_t cols;
  int64_t ld;     /* elements between consecutive rows, >= cols */
  int32_t dtype;  /* lq_dtype */
} lq_mat;

/* The star schema after key mapping (Section 3.1: fact table A, dimensions B, C, D). */
typedef struct {
  int64_t               n_fact; /* n */
  lq_mat                fact;   /* X_f [n x c_f]; cols == 0 allowed (data ignored) */
  int32_t               n_dims; /* K in 0..LQ_MAX_DIMS */
  const lq_mat*         dims;   /* host array of K descriptors, D_k [r_k x c_k] */
  const int32_t* const* fks;    /* host array of K device pointers, fks[k] has n int32 */
} lq_star;

/*
 * The model: a linear operator (n_layers == 1) or a ReLU MLP.
 * W[0] is [(c_f + sum c_k) x l_1]; its rows are ordered like the columns of the
 * joined table T: fact columns first, then dimension 0, 1, ... (the column
 * mapping matrices M_k of Section 2.1 place D_k's columns side by side, so
 * M_k L is simply a block of c_k consecutive rows of L).
 * W[j] is [l_j x l_(j+1)].  ReLU follows every layer but the last.
 * bias[j] is NULL or l_(j+1) elements of W[j]'s dtype, added once after the sum.
 * All of fact, dims and W share one dtype (f32 or bf16).
 */
typedef struct {
  int32_t            n_layers; /* 1..LQ_MAX_LAYERS */
  const lq_mat*      W;        /* host array of n_layers descriptors */
  const void* const* bias;     /* host array of n_layers device pointers, or NULL */
} lq_model;

/*
 * Pre-fusion stage (the underlined terms of Eq. 1): P_k = D_k M_k L, i.e.
 * D_k times rows [c_f + c_0 + .. + c_(k-1), +c_k) of W[0], accumulated in fp32.
 *   P  host array of K descriptors; P[k] must be preallocated [r_k x l_1] with
 *      dtype f32 (any model dtype) or bf16 (bf16 models only; rounded once to
 *      nearest-even on store).
 * Needs no workspace.  Run it again whenever a dimension table or W[0] changes.
 */
int lq_project_dims(const lq_star* star, const lq_model* model, lq_mat* P, void* hip_stream);

/*
 * Incremental pre-fusion: recompute only rows [first_row, first_row + n_rows) of P[dim] after those
 * rows of dimension `dim` changed (the pre-fused tables are "constants in a period", Section 3.2;
 * the cost of refreshing them is the trade-off discussed with Q6 and Q8).  Same result as running
 * lq_project_dims again, restricted to those rows.
 */
int lq_project_dim_rows(const lq_star* star, const lq_model* model, lq_mat* P, int32_t dim,
                        int64_t first_row, int64_t n_rows, void* hip_stream);

/*
 * The complexity model of Section 3.2.1 evaluated for a concrete star schema and model (host only,
 * nothing is enqueued; only shapes are read).  With k the joined width, l = l_1, i = n_fact:
 *   cost_no_fusion = sum_j c_j k r_j + i k sum_j r_j + i k l        (C_mmjoin + C_op)
 *   cost_fusion    = i l sum_j r_j                                   (C_fusion)
 *   ratio          = cost_no_fusion / cost_fusion                    (Eq. 3 for equal c_j, K = 3)
 *   cost_prefusion = sum_j r_j c_j l                                 (D_j M_j L, paid per update)
 *   memory_growth  = sum_j r_j l / sum_j r_j c_j                     (> 1 when l exceeds the columns, Q6)
 * bytes_per_row_*  what one fact row moves in this library's kernels (one nonzero per row of I_k).
 * seconds_*        the time model the decision uses.  The dense model above prices I_k as an n x r_k
 *                  matrix and ends at "fuse when k > l" (Eq. 3); this library stores I_k as one key per
 *                  fact row, so the fused join stage stays ahead well below k = l (its gathers come out
 *                  of the caches while the non-fused pipeline writes T to memory and reads it back).
 *                  Each pipeline is priced by what it streams, gathers and multiplies per fact row at
 *                  the rates these kernels sustain on an MI355X (about 5 TB/s streamed, 14 TB/s
 *                  gathered while the tables fit the Infinity Cache and 3 TB/s in 128-byte lines
 *                  beyond it, 60 / 400 TFLOP/s fp32 / bf16 in the dense products, 4 us per launch).
 *   fuse           = 1 when queries_per_update * (seconds_no_fusion - seconds_fused) > seconds_prefusion
 */
typedef struct {
  double cost_no_fusion, cost_fusion, cost_prefusion;
  double ratio, ratio_leading_term, memory_growth;
  double bytes_per_row_fused, bytes_per_row_no_fusion;
  int32_t fuse;
  double seconds_fused, seconds_no_fusion, seconds_prefusion;
} lq_advice;
int lq_fusion_advice(const lq_star* star, const lq_model* model, double queries_per_update,
                     lq_advice* out);

/*
 * Join-computation stage (last line of Eq. 1) with the rest of the model fused in:
 *   z_i = x_i W[0][0:c_f, :] + sum_k P_k[fks[k][i], :] + bias[0]
 *   y_i = z_i for a linear operator; otherwise ReLU and the remaining layers are
 *   applied to z_i in registers/LDS (a non-linearity that follows a reduction
 *   cannot be pushed below the sum - the argument Section 3.3.2 makes for the
 *   tree's final comparison).  The joined table is never formed.
 *   P   as produced by lq_project_dims (f32 or bf16).  Any base and row stride give the same results; the fast
 *       kernels need every P[k] 16-byte aligned with a row stride that is a multiple of 16 bytes (4 floats / 8 bf16
 *       values).  For fp32 models that is all: a hidden width that is not a multiple of 4 then runs as fast as its
 *       neighbours, the last 16-byte piece of a row ends in the stride's padding, whose contents are never used (so
 *       allocate [r_k x round_up(l_1, 4)] and pass cols = l_1, ld = round_up(l_1, 4)); for bf16 models the same
 *       holds with multiples of 8 values when the model is linear or has one more layer of up to 4 outputs
 *   Y   [n x l_out], dtype f32 or bf16 (bf16 only for bf16 models), overwritten
 *   ws  256-byte aligned, may be NULL.  Its first 256 bytes serve LQ_CHECK_FKS.  A model of two or more
 *       layers that none of the specialised kernels takes and that has a layer wider than 128 or more than 16
 *       fact columns (a wide first layer followed by a wide or a third layer, e.g. 1024 -> 1024 or
 *       512 -> 64 -> 1) runs in a layered form when ws holds at least
 *       lq_workspace_bytes(LQ_CALL_FUSED, star, model, 256) bytes: the join stage as a linear operator that
 *       stores ReLU(z) for a chunk of rows, then the later layers as dense products on the matrix cores, chunk by
 *       chunk (lq_workspace_bytes(LQ_CALL_FUSED, star, model, chunk_rows) sizes it for a chunk; more rows per
 *       chunk, fewer launches).  Without that room the general kernels run: same results, tens of times slower on
 *       such models
 * star->dims may be NULL here: only n_dims, fks and the row counts in P are used.
 */
int lq_fused_join_predict(const lq_star* star, const lq_model* model, const lq_mat* P,
                          lq_mat* Y, void* ws, size_t ws_bytes, uint32_t flags,
                          void* hip_stream);

/*
 * The non-fused pipeline the paper compares against (first two lines of Eq. 1):
 * T = X_f M_f + sum_k I_k D_k M_k is written to memory chunk by chunk, then the
 * model is applied to T by dense matrix products.
 *   ws  holds the chunk of T ([chunk_rows x k], model dtype); ws_bytes decides
 *       chunk_rows (lq_workspace_bytes(LQ_CALL_MATERIALIZED, .., chunk_rows)
 *       gives the size for a wanted chunk; at least one 256-row chunk is needed).
 */
int lq_materialized_join_predict(const lq_star* star, const lq_model* model, lq_mat* Y,
                                 void* ws, size_t ws_bytes, uint32_t flags, void* hip_stream);

/*
 * A filtered star join with GROUP BY and SUM as linear algebra (Sections 2.2-2.4):
 *   s_i = fact_mask[i] * prod_k dim_mask[k][fks[k][i]]     (selection vectors pushed through I_k)
 *   g_i = mixed-radix number of (dim_code[k][fks[k][i]] : k grouping), last grouping
 *         dimension fastest                                 (group-mapping matrix of Section 2.4)
 *   sums[m][g] = sum_i s_i [g_i == g] measures[m][i],  counts[g] = sum_i s_i [g_i == g]
 * All integer, exact: int32 measures, int64 accumulation.
 *   fks        host array of K device pointers; a key < 0 means "no match" and drops
 *              the row (inner join, Section 2.3.2); keys >= dim_rows[k] are undefined
 *              behaviour unless LQ_CHECK_FKS
 *   dim_rows   host array of K row counts
 *   dim_mask   host array of K device pointers (uint8 [r_k], 0 = filtered out) or NULL
 *              entries / NULL array for "no predicate"
 *   dim_code   host array of K device pointers (int32 [r_k] in [0, group_card[k])) or
 *              NULL entries / NULL array for dimensions that do not group
 *   group_card host array of K cardinalities, each 1..65535 (ignored where dim_code[k] is NULL);
 *              G = product over grouping dimensions <= LQ_MAX_GROUPS.  While G * (n_measures + 1)
 *              <= 8192 every scan workgroup keeps private accumulators in LDS; above that (the
 *              multi-column group-by of Section 2.4.2 multiplies cardinalities) the output arrays
 *              themselves are the accumulators, cleared by the call and updated with device-wide
 *              64-bit atomics, or - when ws_bytes is at least lq_groupby_bucket_workspace_bytes(..) -
 *              the surviving rows are first sorted into buckets of neighbouring groups in the workspace
 *              and each bucket is then added up in LDS by the one workgroup that owns its groups
 *              (several times faster when many rows survive) -- same results every way
 *   fact_mask  uint8 [n] or NULL (4-byte aligned for the fast scans; any alignment works)
 *   measures   host array of n_measures (1..LQ_MAX_MEASURES) device pointers, int32 [n]
 *   sums       int64 [n_measures x G], overwritten;  counts int64 [G] or NULL
 *   ws         lq_groupby_workspace_bytes(..) bytes, 256-byte aligned; holds the encoded side
 *              tables between calls for LQ_REUSE_SIDE_TABLES
 * A code outside [0, group_card[k]) on a dimension row that passes its mask is undefined behaviour
 * unless LQ_CHECK_FKS is set: the checked call also verifies the codes (r_k reads per dimension)
 * and returns LQ_ERR_SHAPE for such a code without touching the outputs.
 */
int lq_masked_groupby_sum(int64_t n_fact, int32_t n_dims, const int32_t* const* fks,
                          const int64_t* dim_rows, const uint8_t* const* dim_mask,
                          const int32_t* const* dim_code, const int32_t* group_card,
                          const uint8_t* fact_mask, int32_t n_measures,
                          const int32_t* const* measures, int64_t* sums, int64_t* counts,
                          void* ws, size_t ws_bytes, uint32_t flags, void* hip_stream);

/*
 * lq_masked_groupby_sum for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results, without ws / ws_bytes: the encoded side tables and the per-workgroup partial sums
 * live in a device array of LQ_STATIC_SCRATCH_BYTES bytes that is part of the library image (each
 * GPU the library runs on holds its copy until the process ends).  The call allocates nothing and
 * calls no allocating routine.
 *   - A query whose lq_groupby_workspace_bytes(..) exceeds LQ_STATIC_SCRATCH_BYTES is refused with
 *     LQ_ERR_WORKSPACE (the SSB-shaped query of 6M fact rows over dimensions of 2,556 / 30,000 /
 *     2,000 / 200,000 rows needs about 1.9 MB; roughly 3.5 million dimension rows in total fit).
 *   - flags must be 0 (LQ_ERR_UNSUPPORTED otherwise).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two host threads) race and give undefined results; calls on one stream are safe.
 *     Nothing in the array has to survive between calls and nothing needs clearing: each call
 *     rewrites the side tables and every partial row it later reads.
 */
#define LQ_STATIC_SCRATCH_BYTES (8u << 20)
size_t lq_static_scratch_bytes(void);
int lq_masked_groupby_sum_static(int64_t n_fact, int32_t n_dims, const int32_t* const* fks,
                                 const int64_t* dim_rows, const uint8_t* const* dim_mask,
                                 const int32_t* const* dim_code, const int32_t* group_card,
                                 const uint8_t* fact_mask, int32_t n_measures,
                                 const int32_t* const* measures, int64_t* sums, int64_t* counts,
                                 uint32_t flags, void* hip_stream);

/*
 * The same aggregate with the rest of the query shapes of the benchmark's query groups: range
 * predicates on fact columns (selection vectors on the fact table, Section 2.2), measures that are
 * a column, the element-wise product or the difference of two columns (computed in int64), and
 * SUM / MIN / MAX / COUNT per group (AVG: lq_group_avg on the sums and counts).  Arguments as for
 * lq_masked_groupby_sum, plus:
 *   preds     host array of n_preds (0..4) predicates: keep row i iff lo <= col[i] <= hi
 *   measures  host array of n_measures (1..LQ_MAX_MEASURES) expressions over device int32 columns
 *   sums, mins, maxs  int64 [n_measures x G], each may be NULL; groups without rows get 0,
 *             INT64_MAX and INT64_MIN;  counts int64 [G] or NULL
 *   G <= LQ_MAX_GROUPS (LDS accumulators while G * (3 * n_measures + 1) <= 8192, the output arrays
 *   themselves beyond that);  ws: lq_groupby_agg_workspace_bytes(..)
 * A call without fact predicates that wants sums and counts only, of one column, two columns or one difference of
 * two columns, over more than 8,192 accumulators, is the plain group-by: given a workspace of
 * lq_groupby_agg_bucket_workspace_bytes(..) bytes (0: does not apply) it runs that call's bucketed form (SUM(a - b)
 * as SUM(a) - SUM(b), exact in int64) -- same results, several times faster when many rows survive.
 */
typedef struct { const int32_t* col; int32_t lo; int32_t hi; } lq_range_pred;
#define LQ_MEASURE_COL 0
#define LQ_MEASURE_MUL 1
#define LQ_MEASURE_SUB 2
typedef struct { int32_t op; const int32_t* a; const int32_t* b; } lq_measure;
int lq_groupby_agg(int64_t n_fact, int32_t n_dims, const int32_t* const* fks, const int64_t* dim_rows,
                   const uint8_t* const* dim_mask, const int32_t* const* dim_code,
                   const int32_t* group_card, int32_t n_preds, const lq_range_pred* preds,
                   int32_t n_measures, const lq_measure* measures, int64_t* sums, int64_t* mins,
                   int64_t* maxs, int64_t* counts, void* ws, size_t ws_bytes, uint32_t flags,
                   void* hip_stream);
size_t lq_groupby_agg_workspace_bytes(int32_t n_dims, const int64_t* dim_rows,
                                      const int32_t* group_card, int32_t n_measures);
size_t lq_groupby_agg_bucket_workspace_bytes(int64_t n_fact, int32_t n_dims, const int64_t* dim_rows,
                                             const int32_t* group_card, int32_t n_measures,
                                             const lq_measure* measures);

/*
 * AVG per group from the SUM and COUNT results of lq_masked_groupby_sum / lq_groupby_agg on the same stream
 * (the aggregation functions applied after the group-mapping product, Section 2.4):
 *   avgs[m][g] = sums[m][g] / counts[g] in fp64 (both converted to double, one division, so exact to the last
 *   bit whenever |sum| < 2^53), NaN for a group without rows.
 *   sums device int64 [n_measures x n_groups], counts device int64 [n_groups], avgs device double, same shape as sums
 */
int lq_group_avg(int32_t n_measures, int64_t n_groups, const int64_t* sums, const int64_t* counts, double* avgs,
                 void* hip_stream);

/* Workspace sizes in bytes (0 on invalid arguments).  For the group-by, group_card[k] must be
 * 1 for dimensions that do not group (group_card may be NULL when none does); the size depends
 * on the number of compute units of the current device. */
size_t lq_workspace_bytes(int which_call, const lq_star* star, const lq_model* model,
                          int64_t chunk_rows);
size_t lq_groupby_workspace_bytes(int32_t n_dims, const int64_t* dim_rows,
                                  const int32_t* group_card, int32_t n_measures);
/* Workspace with which lq_masked_groupby_sum over n_fact rows and more than 8,192 accumulators takes the
 * bucketed form (see group_card above): the size above plus two slots of 4 (1 + n_measures) bytes per fact
 * row and a little per bucket (three or four measures run as two such calls of two measures and are sized for
 * those).  0 when that form does not apply (8,192 accumulators or fewer, 2^31 rows or more, more than 8,192
 * buckets); the call then works with the smaller workspace. */
size_t lq_groupby_bucket_workspace_bytes(int64_t n_fact, int32_t n_dims, const int64_t* dim_rows,
                                         const int32_t* group_card, int32_t n_measures);

/* ---------------------------------------------------------------------------------------
 * Decision trees (Section 3.3).  The tree is given in the matrix form of Section 3.3.1:
 *   feature[q]    column of the joined table T that internal node q tests (the matrix F only
 *                 selects columns: its column q has its single 1 in row feature[q])
 *   threshold[q]  the vector v: node q is true when the tested value is > threshold[q]
 *   H [p x l]     +1 / -1 where node q lies on the path to leaf j on its True / False side, else 0
 * The vector h the result is compared with is the number of +1 entries per column of H (the
 * value R = (T F > v) H takes exactly when that leaf is reached).  All three arrays live on the
 * device.  Paths longer than 255 nodes are not supported.
 * ------------------------------------------------------------------------------------- */
typedef struct {
  int32_t        n_nodes;    /* p >= 1 */
  int32_t        n_leaves;   /* l >= 1 */
  const int32_t* feature;    /* device, [p], values in [0, c_f + sum c_k) */
  const float*   threshold;  /* device, [p] */
  const int8_t*  H;          /* device, [p x l] row-major */
} lq_tree;

/* Row stride (bytes) of the pre-fused tree tables for l leaves: l rounded up to 16. */
int64_t lq_tree_table_ld(int32_t n_leaves);

/*
 * Pre-fusion of a tree (the tables T_j of Eq. 2), one uint8 table [r_k x ld] per dimension.
 * Each dimension evaluates only the nodes whose tested column it owns (a node of another table
 * would otherwise be evaluated on a zero and counted where its threshold is negative).  The
 * tables do not hold the signed partial sums of (D_k M_k F > v) H but the same information
 * shifted to be non-negative: entry [r][j] = number of owned nodes on the path to leaf j whose
 * outcome for row r agrees with the path (+1 nodes true, -1 nodes false).  Summed over the
 * tables (and the fact table's own nodes) it equals the path length exactly when R_j = h_j.
 *   tables  host array of K device pointers, each r_k * ld bytes, ld = lq_tree_table_ld(l)
 *   target  device, ld bytes: path length of leaf j for j < l, 0xFF padding after
 * star->fks is not used.  dims must be f32.
 */
int lq_tree_project_dims(const lq_star* star, const lq_tree* tree, void* const* tables,
                         uint8_t* target, void* hip_stream);

/*
 * Join-computation stage of Eq. 2: per fact row, gather one table row per dimension, add them
 * (plus the agreement counts of nodes that test fact-table columns, evaluated on the spot),
 * compare with `target`.
 *   leaf    device int32 [n] or NULL: the first leaf j with R_j = h_j, -1 if none
 *   onehot  device uint8 [n x l] (row stride l) or NULL: (R == h), the paper's binary encoding
 * star->dims is not used (may be NULL); star->fact is needed only if a node tests a fact column
 * (those nodes are then evaluated per fact row, for the leaves whose table sums leave them
 * possible; the mask form below is several times faster for such trees).
 * flags: LQ_CHECK_FKS checks every key against dims[k].rows first (synchronous; star->dims must then
 * give the row counts, ws a 256-byte aligned buffer of at least 256 bytes) and returns
 * LQ_ERR_FK_RANGE instead of reading outside a table; ws is not used otherwise.
 */
int lq_fused_join_tree(const lq_star* star, const lq_tree* tree, const void* const* tables,
                       const uint8_t* target, int32_t* leaf, uint8_t* onehot, uint32_t flags,
                       void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Leaf masks: a compressed form of the pre-fused tables of Eq. 2 (Section 3.3.2).
 * The agreement count of a dimension for (row r, leaf j) never exceeds the number of nodes that
 * dimension owns on the path to j, and the counts of all owners add up to the path length
 * exactly when each one reaches that maximum.  Bit j of row r of masks[k] says "entry [r][j] of
 * tables[k] equals the number of nodes dimension k owns on the path to leaf j"; the sum over the
 * dimensions followed by `== h` is then a bitwise AND of one mask row per dimension, and the join
 * stage gathers l / 8 bytes per dimension instead of l.
 *   lq_tree_mask_words(l)   words (uint64) per mask row: ceil(l / 64), rounded up to an even number from
 *                           three words on (rows of 16-byte pieces); bits past l are 0
 *   tables  as written by lq_tree_project_dims;  masks  host array of K device pointers,
 *           r_k * words uint64 each;  star->dims gives r_k and c_k, star->fact.cols the number of
 *           joined columns before the first dimension's (no data is read through star)
 */
int64_t lq_tree_mask_words(int32_t n_leaves);
int lq_tree_compress_tables(const lq_star* star, const lq_tree* tree, const void* const* tables,
                            uint64_t* const* masks, void* hip_stream);

/*
 * Incremental pre-fusion of the tree tables: recompute rows [first_row, first_row + n_rows) of
 * tables[dim] - and of masks[dim], when masks is not NULL - after those rows of dimension `dim`
 * changed (the pre-fused tables are constants only for a period, Section 3.2; refreshing them is
 * the cost weighed in the discussion of Q8).  Same result as lq_tree_project_dims followed by
 * lq_tree_compress_tables, restricted to those rows; target and the fact-side masks depend on the
 * tree alone and stay as they are.  Only entry `dim` of tables / masks is used.
 */
int lq_tree_project_dim_rows(const lq_star* star, const lq_tree* tree, void* const* tables,
                             uint64_t* const* masks, int32_t dim, int64_t first_row, int64_t n_rows,
                             void* hip_stream);

/*
 * Nodes that test the fact table's own columns (feature < c_f) cannot be folded into a table before
 * the join.  In the mask form each of them becomes two mask rows - the leaves that stay possible
 * when its test is true (all whose path does not want it false) and when it is false - and the join
 * stage evaluates the test on the fact row and ANDs the row that applies: the part of (T F > v) H
 * that Eq. 2 leaves to the join-computation stage, in the same AND form as the tables.
 *   lq_tree_fact_mask_bytes(p, l)   size of the device buffer (16-byte aligned) that holds them
 *   lq_tree_fact_masks              fills it from feature, threshold and H (no fact data is read);
 *                                   valid for any star with this tree and this c_f
 * The buffer also holds, per leaf, the list of such nodes on its path ({column, wanted outcome,
 * threshold}, with room for 64 entries per leaf on average).  From four mask words on the join first
 * ANDs the dimensions' mask rows and then checks each leaf still possible against its own list (a
 * few comparisons per row for a tree, instead of one AND per fact-side node and mask word); when
 * the lists do not fit in that room they are left out and the join applies the nodes one by one.
 */
int64_t lq_tree_fact_mask_bytes(int32_t n_nodes, int32_t n_leaves);
int lq_tree_fact_masks(int32_t c_f, const lq_tree* tree, void* fact_masks, void* hip_stream);

/*
 * Join-computation stage of Eq. 2 on the leaf masks: per fact row the AND of one mask row per
 * dimension and, when the fact table has columns, of one row per node that tests them; leaf =
 * position of the lowest set bit (-1 if none is set), onehot = the bits as bytes.
 * Results are identical to lq_fused_join_tree.  leaf / onehot as there.
 * fact_masks: the buffer written by lq_tree_fact_masks when star->fact.cols > 0 (star->fact is then
 * read, f32), ignored otherwise (may be NULL).
 * star->dims is optional: when given, only dims[k].rows is read (the number of rows of masks[k]),
 * and mask tables that fit are kept in LDS for the call (it must then not be smaller than any key).
 * flags must be 0: the call has no workspace, LQ_CHECK_FKS returns LQ_ERR_UNSUPPORTED.
 */
int lq_fused_join_tree_masks(const lq_star* star, const lq_tree* tree, const uint64_t* const* masks,
                             const void* fact_masks, int32_t* leaf, uint8_t* onehot, uint32_t flags,
                             void* hip_stream);

/*
 * Non-fused tree pipeline in the matrix form of Section 3.3.1: T is written to the workspace chunk
 * by chunk, then B = (T F > v) (0 / 1), R = B H as a dense product on the matrix cores and
 * (R == h) are evaluated on it.  The workspace holds h, H in bf16 and, per chunk row, a row of T, of
 * B and of R; ws_bytes decides the chunk (at least 256 rows must fit;
 * lq_tree_workspace_bytes(star, tree, chunk_rows) gives the size for a wanted chunk).
 * flags: LQ_CHECK_FKS as for lq_fused_join_tree.
 */
int lq_materialized_join_tree(const lq_star* star, const lq_tree* tree, int32_t* leaf,
                              uint8_t* onehot, void* ws, size_t ws_bytes, uint32_t flags,
                              void* hip_stream);
size_t lq_tree_workspace_bytes(const lq_star* star, const lq_tree* tree, int64_t chunk_rows);

/* ---------------------------------------------------------------------------------------
 * Key -> row mapping (the "domain generation" of the MM-Join, Algorithm 1, and the domain
 * caching proposed with it): turns key VALUES of a fact column into row numbers of a dimension
 * table, i.e. builds the row-matching matrix I of Section 2.3 in the form the calls above take.
 * The cached domain is a hash table over the dimension keys kept in a caller-owned buffer.
 * ------------------------------------------------------------------------------------- */

/* Bytes of a key map that can hold max_keys keys (256-byte aligned buffer; 0 if out of range). */
size_t lq_keymap_bytes(int64_t max_keys);

/*
 * Build the map from the n_keys int32 keys of a dimension (device array; key of row j at keys[j];
 * keys must be unique).  With LQ_CHECK_KEYS the call waits and returns LQ_ERR_DUPLICATE_KEY if a
 * value occurs twice; otherwise a duplicate silently keeps the row that got there first.
 * The map takes one of two forms, decided on the device from the key range: if largest - smallest
 * key is below the number of 4-byte cells of the buffer (at least 4 x max_keys) it is a direct
 * array indexed by key - smallest key, otherwise a hash table.  Lookups give the same answers
 * either way.
 */
int lq_keymap_build(void* table, size_t table_bytes, const int32_t* keys, int64_t n_keys,
                    uint32_t flags, void* hip_stream);

/* Add the keys of rows first_row .. first_row + n_keys - 1 to an existing map (the update of a
 * cached domain).  The map must have been sized for the total number of keys.  A direct map only
 * takes keys inside its window [smallest key at build, + number of cells): a key outside it is
 * not added, and LQ_CHECK_KEYS reports LQ_ERR_WORKSPACE (rebuild the map with all keys then). */
int lq_keymap_insert(void* table, size_t table_bytes, const int32_t* keys, int64_t n_keys,
                     int64_t first_row, uint32_t flags, void* hip_stream);

/* fk[i] = row whose key equals fact_keys[i], or -1 (no match: the row drops out of an inner join). */
int lq_keymap_lookup(const void* table, size_t table_bytes, const int32_t* fact_keys, int64_t n,
                     int32_t* fk, void* hip_stream);

/*
 * The same map for 64-bit key values (device arrays of int64); row numbers stay int32.  The smallest
 * int64 marks an empty slot and is not a legal key (LQ_CHECK_KEYS reports LQ_ERR_UNSUPPORTED for it;
 * a lookup of it gives -1).  Sizes, forms, flags and errors as for the 32-bit entry points.
 */
size_t lq_keymap64_bytes(int64_t max_keys);
int lq_keymap64_build(void* table, size_t table_bytes, const int64_t* keys, int64_t n_keys,
                      uint32_t flags, void* hip_stream);
int lq_keymap64_insert(void* table, size_t table_bytes, const int64_t* keys, int64_t n_keys,
                       int64_t first_row, uint32_t flags, void* hip_stream);
int lq_keymap64_lookup(const void* table, size_t table_bytes, const int64_t* fact_keys, int64_t n,
                       int32_t* fk, void* hip_stream);

/*
 * The row-mapping matrices I_R and I_S of Section 2.3.3 as COO index vectors aligned with
 * m = <0 .. nnz-1>: rows[m] is the fact row and cols[m] the dimension row of materialised row m,
 * in ascending fact-row order.  rows / cols need room for n entries; *nnz (device) receives the
 * number of matches.  ws: lq_compact_workspace_bytes(n) bytes, 256-byte aligned.
 */
int lq_compact_matches(const int32_t* fk, int64_t n, int64_t* rows, int32_t* cols, int64_t* nnz,
                       void* ws, size_t ws_bytes, void* hip_stream);
size_t lq_compact_workspace_bytes(int64_t n);

/*
 * Group discovery for one table (Sections 2.4.1-2.4.2): the groups are the distinct values of an
 * attribute (one column) or the distinct tuples of several (the paper's sort-unique); they are
 * numbered in ascending lexicographic order, first column most significant, signed comparison.
 *   cols      host array of n_cols (1..4) device pointers, int32 [rows]
 *   max_card  most groups the caller has room for (1..65535)
 *   code      device int32 [rows]: out, the group number of every row -- the dim_code argument of
 *             lq_masked_groupby_sum / lq_groupby_agg
 *   values    device int32 [max_card x n_cols], row-major: out, row g = the tuple of group g
 *   card      HOST int32: out, the number of groups -- the matching group_card entry
 *   ws        lq_group_domain_workspace_bytes(rows) bytes, 256-byte aligned
 * The call waits for the stream once (it has to learn the number of groups).  More than max_card
 * groups: LQ_ERR_UNSUPPORTED, code and values are then undefined.  rows == 0 gives *card = 0.
 * Because codes follow the sorted domain, a dense group-by result indexed by them is already in
 * ascending order of the grouping attributes (Section 2.5).
 */
int lq_group_domain(int64_t rows, int32_t n_cols, const int32_t* const* cols, int32_t max_card,
                    int32_t* code, int32_t* values, int32_t* card, void* ws, size_t ws_bytes,
                    void* hip_stream);
size_t lq_group_domain_workspace_bytes(int64_t rows);

/* Sort keys of lq_order_groups. */
#define LQ_KEY_GROUP_COLUMN 0 /* the code of grouping column `index` (position among the grouping dimensions) */
#define LQ_KEY_SUM 1          /* sums[index][g] */
#define LQ_KEY_COUNT 2        /* counts[g] */
typedef struct {
  int32_t kind;       /* LQ_KEY_* */
  int32_t index;
  int32_t descending; /* 0 = ascending */
} lq_sort_key;

/*
 * ORDER BY on the result of lq_masked_groupby_sum / lq_groupby_agg (Section 2.5 covers sorting
 * on the join / grouping keys through the sorted domain; sorting by an aggregate is not linear
 * algebra and is done here on the small dense result).  The populated groups (counts[g] > 0) are
 * put in the order given by keys[0], keys[1], ...; remaining ties go by ascending group index, so
 * the result is unique.  Group g decomposes as a mixed-radix number over group_card, last column
 * fastest, exactly as the group-by builds it.
 *   group_card  host array of the n_group_cols (0..LQ_MAX_DIMS) cardinalities of the grouping
 *               dimensions, in dimension order; G = their product <= 8192 (this limit is final: the
 *               sort runs in one workgroup's LDS; a larger result is ordered by the caller)
 *   sums        device int64 [n_measures x G] (may be NULL if no key uses it); counts device int64 [G]
 *   keys        host array of n_keys (0..4) sort keys
 *   order       device int32 [G]: out, the populated groups in order, then -1s
 *   n_out       device int32: out, the number of populated groups
 * Asynchronous; one small workgroup.
 */
int lq_order_groups(int32_t n_group_cols, const int32_t* group_card, int32_t n_measures,
                    const int64_t* sums, const int64_t* counts, int32_t n_keys,
                    const lq_sort_key* keys, int32_t* order, int32_t* n_out, void* hip_stream);

/*
 * Plain device-to-device copy of `bytes` bytes (16-byte aligned pointers, bytes a
 * multiple of 16) by a grid-stride kernel.  Not part of the method: it is the
 * yardstick the benchmarks use for "what a pure stream reaches on this GPU".
 */
int lq_stream_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/*
 * Two more yardsticks (not part of the method either): what the GPU delivers for the access patterns of the
 * join stage, with none of its arithmetic.  Nothing is written; `sink` is 16 bytes of device memory that the
 * kernels only name.
 *   lq_yardstick_read    reads `bytes` bytes (multiple of 16, 16-byte aligned) `repeats` times in one launch:
 *                        a buffer that fits the Infinity Cache gives that cache's read rate, a large one HBM's
 *   lq_yardstick_stream  the same reads and, in the same launch, wbytes bytes of zeros written to wbuf: a pure
 *                        stream with the read : write mix of a kernel under study
 *   lq_yardstick_gather  n_gathers random row reads from a table of `rows` rows of row_bytes bytes each (a
 *                        power of two, 16 .. 1024; a row is fetched by adjacent lanes as one contiguous run,
 *                        eight rows in flight per lane).  keys == NULL: row numbers are hashed from the
 *                        gather's index and `seed` (uniform; no other memory traffic); otherwise
 *                        keys[0 .. n_gathers) are the row numbers (their 4 bytes per gather are streamed)
 */
int lq_yardstick_read(const void* buf, size_t bytes, int32_t repeats, void* sink, void* hip_stream);
int lq_yardstick_stream(const void* buf, size_t bytes, int32_t repeats, void* wbuf, size_t wbytes, void* sink,
                        void* hip_stream);
int lq_yardstick_gather(const void* table, int64_t rows, int32_t row_bytes, int64_t n_gathers,
                        const int32_t* keys, uint32_t seed, void* sink, void* hip_stream);

/*
 * Arithmetic yardstick (not part of the method): on every SIMD of the device, waves_per_simd (1..8)
 * wavefronts each run `iters` iterations of 16 fp32 16x16x4 matrix instructions followed by vector_ops
 * (0, 32, 64 or 128) independent fp32 vector multiply-adds.  Timed with vector_ops = 0 it gives the matrix
 * rate; the extra time with vector_ops > 0, against 4 cycles per vector instruction, says how much of the
 * vector work the matrix instructions hide: the roof of the kernels that run later layers on the matrix
 * cores between gathers and sums.  sink: device memory of at least compute units * waves_per_simd * 1024
 * bytes (sink_bytes says how many there are), overwritten.
 */
int lq_yardstick_matrix(int32_t vector_ops, int32_t waves_per_simd, int32_t iters, void* sink, size_t sink_bytes,
                        void* hip_stream);

/* Description of the last error on this host thread ("" if none). */
const char* lq_last_error(void);

/* Library version string. */
const char* lq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LQ_H_ */
