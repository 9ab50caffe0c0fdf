"""ctypes binding of liblq.so: same names as the C entry points, argument marshalling only.

torch is used for device memory (inputs, outputs, workspaces) and for the current
stream handle; every arithmetic step runs inside the library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblq.so")

LQ_OK = 0
LQ_CHECK_FKS = 1
LQ_FORCE_GENERIC = 0x100
LQ_FORCE_TILE = 0x200
LQ_CALL_FUSED = 1
LQ_CALL_MATERIALIZED = 2
LQ_F32, LQ_BF16 = 0, 1
LQ_CHECK_KEYS = 2
LQ_REUSE_SIDE_TABLES = 4
LQ_KEY_GROUP_COLUMN, LQ_KEY_SUM, LQ_KEY_COUNT = 0, 1, 2
_STATUS = {8: "LQ_ERR_DUPLICATE_KEY", 1: "LQ_ERR_NULL", 2: "LQ_ERR_SHAPE", 3: "LQ_ERR_DTYPE", 4: "LQ_ERR_WORKSPACE",
           5: "LQ_ERR_FK_RANGE", 6: "LQ_ERR_UNSUPPORTED", 7: "LQ_ERR_HIP"}


class LQError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code
        self.status = _STATUS.get(code, str(code))


class lq_mat(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int32),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int32)]


class lq_star(ctypes.Structure):
    _fields_ = [("n_fact", ctypes.c_int64), ("fact", lq_mat), ("n_dims", ctypes.c_int32),
                ("dims", ctypes.POINTER(lq_mat)), ("fks", ctypes.POINTER(ctypes.c_void_p))]


class lq_range_pred(ctypes.Structure):
    _fields_ = [("col", ctypes.c_void_p), ("lo", ctypes.c_int32), ("hi", ctypes.c_int32)]


class lq_measure(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("a", ctypes.c_void_p), ("b", ctypes.c_void_p)]


class lq_sort_key(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("index", ctypes.c_int32), ("descending", ctypes.c_int32)]


class lq_advice(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("cost_no_fusion", "cost_fusion", "cost_prefusion", "ratio",
                                               "ratio_leading_term", "memory_growth", "bytes_per_row_fused",
                                               "bytes_per_row_no_fusion")] + [("fuse", ctypes.c_int32)] + [
        (n, ctypes.c_double) for n in ("seconds_fused", "seconds_no_fusion", "seconds_prefusion")]


class lq_tree(ctypes.Structure):
    _fields_ = [("n_nodes", ctypes.c_int32), ("n_leaves", ctypes.c_int32), ("feature", ctypes.c_void_p),
                ("threshold", ctypes.c_void_p), ("H", ctypes.c_void_p)]


class lq_model(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("W", ctypes.POINTER(lq_mat)),
                ("bias", ctypes.POINTER(ctypes.c_void_p))]


def lib_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2306_08367_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, u32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_size_t
    pm, ps, pmod = ctypes.POINTER(lq_mat), ctypes.POINTER(lq_star), ctypes.POINTER(lq_model)
    lib.lq_project_dims.argtypes = [ps, pmod, pm, vp]
    lib.lq_fused_join_predict.argtypes = [ps, pmod, pm, pm, vp, sz, u32, vp]
    lib.lq_materialized_join_predict.argtypes = [ps, pmod, pm, vp, sz, u32, vp]
    lib.lq_masked_groupby_sum.argtypes = [i64, i32, ctypes.POINTER(vp), ctypes.POINTER(i64),
                                          ctypes.POINTER(vp), ctypes.POINTER(vp),
                                          ctypes.POINTER(i32), vp, i32, ctypes.POINTER(vp), vp, vp,
                                          vp, sz, u32, vp]
    lib.lq_masked_groupby_sum_static.argtypes = [i64, i32, ctypes.POINTER(vp), ctypes.POINTER(i64),
                                                 ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                 ctypes.POINTER(i32), vp, i32, ctypes.POINTER(vp), vp, vp,
                                                 u32, vp]
    lib.lq_masked_groupby_sum_static.restype = ctypes.c_int
    lib.lq_static_scratch_bytes.argtypes = []
    lib.lq_static_scratch_bytes.restype = sz
    lib.lq_workspace_bytes.argtypes = [ctypes.c_int, ps, pmod, i64]
    lib.lq_workspace_bytes.restype = sz
    lib.lq_groupby_workspace_bytes.argtypes = [i32, ctypes.POINTER(i64), ctypes.POINTER(i32), i32]
    lib.lq_groupby_workspace_bytes.restype = sz
    lib.lq_groupby_bucket_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(i64), ctypes.POINTER(i32), i32]
    lib.lq_groupby_bucket_workspace_bytes.restype = sz
    lib.lq_stream_copy.argtypes = [vp, vp, sz, vp]
    lib.lq_group_avg.argtypes = [i32, i64, vp, vp, vp, vp]
    lib.lq_group_avg.restype = ctypes.c_int
    lib.lq_yardstick_read.argtypes = [vp, sz, i32, vp, vp]
    lib.lq_yardstick_read.restype = ctypes.c_int
    lib.lq_yardstick_stream.argtypes = [vp, sz, i32, vp, sz, vp, vp]
    lib.lq_yardstick_stream.restype = ctypes.c_int
    lib.lq_yardstick_gather.argtypes = [vp, i64, i32, i64, vp, u32, vp, vp]
    lib.lq_yardstick_gather.restype = ctypes.c_int
    lib.lq_yardstick_matrix.argtypes = [i32, i32, i32, vp, sz, vp]
    lib.lq_yardstick_matrix.restype = ctypes.c_int
    lib.lq_groupby_agg.argtypes = [i64, i32, ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.POINTER(vp),
                                   ctypes.POINTER(vp), ctypes.POINTER(i32), i32, ctypes.POINTER(lq_range_pred),
                                   i32, ctypes.POINTER(lq_measure), vp, vp, vp, vp, vp, sz, u32, vp]
    lib.lq_groupby_agg.restype = ctypes.c_int
    lib.lq_groupby_agg_workspace_bytes.argtypes = [i32, ctypes.POINTER(i64), ctypes.POINTER(i32), i32]
    lib.lq_groupby_agg_workspace_bytes.restype = sz
    lib.lq_groupby_agg_bucket_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(i64), ctypes.POINTER(i32), i32, vp]
    lib.lq_groupby_agg_bucket_workspace_bytes.restype = sz
    lib.lq_project_dim_rows.argtypes = [ps, pmod, pm, i32, i64, i64, vp]
    lib.lq_project_dim_rows.restype = ctypes.c_int
    lib.lq_fusion_advice.argtypes = [ps, pmod, ctypes.c_double, ctypes.POINTER(lq_advice)]
    lib.lq_fusion_advice.restype = ctypes.c_int
    lib.lq_keymap_bytes.argtypes = [i64]
    lib.lq_keymap_bytes.restype = sz
    lib.lq_keymap_build.argtypes = [vp, sz, vp, i64, u32, vp]
    lib.lq_keymap_insert.argtypes = [vp, sz, vp, i64, i64, u32, vp]
    lib.lq_keymap_lookup.argtypes = [vp, sz, vp, i64, vp, vp]
    lib.lq_keymap64_bytes.argtypes = [i64]
    lib.lq_keymap64_bytes.restype = sz
    lib.lq_keymap64_build.argtypes = [vp, sz, vp, i64, u32, vp]
    lib.lq_keymap64_insert.argtypes = [vp, sz, vp, i64, i64, u32, vp]
    lib.lq_keymap64_lookup.argtypes = [vp, sz, vp, i64, vp, vp]
    for f in ("lq_keymap64_build", "lq_keymap64_insert", "lq_keymap64_lookup"):
        getattr(lib, f).restype = ctypes.c_int
    lib.lq_compact_matches.argtypes = [vp, i64, vp, vp, vp, vp, sz, vp]
    lib.lq_compact_workspace_bytes.argtypes = [i64]
    lib.lq_compact_workspace_bytes.restype = sz
    lib.lq_group_domain.argtypes = [i64, i32, ctypes.POINTER(vp), i32, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.lq_group_domain.restype = ctypes.c_int
    lib.lq_group_domain_workspace_bytes.argtypes = [i64]
    lib.lq_group_domain_workspace_bytes.restype = sz
    lib.lq_order_groups.argtypes = [i32, ctypes.POINTER(i32), i32, vp, vp, i32, ctypes.POINTER(lq_sort_key), vp, vp, vp]
    lib.lq_order_groups.restype = ctypes.c_int
    pt = ctypes.POINTER(lq_tree)
    lib.lq_tree_table_ld.argtypes = [i32]
    lib.lq_tree_table_ld.restype = i64
    lib.lq_tree_project_dims.argtypes = [ps, pt, ctypes.POINTER(vp), vp, vp]
    lib.lq_fused_join_tree.argtypes = [ps, pt, ctypes.POINTER(vp), vp, vp, vp, u32, vp, sz, vp]
    lib.lq_materialized_join_tree.argtypes = [ps, pt, vp, vp, vp, sz, u32, vp]
    lib.lq_tree_mask_words.argtypes = [i32]
    lib.lq_tree_mask_words.restype = i64
    lib.lq_tree_compress_tables.argtypes = [ps, pt, ctypes.POINTER(vp), ctypes.POINTER(vp), vp]
    lib.lq_tree_compress_tables.restype = ctypes.c_int
    lib.lq_tree_project_dim_rows.argtypes = [ps, pt, ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i64, i64, vp]
    lib.lq_tree_project_dim_rows.restype = ctypes.c_int
    lib.lq_tree_fact_mask_bytes.argtypes = [i32, i32]
    lib.lq_tree_fact_mask_bytes.restype = i64
    lib.lq_tree_fact_masks.argtypes = [i32, pt, vp, vp]
    lib.lq_tree_fact_masks.restype = ctypes.c_int
    lib.lq_fused_join_tree_masks.argtypes = [ps, pt, ctypes.POINTER(vp), vp, vp, vp, u32, vp]
    lib.lq_fused_join_tree_masks.restype = ctypes.c_int
    lib.lq_tree_workspace_bytes.argtypes = [ps, pt, i64]
    lib.lq_tree_workspace_bytes.restype = sz
    lib.lq_last_error.restype = ctypes.c_char_p
    lib.lq_version.restype = ctypes.c_char_p
    for f in ("lq_project_dims", "lq_fused_join_predict", "lq_materialized_join_predict",
              "lq_masked_groupby_sum", "lq_stream_copy", "lq_tree_project_dims", "lq_fused_join_tree",
              "lq_materialized_join_tree", "lq_keymap_build", "lq_keymap_insert", "lq_keymap_lookup",
              "lq_compact_matches"):
        getattr(lib, f).restype = ctypes.c_int
    return lib


_lib = _load()


def lq_last_error() -> str:
    return _lib.lq_last_error().decode()


def lq_version() -> str:
    return _lib.lq_version().decode()


def _check(rc: int):
    if rc != LQ_OK:
        raise LQError(rc, lq_last_error())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LQ_F32
    if t.dtype == torch.bfloat16:
        return LQ_BF16
    raise TypeError(f"unsupported dtype {t.dtype} (float32 or bfloat16)")


def _mat(t: Optional[torch.Tensor], rows: int = 0, cols: int = 0, dtype: int = LQ_F32) -> lq_mat:
    if t is None:
        return lq_mat(None, rows, cols, max(cols, 1), dtype)
    shape = t.shape
    if len(shape) != 2:
        raise ValueError("matrices are 2-D tensors")
    r, c = shape
    if r == 0 or c == 0:
        return lq_mat(None, r, c, max(c, 1), _dtype_code(t))
    s0, s1 = t.stride()
    if c > 1 and s1 != 1:
        raise ValueError("matrix columns must be contiguous (row-major)")
    ld = s0 if (r > 1 or s0 >= c) else max(c, 1)
    if r > 1 and ld < c:
        raise ValueError("row stride smaller than the row")
    return lq_mat(t.data_ptr(), r, c, ld, _dtype_code(t))


def _mat_array(ts: Sequence[torch.Tensor]):
    arr = (lq_mat * max(1, len(ts)))()
    for j, t in enumerate(ts):
        arr[j] = _mat(t)
    return arr


def _ptr_array(ts: Sequence[Optional[torch.Tensor]]):
    arr = (ctypes.c_void_p * max(1, len(ts)))()
    for j, t in enumerate(ts):
        arr[j] = None if t is None else t.data_ptr()
    return arr


def _stream(stream) -> Optional[int]:
    if stream is None:     # the raw handle of torch's current stream, without building a Stream object
        return int(torch._C._cuda_getCurrentRawStream(torch._C._cuda_getDevice())) or None
    return int(stream.cuda_stream) or None


def _empty(stream, *shape, **kw) -> torch.Tensor:
    """torch.empty for outputs and workspaces of a call that runs on `stream`.  torch hands a freed block to
    the next allocation on the stream it was allocated on; when the kernels run on another stream the block is
    marked as in use there, so that it is not recycled while they still read or write it."""
    t = torch.empty(*shape, **kw)
    if stream is not None and t.is_cuda and t.numel() > 0:
        t.record_stream(stream)
    return t


def _expect(t: torch.Tensor, dtype, what: str):
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError(f"{what} must live on the GPU")
    if t.dim() == 1 and t.numel() > 1 and t.stride(0) != 1:
        raise ValueError(f"{what} must be contiguous")


class _Star:
    """Keeps the ctypes arrays of a star schema alive for the duration of a call."""

    def __init__(self, n: int, X, dims, fks, n_dims: Optional[int] = None):
        self.keep = [X, dims, fks]
        K = len(fks) if n_dims is None else n_dims
        for f in fks:
            _expect(f, torch.int32, "foreign-key column")
        self.dims_arr = _mat_array(dims) if dims is not None else None
        self.fks_arr = _ptr_array(fks)
        fact = _mat(X) if X is not None else _mat(None, n, 0)
        self.c = lq_star(n, fact, K,
                         self.dims_arr if dims is not None else ctypes.POINTER(lq_mat)(),
                         self.fks_arr)


class _Model:
    def __init__(self, weights, biases):
        self.keep = [weights, biases]
        self.W = _mat_array(weights)
        self.b = _ptr_array(biases if biases is not None else [None] * len(weights))
        self.c = lq_model(len(weights), self.W, self.b)


def _n_of(X, fks) -> int:
    if X is not None:
        return int(X.shape[0])
    if fks:
        return int(fks[0].shape[0])
    raise ValueError("need fact columns or at least one foreign-key column")


def lq_project_dims(dims: Sequence[torch.Tensor], W0: torch.Tensor, c_f: int,
                    P: Optional[List[torch.Tensor]] = None, p_dtype: Optional[torch.dtype] = None,
                    stream=None) -> List[torch.Tensor]:
    """P_k = D_k times its rows of W0 (pre-fusion stage).  Allocates P unless given: in the model's element type
    unless p_dtype says otherwise (the specialised kernels of the join stage take tables of the model's type;
    fp32 tables under a bf16 model run on the shape-agnostic kernel, several times slower)."""
    if P is None:
        # rows start 16 bytes apart at the least (the stride is padded to 4 floats / 8 bf16 values): the fast kernels of
        # the join stage then take any hidden width, the padding is never read as data
        pd = p_dtype or W0.dtype
        per16 = 4 if pd == torch.float32 else 8
        l1 = int(W0.shape[1])
        ld = (l1 + per16 - 1) // per16 * per16
        P = [_empty(stream, (d.shape[0], ld), dtype=pd, device=d.device)[:, :l1] for d in dims]
    fact = lq_mat(None, 0, int(c_f), max(int(c_f), 1), _dtype_code(W0))
    dims_arr = _mat_array(dims)
    star = lq_star(0, fact, len(dims), dims_arr, _ptr_array([None] * len(dims)))
    model = _Model([W0], None)
    P_arr = _mat_array(P)
    _check(_lib.lq_project_dims(ctypes.byref(star), ctypes.byref(model.c), P_arr, _stream(stream)))
    return P


def lq_fused_join_predict(X: Optional[torch.Tensor], fks: Sequence[torch.Tensor],
                          P: Sequence[torch.Tensor], weights: Sequence[torch.Tensor],
                          biases: Optional[Sequence[Optional[torch.Tensor]]] = None,
                          Y: Optional[torch.Tensor] = None, y_dtype: Optional[torch.dtype] = None,
                          flags: int = 0, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Y = MLP(x W_f + sum_k P_k[fk_k]) without forming the joined table."""
    n = _n_of(X, fks)
    dev = weights[0].device
    if Y is None:
        Y = _empty(stream, (n, weights[-1].shape[1]), dtype=y_dtype or weights[0].dtype, device=dev)
    star = _Star(n, X, None, fks)
    model = _Model(weights, biases)
    if ws is None and n > 0 and len(weights) >= 2 and (max(int(w.shape[1]) for w in weights) > 128 or
                                                       (X is not None and X.shape[1] > 16)):
        # a model that the fused kernels may not take (a layer wider than 128, more than 16 fact columns): room for the
        # layered form (activations of a chunk of rows, at most a quarter of a gigabyte); the library uses it only if
        # it needs to
        per_row = int(_lib.lq_workspace_bytes(LQ_CALL_FUSED, ctypes.byref(star.c), ctypes.byref(model.c), 256) - 256) // 256
        rows = max(4096, min(n, (256 << 20) // max(per_row, 1)))
        ws = _empty(stream, int(_lib.lq_workspace_bytes(LQ_CALL_FUSED, ctypes.byref(star.c), ctypes.byref(model.c), rows)),
                    dtype=torch.uint8, device=dev)
    if ws is None and (flags & LQ_CHECK_FKS):
        ws = _empty(stream, 256, dtype=torch.uint8, device=dev)
    P_arr = _mat_array(P)
    Ym = _mat(Y)
    _check(_lib.lq_fused_join_predict(ctypes.byref(star.c), ctypes.byref(model.c), P_arr,
                                      ctypes.byref(Ym), None if ws is None else ws.data_ptr(),
                                      0 if ws is None else ws.numel() * ws.element_size(),
                                      flags, _stream(stream)))
    return Y


def lq_workspace_bytes(which_call: int, k: int, weights: Sequence[torch.Tensor], chunk_rows: int) -> int:
    model = _Model(weights, None)
    star = lq_star(0, lq_mat(None, 0, 0, 1, _dtype_code(weights[0])), 0, ctypes.POINTER(lq_mat)(),
                   _ptr_array([]))
    return int(_lib.lq_workspace_bytes(which_call, ctypes.byref(star), ctypes.byref(model.c), chunk_rows))


def lq_materialized_join_predict(X: Optional[torch.Tensor], dims: Sequence[torch.Tensor],
                                 fks: Sequence[torch.Tensor], weights: Sequence[torch.Tensor],
                                 biases: Optional[Sequence[Optional[torch.Tensor]]] = None,
                                 Y: Optional[torch.Tensor] = None, y_dtype: Optional[torch.dtype] = None,
                                 ws: Optional[torch.Tensor] = None, chunk_rows: Optional[int] = None,
                                 flags: int = 0, stream=None) -> torch.Tensor:
    """The non-fused pipeline: write T chunk by chunk, then run the model on it layer by layer."""
    n = _n_of(X, fks)
    dev = weights[0].device
    if Y is None:
        Y = _empty(stream, (n, weights[-1].shape[1]), dtype=y_dtype or weights[0].dtype, device=dev)
    if ws is None:
        rows = chunk_rows or min(max(n, 256), 1 << 22)
        nbytes = lq_workspace_bytes(LQ_CALL_MATERIALIZED, int(weights[0].shape[0]), weights, rows)
        ws = _empty(stream, nbytes, dtype=torch.uint8, device=dev)
    star = _Star(n, X, dims, fks)
    model = _Model(weights, biases)
    Ym = _mat(Y)
    _check(_lib.lq_materialized_join_predict(ctypes.byref(star.c), ctypes.byref(model.c),
                                             ctypes.byref(Ym), ws.data_ptr(),
                                             ws.numel() * ws.element_size(), flags, _stream(stream)))
    return Y


def lq_groupby_workspace_bytes(dim_rows: Sequence[int], group_card: Sequence[int], n_measures: int) -> int:
    K = len(dim_rows)
    rows = (ctypes.c_int64 * max(1, K))(*[int(r) for r in dim_rows])
    card = (ctypes.c_int32 * max(1, K))(*[int(c) for c in group_card])
    return int(_lib.lq_groupby_workspace_bytes(K, rows, card, n_measures))


def lq_groupby_bucket_workspace_bytes(n_fact: int, dim_rows: Sequence[int], group_card: Sequence[int], n_measures: int) -> int:
    """Workspace that lets a group-by over more than 8,192 accumulators take the bucketed form (0: does not apply)."""
    K = len(dim_rows)
    rows = (ctypes.c_int64 * max(1, K))(*[int(r) for r in dim_rows])
    card = (ctypes.c_int32 * max(1, K))(*[int(c) for c in group_card])
    return int(_lib.lq_groupby_bucket_workspace_bytes(int(n_fact), K, rows, card, n_measures))


def lq_masked_groupby_sum(fks: Sequence[torch.Tensor], dim_rows: Sequence[int],
                          dim_mask: Optional[Sequence[Optional[torch.Tensor]]],
                          dim_code: Optional[Sequence[Optional[torch.Tensor]]],
                          group_card: Sequence[int], fact_mask: Optional[torch.Tensor],
                          measures: Sequence[torch.Tensor], sums: Optional[torch.Tensor] = None,
                          counts: Optional[torch.Tensor] = None, want_counts: bool = True,
                          ws: Optional[torch.Tensor] = None, flags: int = 0, stream=None):
    """Filtered star join + GROUP BY + SUM/COUNT.  Returns (sums [M x G] int64, counts [G] int64 or None)."""
    K = len(fks)
    n = int(measures[0].shape[0])
    dev = measures[0].device
    for f in fks:
        _expect(f, torch.int32, "foreign-key column")
        if f.shape[0] != n:
            raise ValueError("foreign-key column length differs from the measures")
    for m in measures:
        _expect(m, torch.int32, "measure column")
    masks = list(dim_mask) if dim_mask is not None else [None] * K
    codes = list(dim_code) if dim_code is not None else [None] * K
    for k in range(K):
        if masks[k] is not None:
            _expect(masks[k], torch.uint8, "dimension mask")
            if masks[k].shape[0] != dim_rows[k]:
                raise ValueError("mask length differs from dim_rows")
        if codes[k] is not None:
            _expect(codes[k], torch.int32, "dimension group code")
            if codes[k].shape[0] != dim_rows[k]:
                raise ValueError("code length differs from dim_rows")
    if fact_mask is not None:
        _expect(fact_mask, torch.uint8, "fact mask")
    G = 1
    for k in range(K):
        if codes[k] is not None:
            G *= int(group_card[k])
    if sums is None:
        sums = _empty(stream, (len(measures), G), dtype=torch.int64, device=dev)
    if counts is None and want_counts:
        counts = _empty(stream, (G,), dtype=torch.int64, device=dev)
    if ws is None:
        eff_card = [int(group_card[k]) if codes[k] is not None else 1 for k in range(K)]
        ws = _empty(stream, max(lq_groupby_workspace_bytes(dim_rows, group_card, len(measures)),
                                lq_groupby_bucket_workspace_bytes(n, dim_rows, eff_card, len(measures))),
                    dtype=torch.uint8, device=dev)
    rows = (ctypes.c_int64 * max(1, K))(*[int(r) for r in dim_rows])
    card = (ctypes.c_int32 * max(1, K))(*[int(c) for c in group_card])
    _check(_lib.lq_masked_groupby_sum(
        n, K, _ptr_array(fks), rows, _ptr_array(masks), _ptr_array(codes), card,
        None if fact_mask is None else fact_mask.data_ptr(), len(measures), _ptr_array(measures),
        sums.data_ptr(), None if counts is None else counts.data_ptr(), ws.data_ptr(),
        ws.numel() * ws.element_size(), flags, _stream(stream)))
    return sums, counts


def lq_static_scratch_bytes() -> int:
    return int(_lib.lq_static_scratch_bytes())


def lq_masked_groupby_sum_static(fks: Sequence[torch.Tensor], dim_rows: Sequence[int],
                                 dim_mask: Optional[Sequence[Optional[torch.Tensor]]],
                                 dim_code: Optional[Sequence[Optional[torch.Tensor]]],
                                 group_card: Sequence[int], fact_mask: Optional[torch.Tensor],
                                 measures: Sequence[torch.Tensor], sums: torch.Tensor,
                                 counts: Optional[torch.Tensor], flags: int = 0, stream=None):
    """lq_masked_groupby_sum without a workspace and without any allocation: the caller brings
    `sums` [M x G] (and `counts` [G] or None), the library's own static device array is the scratch."""
    K = len(fks)
    n = int(measures[0].shape[0])
    for f in fks:
        _expect(f, torch.int32, "foreign-key column")
        if f.shape[0] != n:
            raise ValueError("foreign-key column length differs from the measures")
    for m in measures:
        _expect(m, torch.int32, "measure column")
    masks = list(dim_mask) if dim_mask is not None else [None] * K
    codes = list(dim_code) if dim_code is not None else [None] * K
    for k in range(K):
        if masks[k] is not None:
            _expect(masks[k], torch.uint8, "dimension mask")
            if masks[k].shape[0] != dim_rows[k]:
                raise ValueError("mask length differs from dim_rows")
        if codes[k] is not None:
            _expect(codes[k], torch.int32, "dimension group code")
            if codes[k].shape[0] != dim_rows[k]:
                raise ValueError("code length differs from dim_rows")
    if fact_mask is not None:
        _expect(fact_mask, torch.uint8, "fact mask")
    G = 1
    for k in range(K):
        if codes[k] is not None:
            G *= int(group_card[k])
    _expect(sums, torch.int64, "sums")
    if sums.numel() != len(measures) * G or not sums.is_contiguous():
        raise ValueError("sums must be a contiguous int64 tensor of n_measures x G elements")
    if counts is not None:
        _expect(counts, torch.int64, "counts")
        if counts.numel() != G:
            raise ValueError("counts must have G elements")
    rows = (ctypes.c_int64 * max(1, K))(*[int(r) for r in dim_rows])
    card = (ctypes.c_int32 * max(1, K))(*[int(c) for c in group_card])
    _check(_lib.lq_masked_groupby_sum_static(
        n, K, _ptr_array(fks), rows, _ptr_array(masks), _ptr_array(codes), card,
        None if fact_mask is None else fact_mask.data_ptr(), len(measures), _ptr_array(measures),
        sums.data_ptr(), None if counts is None else counts.data_ptr(), flags, _stream(stream)))
    return sums, counts


def lq_group_avg(sums: torch.Tensor, counts: torch.Tensor, avgs: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """AVG per group = sums / counts in fp64 ([M x G]); NaN where a group has no rows."""
    _expect(sums, torch.int64, "sums")
    _expect(counts, torch.int64, "counts")
    if sums.dim() != 2 or sums.shape[1] != counts.shape[0] or not sums.is_contiguous():
        raise ValueError("sums must be a contiguous [n_measures x G] tensor and counts [G]")
    if avgs is None:
        avgs = _empty(stream, sums.shape, dtype=torch.float64, device=sums.device)
    _expect(avgs, torch.float64, "avgs")
    if avgs.shape != sums.shape or not avgs.is_contiguous():
        raise ValueError("avgs must be contiguous and shaped like sums")
    _check(_lib.lq_group_avg(int(sums.shape[0]), int(sums.shape[1]), sums.data_ptr(), counts.data_ptr(), avgs.data_ptr(),
                             _stream(stream)))
    return avgs


def lq_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("destination smaller than source")
    _check(_lib.lq_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream(stream)))


def lq_yardstick_read(buf: torch.Tensor, repeats: int, sink: torch.Tensor, stream=None) -> None:
    """Reads `buf` `repeats` times in one launch (bandwidth yardstick; nothing is written)."""
    _check(_lib.lq_yardstick_read(buf.data_ptr(), buf.numel() * buf.element_size(), int(repeats), sink.data_ptr(),
                                  _stream(stream)))


def lq_yardstick_stream(buf: torch.Tensor, repeats: int, wbuf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Reads `buf` `repeats` times and overwrites `wbuf` with zeros, in one launch (stream yardstick)."""
    _check(_lib.lq_yardstick_stream(buf.data_ptr(), buf.numel() * buf.element_size(), int(repeats), wbuf.data_ptr(),
                                    wbuf.numel() * wbuf.element_size(), sink.data_ptr(), _stream(stream)))


def lq_yardstick_gather(table: torch.Tensor, row_bytes: int, n_gathers: int, sink: torch.Tensor,
                        keys: Optional[torch.Tensor] = None, seed: int = 1, stream=None) -> None:
    """n_gathers random reads of row_bytes-byte rows of `table` (gather yardstick; nothing is written)."""
    rows = table.numel() * table.element_size() // int(row_bytes)
    if keys is not None:
        _expect(keys, torch.int32, "keys")
        if keys.numel() < n_gathers:
            raise ValueError("fewer keys than gathers")
    _check(_lib.lq_yardstick_gather(table.data_ptr(), rows, int(row_bytes), int(n_gathers),
                                    None if keys is None else keys.data_ptr(), int(seed) & 0xffffffff, sink.data_ptr(),
                                    _stream(stream)))


def lq_yardstick_matrix(vector_ops: int, waves_per_simd: int, iters: int, sink: torch.Tensor, stream=None) -> None:
    """`iters` rounds of 16 fp32 matrix instructions and `vector_ops` vector multiply-adds on every SIMD."""
    _check(_lib.lq_yardstick_matrix(int(vector_ops), int(waves_per_simd), int(iters), sink.data_ptr(),
                                    sink.numel() * sink.element_size(), _stream(stream)))


# ---------------------------------------------------------------- decision trees --------------

def _tree(feature: torch.Tensor, threshold: torch.Tensor, H: torch.Tensor) -> lq_tree:
    _expect(feature, torch.int32, "tree feature index")
    _expect(threshold, torch.float32, "tree thresholds")
    if H.dtype != torch.int8 or not H.is_cuda or H.dim() != 2 or not H.is_contiguous():
        raise TypeError("H must be a contiguous int8 [nodes x leaves] tensor on the GPU")
    if feature.shape[0] != H.shape[0] or threshold.shape[0] != H.shape[0]:
        raise ValueError("feature, threshold and H disagree on the number of nodes")
    return lq_tree(int(H.shape[0]), int(H.shape[1]), feature.data_ptr(), threshold.data_ptr(), H.data_ptr())


def lq_tree_table_ld(n_leaves: int) -> int:
    return int(_lib.lq_tree_table_ld(n_leaves))


def lq_tree_project_dims(dims: Sequence[torch.Tensor], c_f: int, feature, threshold, H, stream=None):
    """Pre-fused tree tables (uint8 [r_k x ld] per dimension) and the target vector (uint8 [ld])."""
    tree = _tree(feature, threshold, H)
    ld = lq_tree_table_ld(tree.n_leaves)
    dev = H.device
    tables = [_empty(stream, (d.shape[0], ld), dtype=torch.uint8, device=dev) for d in dims]
    target = _empty(stream, (ld,), dtype=torch.uint8, device=dev)
    fact = lq_mat(None, 0, int(c_f), max(int(c_f), 1), LQ_F32)
    dims_arr = _mat_array(dims)
    star = lq_star(0, fact, len(dims), dims_arr, _ptr_array([None] * len(dims)))
    _check(_lib.lq_tree_project_dims(ctypes.byref(star), ctypes.byref(tree), _ptr_array(tables),
                                     target.data_ptr(), _stream(stream)))
    return tables, target


def lq_fused_join_tree(X: Optional[torch.Tensor], fks: Sequence[torch.Tensor], tables, target, feature,
                       threshold, H, want_leaf: bool = True, want_onehot: bool = False, flags: int = 0,
                       stream=None):
    """Leaf reached by every fact row (int32 [n]) and / or the one-hot matrix (uint8 [n x l]).
    With LQ_CHECK_FKS the keys are first checked against the row counts of the tables."""
    tree = _tree(feature, threshold, H)
    n = _n_of(X, fks)
    dev = H.device
    leaf = _empty(stream, (n,), dtype=torch.int32, device=dev) if want_leaf else None
    onehot = _empty(stream, (n, tree.n_leaves), dtype=torch.uint8, device=dev) if want_onehot else None
    star = _Star(n, X, None, fks)
    ws = None
    if flags & LQ_CHECK_FKS:
        rows_arr = (lq_mat * max(1, len(tables)))(*[lq_mat(None, int(t.shape[0]), 1, 1, LQ_F32) for t in tables])
        star.c.dims = rows_arr
        ws = _empty(stream, 256, dtype=torch.uint8, device=dev)
    _check(_lib.lq_fused_join_tree(ctypes.byref(star.c), ctypes.byref(tree), _ptr_array(tables),
                                   target.data_ptr(), None if leaf is None else leaf.data_ptr(),
                                   None if onehot is None else onehot.data_ptr(), flags,
                                   None if ws is None else ws.data_ptr(), 0 if ws is None else ws.numel(),
                                   _stream(stream)))
    return leaf, onehot


def lq_tree_mask_words(n_leaves: int) -> int:
    return int(_lib.lq_tree_mask_words(n_leaves))


def lq_tree_compress_tables(dims: Sequence[torch.Tensor], tables, feature, threshold, H, c_f: int = 0, stream=None):
    """Leaf masks (int64 bit patterns [r_k x words] per dimension) of pre-fused tree tables."""
    tree = _tree(feature, threshold, H)
    words = lq_tree_mask_words(tree.n_leaves)
    dev = H.device
    masks = [_empty(stream, (d.shape[0], words), dtype=torch.int64, device=dev) for d in dims]
    fact = lq_mat(None, 0, int(c_f), max(int(c_f), 1), LQ_F32)
    dims_arr = _mat_array(dims)
    star = lq_star(0, fact, len(dims), dims_arr, _ptr_array([None] * len(dims)))
    _check(_lib.lq_tree_compress_tables(ctypes.byref(star), ctypes.byref(tree), _ptr_array(tables), _ptr_array(masks),
                                        _stream(stream)))
    return masks


def lq_tree_project_dim_rows(dims: Sequence[torch.Tensor], c_f: int, tables, masks, feature, threshold, H,
                             dim: int, first_row: int, n_rows: int, stream=None) -> None:
    """Refresh rows [first_row, first_row + n_rows) of tables[dim] (and of masks[dim] unless masks is None) in place."""
    tree = _tree(feature, threshold, H)
    fact = lq_mat(None, 0, int(c_f), max(int(c_f), 1), LQ_F32)
    dims_arr = _mat_array(dims)
    star = lq_star(0, fact, len(dims), dims_arr, _ptr_array([None] * len(dims)))
    _check(_lib.lq_tree_project_dim_rows(ctypes.byref(star), ctypes.byref(tree), _ptr_array(tables),
                                         None if masks is None else _ptr_array(masks), int(dim), int(first_row),
                                         int(n_rows), _stream(stream)))


def lq_tree_fact_mask_bytes(n_nodes: int, n_leaves: int) -> int:
    return int(_lib.lq_tree_fact_mask_bytes(n_nodes, n_leaves))


def lq_tree_fact_masks(c_f: int, feature, threshold, H, stream=None):
    """Packed mask rows (opaque uint8 buffer) of the nodes that test the fact table's own columns."""
    tree = _tree(feature, threshold, H)
    buf = _empty(stream, (lq_tree_fact_mask_bytes(tree.n_nodes, tree.n_leaves),), dtype=torch.uint8, device=H.device)
    _check(_lib.lq_tree_fact_masks(int(c_f), ctypes.byref(tree), buf.data_ptr(), _stream(stream)))
    return buf


def lq_fused_join_tree_masks(fks: Sequence[torch.Tensor], masks, feature, threshold, H, want_leaf: bool = True,
                             want_onehot: bool = False, flags: int = 0, stream=None,
                             X: Optional[torch.Tensor] = None, fact_masks: Optional[torch.Tensor] = None):
    """The join stage on leaf masks: same results as lq_fused_join_tree.  X / fact_masks: the fact
    table's own columns and the buffer of lq_tree_fact_masks, when the tree tests such columns."""
    tree = _tree(feature, threshold, H)
    n = _n_of(X, fks)
    dev = H.device
    leaf = _empty(stream, (n,), dtype=torch.int32, device=dev) if want_leaf else None
    onehot = _empty(stream, (n, tree.n_leaves), dtype=torch.uint8, device=dev) if want_onehot else None
    star = _Star(n, X, None, fks)
    # row counts of the mask tables (the library may then keep small tables in LDS); no data pointers
    rows_arr = (lq_mat * max(1, len(masks)))(*[lq_mat(None, int(m.shape[0]), 1, 1, LQ_F32) for m in masks])
    star.c.dims = rows_arr
    _check(_lib.lq_fused_join_tree_masks(ctypes.byref(star.c), ctypes.byref(tree), _ptr_array(masks),
                                         None if fact_masks is None else fact_masks.data_ptr(),
                                         None if leaf is None else leaf.data_ptr(),
                                         None if onehot is None else onehot.data_ptr(), flags, _stream(stream)))
    return leaf, onehot


def lq_materialized_join_tree(X: Optional[torch.Tensor], dims, fks, feature, threshold, H,
                              want_leaf: bool = True, want_onehot: bool = False,
                              ws: Optional[torch.Tensor] = None, chunk_rows: Optional[int] = None, flags: int = 0,
                              stream=None):
    """Non-fused tree pipeline: materialise T chunk by chunk, then ((T F > v) H) == h."""
    tree = _tree(feature, threshold, H)
    n = _n_of(X, fks)
    dev = H.device
    leaf = _empty(stream, (n,), dtype=torch.int32, device=dev) if want_leaf else None
    onehot = _empty(stream, (n, tree.n_leaves), dtype=torch.uint8, device=dev) if want_onehot else None
    star = _Star(n, X, dims, fks)
    if ws is None:
        rows = chunk_rows or min(max(n, 256), 1 << 22)
        ws = _empty(stream, int(_lib.lq_tree_workspace_bytes(ctypes.byref(star.c), ctypes.byref(tree), rows)), dtype=torch.uint8,
                         device=dev)
    _check(_lib.lq_materialized_join_tree(ctypes.byref(star.c), ctypes.byref(tree),
                                          None if leaf is None else leaf.data_ptr(),
                                          None if onehot is None else onehot.data_ptr(), ws.data_ptr(),
                                          ws.numel(), flags, _stream(stream)))
    return leaf, onehot


# ---------------------------------------------------------------- key -> row mapping ----------

def lq_keymap_bytes(max_keys: int) -> int:
    return int(_lib.lq_keymap_bytes(max_keys))


def lq_keymap_build(keys: torch.Tensor, max_keys: Optional[int] = None, flags: int = 0, stream=None) -> torch.Tensor:
    """Hash map from the key values of a dimension to its row numbers; returns the map buffer."""
    _expect(keys, torch.int32, "dimension key column")
    nbytes = lq_keymap_bytes(max(int(keys.shape[0]), max_keys or 0))
    table = _empty(stream, nbytes, dtype=torch.uint8, device=keys.device)
    _check(_lib.lq_keymap_build(table.data_ptr(), nbytes, keys.data_ptr(), int(keys.shape[0]), flags, _stream(stream)))
    return table


def lq_keymap_insert(table: torch.Tensor, keys: torch.Tensor, first_row: int, flags: int = 0, stream=None) -> None:
    _expect(keys, torch.int32, "dimension key column")
    _check(_lib.lq_keymap_insert(table.data_ptr(), table.numel(), keys.data_ptr(), int(keys.shape[0]),
                                 int(first_row), flags, _stream(stream)))


def lq_keymap_lookup(table: torch.Tensor, fact_keys: torch.Tensor, fk: Optional[torch.Tensor] = None,
                     stream=None) -> torch.Tensor:
    """fk[i] = dimension row whose key equals fact_keys[i], -1 where there is none."""
    _expect(fact_keys, torch.int32, "fact key column")
    if fk is None:
        fk = _empty(stream, fact_keys.shape, dtype=fact_keys.dtype, device=fact_keys.device)
    _check(_lib.lq_keymap_lookup(table.data_ptr(), table.numel(), fact_keys.data_ptr(),
                                 int(fact_keys.shape[0]), fk.data_ptr(), _stream(stream)))
    return fk


def lq_keymap64_bytes(max_keys: int) -> int:
    return int(_lib.lq_keymap64_bytes(int(max_keys)))


def lq_keymap64_build(keys: torch.Tensor, max_keys: Optional[int] = None, flags: int = 0, stream=None) -> torch.Tensor:
    """Map from the int64 key values of a dimension to its row numbers; returns the map buffer."""
    _expect(keys, torch.int64, "dimension key column")
    nbytes = lq_keymap64_bytes(max(int(keys.shape[0]), max_keys or 0))
    table = _empty(stream, nbytes, dtype=torch.uint8, device=keys.device)
    _check(_lib.lq_keymap64_build(table.data_ptr(), nbytes, keys.data_ptr(), int(keys.shape[0]), flags, _stream(stream)))
    return table


def lq_keymap64_insert(table: torch.Tensor, keys: torch.Tensor, first_row: int, flags: int = 0, stream=None) -> None:
    _expect(keys, torch.int64, "dimension key column")
    _check(_lib.lq_keymap64_insert(table.data_ptr(), table.numel(), keys.data_ptr(), int(keys.shape[0]),
                                   int(first_row), flags, _stream(stream)))


def lq_keymap64_lookup(table: torch.Tensor, fact_keys: torch.Tensor, fk: Optional[torch.Tensor] = None,
                       stream=None) -> torch.Tensor:
    """fk[i] = dimension row whose key equals fact_keys[i] (int64), -1 where there is none."""
    _expect(fact_keys, torch.int64, "fact key column")
    if fk is None:
        fk = _empty(stream, fact_keys.shape, dtype=torch.int32, device=fact_keys.device)
    _check(_lib.lq_keymap64_lookup(table.data_ptr(), table.numel(), fact_keys.data_ptr(),
                                   int(fact_keys.shape[0]), fk.data_ptr(), _stream(stream)))
    return fk


def lq_compact_matches(fk: torch.Tensor, stream=None):
    """COO index vectors of the row-matching matrix: (rows int64 [n], cols int32 [n], nnz int64 [1]);
    only the first nnz entries of rows / cols are meaningful."""
    _expect(fk, torch.int32, "mapped key column")
    n = int(fk.shape[0])
    rows = _empty(stream, n, dtype=torch.int64, device=fk.device)
    cols = _empty(stream, n, dtype=torch.int32, device=fk.device)
    nnz = _empty(stream, 1, dtype=torch.int64, device=fk.device)
    ws = _empty(stream, int(_lib.lq_compact_workspace_bytes(n)), dtype=torch.uint8, device=fk.device)
    _check(_lib.lq_compact_matches(fk.data_ptr(), n, rows.data_ptr(), cols.data_ptr(), nnz.data_ptr(),
                                   ws.data_ptr(), ws.numel(), _stream(stream)))
    return rows, cols, nnz


# ---------------------------------------------------------------- group discovery, result ordering

def lq_group_domain_workspace_bytes(rows: int) -> int:
    return int(_lib.lq_group_domain_workspace_bytes(int(rows)))


def lq_group_domain(cols: Sequence[torch.Tensor], max_card: int = 65535, stream=None):
    """Distinct tuples of the attribute columns of one table, numbered in ascending order.
    Returns (code int32 [rows], values int32 [card x n_cols], card)."""
    for c in cols:
        _expect(c, torch.int32, "attribute column")
        if c.shape[0] != cols[0].shape[0]:
            raise ValueError("attribute columns differ in length")
    rows = int(cols[0].shape[0])
    dev = cols[0].device
    code = _empty(stream, rows, dtype=torch.int32, device=dev)
    values = _empty(stream, (int(max_card), len(cols)), dtype=torch.int32, device=dev)
    ws = _empty(stream, lq_group_domain_workspace_bytes(rows), dtype=torch.uint8, device=dev)
    card = ctypes.c_int32(0)
    _check(_lib.lq_group_domain(rows, len(cols), _ptr_array(cols), int(max_card), code.data_ptr(),
                                values.data_ptr(), ctypes.byref(card), ws.data_ptr(), ws.numel(), _stream(stream)))
    return code, values[:card.value], int(card.value)


def lq_order_groups(group_card: Sequence[int], sums: Optional[torch.Tensor], counts: torch.Tensor,
                    keys: Sequence[Sequence[int]], order: Optional[torch.Tensor] = None,
                    n_out: Optional[torch.Tensor] = None, stream=None):
    """ORDER BY over the populated groups.  keys: (kind, index, descending) triples.
    Returns (order int32 [G] padded with -1, n_out int32 [1]), both on the device."""
    _expect(counts, torch.int64, "counts")
    G = int(counts.shape[0])
    n_measures = 0
    if sums is not None:
        _expect(sums, torch.int64, "sums")
        if sums.dim() != 2 or sums.shape[1] != G or not sums.is_contiguous():
            raise ValueError("sums must be a contiguous [n_measures x G] tensor")
        n_measures = int(sums.shape[0])
    prod = 1
    for c in group_card:
        prod *= int(c)
    if prod != G:
        raise ValueError("counts length differs from the product of group_card")
    card = (ctypes.c_int32 * max(1, len(group_card)))(*[int(c) for c in group_card])
    karr = (lq_sort_key * max(1, len(keys)))()
    for q, (kind, index, desc) in enumerate(keys):
        karr[q] = lq_sort_key(int(kind), int(index), int(bool(desc)))
    if order is None:
        order = _empty(stream, G, dtype=torch.int32, device=counts.device)
    if n_out is None:
        n_out = _empty(stream, 1, dtype=torch.int32, device=counts.device)
    _expect(order, torch.int32, "order")
    _expect(n_out, torch.int32, "n_out")
    if order.numel() < G or n_out.numel() < 1:
        raise ValueError("order needs G entries and n_out one")
    _check(_lib.lq_order_groups(len(group_card), card, n_measures, None if sums is None else sums.data_ptr(),
                                counts.data_ptr(), len(keys), karr, order.data_ptr(), n_out.data_ptr(),
                                _stream(stream)))
    return order, n_out


# ---------------------------------------------------------------- incremental pre-fusion, advice

def lq_project_dim_rows(dims: Sequence[torch.Tensor], W0: torch.Tensor, c_f: int, P: List[torch.Tensor],
                        dim: int, first_row: int, n_rows: int, stream=None) -> None:
    """Refresh rows [first_row, first_row + n_rows) of P[dim] after those dimension rows changed."""
    fact = lq_mat(None, 0, int(c_f), max(int(c_f), 1), _dtype_code(W0))
    dims_arr = _mat_array(dims)
    star = lq_star(0, fact, len(dims), dims_arr, _ptr_array([None] * len(dims)))
    model = _Model([W0], None)
    P_arr = _mat_array(P)
    _check(_lib.lq_project_dim_rows(ctypes.byref(star), ctypes.byref(model.c), P_arr, dim, first_row, n_rows,
                                    _stream(stream)))


def lq_fusion_advice(n_fact: int, c_f: int, dim_shapes: Sequence[Sequence[int]], layer_widths: Sequence[int],
                     queries_per_update: float = 1.0, dtype: int = LQ_F32) -> dict:
    """Complexity model of Section 3.2.1 for a star of the given shapes (no device memory touched)."""
    fake = 0x10000
    dims_arr = (lq_mat * max(1, len(dim_shapes)))()
    for j, (r, c) in enumerate(dim_shapes):
        dims_arr[j] = lq_mat(fake, int(r), int(c), int(c), dtype)
    fks = (ctypes.c_void_p * max(1, len(dim_shapes)))(*([fake] * len(dim_shapes)))
    star = lq_star(int(n_fact), lq_mat(fake, int(n_fact), int(c_f), max(int(c_f), 1), dtype), len(dim_shapes), dims_arr, fks)
    W = (lq_mat * len(layer_widths))()
    rows = int(c_f) + sum(int(c) for _, c in dim_shapes)
    for j, lo in enumerate(layer_widths):
        W[j] = lq_mat(fake, rows, int(lo), int(lo), dtype)
        rows = int(lo)
    bias = (ctypes.c_void_p * len(layer_widths))()
    model = lq_model(len(layer_widths), W, bias)
    out = lq_advice()
    _check(_lib.lq_fusion_advice(ctypes.byref(star), ctypes.byref(model), float(queries_per_update), ctypes.byref(out)))
    return {n: getattr(out, n) for n, _ in lq_advice._fields_}


# ---------------------------------------------------------------- wider aggregate query --------

_MEASURE_OPS = {"col": 0, "mul": 1, "sub": 2}


def lq_groupby_agg(fks: Sequence[torch.Tensor], dim_rows: Sequence[int], dim_mask, dim_code,
                   group_card: Sequence[int], preds, measures, want=("sum", "min", "max", "count"),
                   ws: Optional[torch.Tensor] = None, flags: int = 0, stream=None) -> dict:
    """Filtered star join + GROUP BY with fact range predicates ``[(column, lo, hi)]``, measures
    ``[(op, a, b)]`` (op in col / mul / sub) and SUM / MIN / MAX / COUNT.  Returns a dict of int64 tensors."""
    K = len(fks)
    n = int(measures[0][1].shape[0])
    dev = measures[0][1].device
    for f in fks:
        _expect(f, torch.int32, "foreign-key column")
    masks = list(dim_mask) if dim_mask is not None else [None] * K
    codes = list(dim_code) if dim_code is not None else [None] * K
    G = 1
    for k in range(K):
        if codes[k] is not None:
            G *= int(group_card[k])
    M = len(measures)
    pa = (lq_range_pred * max(1, len(preds)))()
    for q, (col, lo, hi) in enumerate(preds):
        _expect(col, torch.int32, "predicate column")
        pa[q] = lq_range_pred(col.data_ptr(), int(lo), int(hi))
    ma = (lq_measure * M)()
    for m, (op, a, b) in enumerate(measures):
        _expect(a, torch.int32, "measure column")
        if b is not None:
            _expect(b, torch.int32, "measure column")
        ma[m] = lq_measure(_MEASURE_OPS[op], a.data_ptr(), None if b is None else b.data_ptr())
    out = {}
    for name in ("sum", "min", "max"):
        out[name] = _empty(stream, (M, G), dtype=torch.int64, device=dev) if name in want else None
    out["count"] = _empty(stream, (G,), dtype=torch.int64, device=dev) if "count" in want else None
    rows = (ctypes.c_int64 * max(1, K))(*[int(r) for r in dim_rows])
    card = (ctypes.c_int32 * max(1, K))(*[int(c) for c in group_card])
    if ws is None:
        need = int(_lib.lq_groupby_agg_workspace_bytes(K, rows, card, M))
        if not preds and "min" not in want and "max" not in want and "sum" in want:
            eff = (ctypes.c_int32 * max(1, K))(*[int(group_card[k]) if codes[k] is not None else 1 for k in range(K)])
            need = max(need, int(_lib.lq_groupby_agg_bucket_workspace_bytes(n, K, rows, eff, M, ctypes.cast(ma, ctypes.c_void_p))))
        ws = _empty(stream, need, dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(_lib.lq_groupby_agg(n, K, _ptr_array(fks), rows, _ptr_array(masks), _ptr_array(codes), card,
                               len(preds), pa, M, ma, ptr(out["sum"]), ptr(out["min"]), ptr(out["max"]),
                               ptr(out["count"]), ws.data_ptr(), ws.numel(), flags, _stream(stream)))
    return out
