"""ctypes front end of the CPU oracle (``lq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU package never imports this module and
this module never imports the GPU package.

Every floating-point input (numpy fp32/fp64 array or torch CPU tensor in fp32
or bf16) is widened exactly to fp64 before the C code sees it; integer inputs
are passed as int32 / uint8.  Results come back as fp64 / int64 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lq_oracle.c")
_LIB = os.path.join(_HERE, "liblq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``lq_oracle.c`` with gcc into ``liblq_oracle.so`` beside it."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.lqo_max_threads.restype = ctypes.c_int
        for name in ("lqo_join_predict", "lqo_materialize", "lqo_project_dims",
                     "lqo_gather_sum", "lqo_groupby_sum", "lqo_tree_predict", "lqo_tree_project", "lqo_groupby_agg"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().lqo_max_threads())


def _f64(a) -> np.ndarray:
    """Exact widening to a C-contiguous fp64 array."""
    if a is None:
        return None
    if hasattr(a, "detach"):  # torch tensor (fp32 / bf16 / fp64), CPU
        a = a.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a) -> np.ndarray:
    if hasattr(a, "detach"):
        a = a.detach().cpu().numpy()
    a = np.asarray(a)
    if a.dtype != np.int32:
        if a.size and (a.min() < -2**31 or a.max() >= 2**31):
            raise ValueError("value does not fit int32")
        a = a.astype(np.int32)
    return np.ascontiguousarray(a)


def _u8(a) -> np.ndarray:
    if hasattr(a, "detach"):
        a = a.detach().cpu().numpy()
    return np.ascontiguousarray(np.asarray(a).astype(np.uint8))


def _pd(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    out = (ctypes.c_void_p * max(1, len(arrs)))()
    for j, a in enumerate(arrs):
        out[j] = None if a is None else a.ctypes.data
    return out


def _i32_array(vals: Sequence[int]):
    return (ctypes.c_int32 * max(1, len(vals)))(*[int(v) for v in vals])


def _prep_star(X, dims, fks):
    dims = [_f64(d) for d in dims]
    fks = [_i32(f) for f in fks]
    if len(dims) != len(fks):
        raise ValueError("one foreign-key column per dimension table")
    n = None
    if X is not None:
        X = _f64(X)
        if X.ndim != 2:
            raise ValueError("X must be 2-D")
        n = X.shape[0]
    for d, f in zip(dims, fks):
        if d.ndim != 2 or f.ndim != 1:
            raise ValueError("dimension tables are 2-D, key columns 1-D")
        if n is None:
            n = f.shape[0]
        if f.shape[0] != n:
            raise ValueError("key column length differs from fact rows")
        if f.size and (f.min() < 0 or f.max() >= d.shape[0]):
            raise ValueError("foreign key outside its dimension table")
    if n is None:
        raise ValueError("need fact columns or at least one dimension")
    c_f = 0 if X is None else X.shape[1]
    if X is not None and c_f == 0:
        X = None
    return n, c_f, X, dims, fks


def join_predict(X, dims, fks, weights, biases=None, nthreads: int = 1) -> np.ndarray:
    """Materialise each joined tuple, apply the (ReLU-)MLP; returns [n x l_out] fp64."""
    lib = _load()
    n, c_f, X, dims, fks = _prep_star(X, dims, fks)
    W = [_f64(w) for w in weights]
    for w in W:
        if w.ndim != 2:
            raise ValueError("weights are 2-D [in x out]")
    if biases is None:
        biases = [None] * len(W)
    B = [None if b is None else _f64(b).reshape(-1) for b in biases]
    for w, b in zip(W, B):
        if b is not None and b.shape[0] != w.shape[1]:
            raise ValueError("bias length differs from layer width")
    Y = np.empty((n, W[-1].shape[1]), dtype=np.float64)
    rc = lib.lqo_join_predict(
        ctypes.c_int64(n), ctypes.c_int32(c_f), _pd(X), ctypes.c_int32(len(dims)),
        _i32_array([d.shape[1] for d in dims]), _ptr_array(dims), _ptr_array(fks),
        ctypes.c_int32(len(W)), _i32_array([w.shape[0] for w in W]),
        _i32_array([w.shape[1] for w in W]), _ptr_array(W), _ptr_array(B),
        _pd(Y), ctypes.c_int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected the shapes (layer widths must chain and "
                         "match the joined width)")
    return Y


def materialize(X, dims, fks) -> np.ndarray:
    """The joined table T = [X | D_0[fk_0] | ...], fp64."""
    lib = _load()
    n, c_f, X, dims, fks = _prep_star(X, dims, fks)
    kw = c_f + sum(d.shape[1] for d in dims)
    T = np.empty((n, kw), dtype=np.float64)
    lib.lqo_materialize(ctypes.c_int64(n), ctypes.c_int32(c_f), _pd(X),
                        ctypes.c_int32(len(dims)),
                        _i32_array([d.shape[1] for d in dims]), _ptr_array(dims),
                        _ptr_array(fks), _pd(T))
    return T


def project_dims(dims, W, c_f: int) -> list:
    """P_k = D_k times its rows of the first-layer weights W; list of fp64 [r_k x l]."""
    lib = _load()
    W = _f64(W)
    out = []
    off = int(c_f)
    for d in dims:
        d = _f64(d)
        if off + d.shape[1] > W.shape[0]:
            raise ValueError("first-layer weights have too few rows")
        P = np.empty((d.shape[0], W.shape[1]), dtype=np.float64)
        lib.lqo_project_dims(ctypes.c_int64(d.shape[0]), ctypes.c_int32(d.shape[1]),
                             _pd(d), ctypes.c_int32(off), ctypes.c_int32(W.shape[1]),
                             _pd(W), _pd(P))
        out.append(P)
        off += d.shape[1]
    return out


def gather_sum(X, W, P, fks, bias=None) -> np.ndarray:
    """Z = X W[0:c_f] + sum_k P_k[fk_k] (+ bias): the fused side of Eq. 1, fp64."""
    lib = _load()
    W = _f64(W)
    P = [_f64(p) for p in P]
    fks = [_i32(f) for f in fks]
    X = None if X is None else _f64(X)
    c_f = 0 if X is None else X.shape[1]
    n = X.shape[0] if X is not None else fks[0].shape[0]
    if c_f == 0:
        X = None
    for p, f in zip(P, fks):
        if f.size and (f.min() < 0 or f.max() >= p.shape[0]):
            raise ValueError("foreign key outside its projected table")
    b = None if bias is None else _f64(bias).reshape(-1)
    Z = np.empty((n, W.shape[1]), dtype=np.float64)
    lib.lqo_gather_sum(ctypes.c_int64(n), ctypes.c_int32(c_f), _pd(X),
                       ctypes.c_int32(W.shape[1]), _pd(W), ctypes.c_int32(len(P)),
                       _ptr_array(P), _ptr_array(fks), _pd(b), _pd(Z))
    return Z


def groupby_sum(fks, dim_rows, dim_mask, dim_code, group_card, fact_mask, measures,
                nthreads: int = 1):
    """Filter + star join + GROUP BY + SUM/COUNT.  Returns (sums [M x G], counts [G]) int64."""
    lib = _load()
    fks = [_i32(f) for f in fks]
    K = len(fks)
    n = fks[0].shape[0] if K else (_i32(measures[0]).shape[0])
    masks = [None if m is None else _u8(m) for m in (dim_mask or [None] * K)]
    codes = [None if c is None else _i32(c) for c in (dim_code or [None] * K)]
    card = [1 if codes[k] is None else int(group_card[k]) for k in range(K)]
    for k in range(K):
        r = int(dim_rows[k])
        if fks[k].size and fks[k].max() >= r:
            raise ValueError("foreign key outside its dimension table")
        if masks[k] is not None and masks[k].shape[0] != r:
            raise ValueError("mask length differs from dimension rows")
        if codes[k] is not None and codes[k].shape[0] != r:
            raise ValueError("code length differs from dimension rows")
    fm = None if fact_mask is None else _u8(fact_mask)
    meas = [_i32(m) for m in measures]
    G = 1
    for k in range(K):
        G *= card[k]
    sums = np.empty((len(meas), G), dtype=np.int64)
    counts = np.empty((G,), dtype=np.int64)
    rc = lib.lqo_groupby_sum(ctypes.c_int64(n), ctypes.c_int32(K), _ptr_array(fks),
                             _ptr_array(masks), _ptr_array(codes), _i32_array(card),
                             _pd(fm), ctypes.c_int32(len(meas)), _ptr_array(meas),
                             _pd(sums), _pd(counts), ctypes.c_int(nthreads))
    if rc == -2:
        raise ValueError("group code outside [0, cardinality)")
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return sums, counts


def _tree_arrays(feature, threshold, H):
    feature = _i32(feature).reshape(-1)
    v = _f64(threshold).reshape(-1)
    if hasattr(H, "detach"):
        H = H.detach().cpu().numpy()
    H = np.ascontiguousarray(np.asarray(H).astype(np.int8))
    if H.ndim != 2 or H.shape[0] != feature.shape[0] or v.shape[0] != feature.shape[0]:
        raise ValueError("feature, threshold and H disagree on the number of nodes")
    if H.size and (H.min() < -1 or H.max() > 1):
        raise ValueError("H entries must be -1, 0 or 1")
    return feature, v, H


def tree_predict(X, dims, fks, feature, threshold, H):
    """((T F > v) H) == h on the materialised join.  Returns (R int32 [n x l], onehot uint8 [n x l],
    leaf int32 [n])."""
    lib = _load()
    n, c_f, X, dims, fks = _prep_star(X, dims, fks)
    feature, v, H = _tree_arrays(feature, threshold, H)
    p, l = H.shape
    R = np.empty((n, l), dtype=np.int32)
    onehot = np.empty((n, l), dtype=np.uint8)
    leaf = np.empty((n,), dtype=np.int32)
    rc = lib.lqo_tree_predict(ctypes.c_int64(n), ctypes.c_int32(c_f), _pd(X), ctypes.c_int32(len(dims)),
                              _i32_array([d.shape[1] for d in dims]), _ptr_array(dims), _ptr_array(fks),
                              ctypes.c_int32(p), ctypes.c_int32(l), _pd(feature), _pd(v), _pd(H),
                              _pd(R), _pd(onehot), _pd(leaf))
    if rc != 0:
        raise ValueError("a node tests a column outside the joined table")
    return R, onehot, leaf


def tree_project(dims, c_f, feature, threshold, H) -> list:
    """Pre-fused tables of Eq. 2, one int32 [r_k x l] per dimension (each node is evaluated only
    in the table that owns its column)."""
    lib = _load()
    feature, v, H = _tree_arrays(feature, threshold, H)
    p, l = H.shape
    out, off = [], int(c_f)
    for d in dims:
        d = _f64(d)
        Tk = np.empty((d.shape[0], l), dtype=np.int32)
        lib.lqo_tree_project(ctypes.c_int64(d.shape[0]), ctypes.c_int32(d.shape[1]), _pd(d),
                             ctypes.c_int32(off), ctypes.c_int32(p), ctypes.c_int32(l), _pd(feature),
                             _pd(v), _pd(H), _pd(Tk))
        out.append(Tk)
        off += d.shape[1]
    return out


def groupby_agg(fks, dim_rows, dim_mask, dim_code, group_card, preds, measures):
    """Filter (dimension masks + fact range predicates) + star join + GROUP BY + SUM/MIN/MAX/COUNT.

    preds:    list of (column, lo, hi): keep rows with lo <= column <= hi
    measures: list of (op, a, b) with op in {"col", "mul", "sub"} (b is None for "col")
    Returns (sums, mins, maxs [M x G] int64, counts [G] int64)."""
    lib = _load()
    fks = [_i32(f) for f in fks]
    K = len(fks)
    masks = [None if m is None else _u8(m) for m in (dim_mask or [None] * K)]
    codes = [None if c is None else _i32(c) for c in (dim_code or [None] * K)]
    card = [1 if codes[k] is None else int(group_card[k]) for k in range(K)]
    for k in range(K):
        if fks[k].size and fks[k].max() >= int(dim_rows[k]):
            raise ValueError("foreign key outside its dimension table")
    pc = [_i32(p[0]) for p in preds]
    ops = {"col": 0, "mul": 1, "sub": 2}
    A = [_i32(m[1]) for m in measures]
    B = [A[j] if m[2] is None else _i32(m[2]) for j, m in enumerate(measures)]
    n = A[0].shape[0]
    G = 1
    for c in card:
        G *= c
    M = len(measures)
    sums, mins, maxs = (np.empty((M, G), dtype=np.int64) for _ in range(3))
    counts = np.empty((G,), dtype=np.int64)
    rc = lib.lqo_groupby_agg(ctypes.c_int64(n), ctypes.c_int32(K), _ptr_array(fks), _ptr_array(masks),
                             _ptr_array(codes), _i32_array(card), ctypes.c_int32(len(pc)), _ptr_array(pc),
                             _i32_array([p[1] for p in preds]), _i32_array([p[2] for p in preds]),
                             ctypes.c_int32(M), _i32_array([ops[m[0]] for m in measures]), _ptr_array(A),
                             _ptr_array(B), _pd(sums), _pd(mins), _pd(maxs), _pd(counts))
    if rc != 0:
        raise ValueError("group code outside [0, cardinality)")
    return sums, mins, maxs, counts


def group_avg(sums, counts) -> np.ndarray:
    """AVG per group = SUM / COUNT in fp64 ([M x G] from sums [M x G] and counts [G]); NaN where a group has no rows."""
    lib = _load()
    sums = np.ascontiguousarray(np.asarray(sums, dtype=np.int64))
    counts = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    M, G = sums.shape
    avgs = np.empty((M, G), dtype=np.float64)
    lib.lqo_group_avg(ctypes.c_int64(M), ctypes.c_int64(G), _pd(sums), _pd(counts), _pd(avgs))
    return avgs
