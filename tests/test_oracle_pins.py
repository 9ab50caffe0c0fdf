"""Pins for the CPU oracle: each test checks it against something that is not the oracle
(brute-force relational evaluation, dense indicator-matrix algebra, numpy library routines,
hand-worked numbers, invariants), chosen so that a dropped term, a wrong index or a
transposed operand fails at least one of them.  All CPU, all tiny."""
import os

import numpy as np
import pytest

from oracle import lq_oracle as O
from tests import bruteforce_relational as BF

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _tiny_star(seed, n=37, c_f=3, rows=(5, 8, 3), cols=(2, 4, 1), integer=False):
    r = _rng(seed)
    draw = (lambda s: r.integers(-4, 5, size=s).astype(np.float64)) if integer \
        else (lambda s: r.standard_normal(s))
    X = draw((n, c_f)) if c_f else None
    dims = [draw((a, b)) for a, b in zip(rows, cols)]
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    return X, dims, fks


def _weights(seed, widths, integer=False, positive=False):
    r = _rng(seed)
    out = []
    for a, b in zip(widths[:-1], widths[1:]):
        if integer:
            w = r.integers(-2, 3, size=(a, b)).astype(np.float64)
        else:
            w = r.standard_normal((a, b))
        out.append(np.abs(w) + 0.1 if positive else w)
    return out


# ---------------------------------------------------------------- join semantics ---------

def test_join_predict_matches_bruteforce_relational_join_on_shuffled_keys():
    """Dimensions carry explicit, shuffled, non-contiguous primary keys; the join is a nested
    loop on key equality; the model is a plain-Python MLP."""
    r = _rng(1)
    n, c_f, rows, cols = 41, 2, (6, 4), (3, 2)
    X, dims, fks = _tiny_star(2, n, c_f, rows, cols)
    pks = [r.permutation(np.arange(100, 100 + 7 * a, 7))[:a] for a in rows]   # e.g. 121, 100, 135...
    dim_tables = [[(int(pk[j]), tuple(d[j])) for j in range(d.shape[0])] for pk, d in zip(pks, dims)]
    # shuffle the stored order of each dimension table: brute force must not depend on it
    for t in dim_tables:
        r.shuffle(t)
    fact_rows = [(tuple(X[i]), [int(pks[k][fks[k][i]]) for k in range(2)]) for i in range(n)]
    W = _weights(3, [c_f + sum(cols), 5, 3])
    b = [r.standard_normal(5), r.standard_normal(3)]
    joined = BF.star_join(fact_rows, dim_tables)
    assert len(joined) == n                      # PK-FK: exactly one match per fact row
    want = np.array([BF.mlp(t, [w.tolist() for w in W], [x.tolist() for x in b]) for t in joined])
    got = O.join_predict(X, dims, fks, W, b)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    T = O.materialize(X, dims, fks)
    np.testing.assert_array_equal(T, np.array(joined))


def test_materialize_equals_indicator_matrix_algebra_and_projection_orientation():
    """T = X M_f + sum_k I_k D_k M_k with dense 0/1 matrices (Eq. 1, first line).  M is
    [source cols x target cols] and target = source * M, as the Patient example fixes."""
    X, dims, fks = _tiny_star(4, n=19, c_f=2, rows=(4, 6), cols=(3, 2), integer=True)
    n, kw = 19, 2 + 3 + 2
    T = np.zeros((n, kw))
    Mf = np.zeros((2, kw)); Mf[0, 0] = Mf[1, 1] = 1
    T += X @ Mf
    off = 2
    for d, f in zip(dims, fks):
        I = np.zeros((n, d.shape[0]))
        I[np.arange(n), f] = 1
        assert (I.sum(axis=1) == 1).all()        # one 1 per materialised row
        M = np.zeros((d.shape[1], kw))
        for s in range(d.shape[1]):
            M[s, off + s] = 1
        T += I @ d @ M
        off += d.shape[1]
    np.testing.assert_array_equal(O.materialize(X, dims, fks), T)

    # the paper's projection example: Patient(weight, height, age) -> (weight, age)
    pairs = [tuple(map(int, l.split()[1:])) for l in open(os.path.join(GOLDEN, "projection_example.txt"))
             if l.startswith("M ")]
    M = np.zeros((3, 2))
    for s, t in pairs:
        M[s, t] = 1
    patient = np.array([[70., 180., 33.], [55., 160., 41.]])
    np.testing.assert_array_equal(patient @ M, patient[:, [0, 2]])
    # the same selection expressed as a 1-dimension star: D = patient, W = M
    got = O.join_predict(None, [patient], [np.array([1, 0, 1], dtype=np.int32)], [M])
    np.testing.assert_array_equal(got, patient[[1, 0, 1]][:, [0, 2]])


def test_eq1_identity_exact_on_integer_data_and_close_on_reals():
    """(sum_k I_k D_k M_k) L == sum_k I_k (D_k M_k L)."""
    for integer in (True, False):
        X, dims, fks = _tiny_star(5, n=53, c_f=3, rows=(7, 5, 9), cols=(4, 2, 3), integer=integer)
        (W,) = _weights(6, [3 + 9, 6], integer=integer)
        b = np.arange(6, dtype=np.float64) - 2
        lhs = O.join_predict(X, dims, fks, [W], [b])
        P = O.project_dims(dims, W, c_f=3)
        rhs = O.gather_sum(X, W, P, fks, b)
        if integer:
            np.testing.assert_array_equal(lhs, rhs)
        else:
            np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_project_dims_is_numpy_matmul_on_the_dimension_slice_of_W():
    X, dims, fks = _tiny_star(7, rows=(5, 8, 3), cols=(2, 4, 1))
    (W,) = _weights(8, [3 + 7, 5])
    P = O.project_dims(dims, W, c_f=3)
    off = 3
    for d, p in zip(dims, P):
        np.testing.assert_allclose(p, d @ W[off:off + d.shape[1]], rtol=1e-13, atol=1e-13)
        off += d.shape[1]


# ------------------------------------------------------------ special cases -------------

def test_no_dimensions_reduces_to_numpy_matmul():
    r = _rng(9)
    X = r.standard_normal((23, 6))
    W = r.standard_normal((6, 4))
    np.testing.assert_allclose(O.join_predict(X, [], [], [W]), X @ W, rtol=1e-13, atol=1e-13)


def test_all_keys_equal_adds_one_constant_row():
    X, dims, _ = _tiny_star(10, n=17, c_f=2, rows=(4, 3), cols=(3, 2))
    fks = [np.full(17, 2, np.int32), np.full(17, 1, np.int32)]
    (W,) = _weights(11, [7, 3])
    const = dims[0][2] @ W[2:5] + dims[1][1] @ W[5:7]
    np.testing.assert_allclose(O.join_predict(X, dims, fks, [W]), X @ W[:2] + const,
                               rtol=1e-13, atol=1e-13)


def test_zero_weights_give_the_bias():
    X, dims, fks = _tiny_star(12)
    b = np.array([1.5, -2.0])
    got = O.join_predict(X, dims, fks, [np.zeros((3 + 7, 2))], [b])
    np.testing.assert_array_equal(got, np.tile(b, (37, 1)))


def test_one_hot_weights_make_the_output_a_pure_gather():
    """Column o of W selects tuple column sel[o]; Y must be exactly those table entries."""
    X, dims, fks = _tiny_star(13, n=29, c_f=2, rows=(6, 5), cols=(3, 4), integer=True)
    sel = [8, 0, 3, 6]                            # dim1 col 3, fact col 0, dim0 col 1, dim1 col 1
    W = np.zeros((9, 4))
    for o, s in enumerate(sel):
        W[s, o] = 1
    got = O.join_predict(X, dims, fks, [W])
    want = np.stack([dims[1][fks[1], 3], X[:, 0], dims[0][fks[0], 1], dims[1][fks[1], 1]], axis=1)
    np.testing.assert_array_equal(got, want)


def test_hand_worked_two_layer_example():
    """x = (1, -2); D_0 = [[3], [-1]]; fk = (1, 0).  W1 = [[1, 0], [0, 1], [2, -1]], b1 = (0.5, 0),
    W2 = [[1], [-3]], b2 = (10).
    row 0: t = (1, -2, -1): z = (1 - 2 + 0.5, -2 + 1) = (-0.5, -1) -> relu (0, 0) -> y = 10
    row 1: t = (1, -2, 3):  z = (1 + 6 + 0.5, -2 - 3) = (7.5, -5)  -> relu (7.5, 0) -> y = 17.5"""
    X = np.array([[1., -2.], [1., -2.]])
    D0 = np.array([[3.], [-1.]])
    fk = np.array([1, 0], dtype=np.int32)
    W1 = np.array([[1., 0.], [0., 1.], [2., -1.]])
    W2 = np.array([[1.], [-3.]])
    got = O.join_predict(X, [D0], [fk], [W1, W2], [np.array([0.5, 0.]), np.array([10.])])
    np.testing.assert_array_equal(got, np.array([[10.], [17.5]]))
    # without the ReLU the answer would be 10 + (-0.5) - 3*(-1) = 12.5 and 10 + 7.5 + 15 = 32.5
    lin = O.join_predict(X, [D0], [fk], [W1 @ W2], [np.array([0.5, 0.]) @ W2 + 10.])
    np.testing.assert_array_equal(lin, np.array([[12.5], [32.5]]))


def test_single_layer_mlp_is_the_linear_case_and_inactive_relu_collapses_layers():
    X, dims, fks = _tiny_star(14, n=31, c_f=2, rows=(5, 4), cols=(3, 2))
    W1, W2, W3 = _weights(15, [7, 6, 4, 2], positive=True)
    Xp, dp = np.abs(X), [np.abs(d) for d in dims]
    got = O.join_predict(Xp, dp, fks, [W1, W2, W3])
    T = np.concatenate([Xp] + [d[f] for d, f in zip(dp, fks)], axis=1)
    np.testing.assert_allclose(got, T @ (W1 @ W2 @ W3), rtol=1e-12, atol=1e-12)
    # with signs, ReLU matters: compare against numpy layer by layer
    W = _weights(16, [7, 6, 3])
    T = np.concatenate([X] + [d[f] for d, f in zip(dims, fks)], axis=1)
    want = np.maximum(T @ W[0], 0) @ W[1]
    np.testing.assert_allclose(O.join_predict(X, dims, fks, W), want, rtol=1e-12, atol=1e-12)
    assert np.abs(want - T @ W[0] @ W[1]).max() > 1e-3


def test_threads_do_not_change_results():
    X, dims, fks = _tiny_star(17, n=1001)
    W = _weights(18, [10, 8, 2])
    a = O.join_predict(X, dims, fks, W, nthreads=1)
    b = O.join_predict(X, dims, fks, W, nthreads=4)
    np.testing.assert_array_equal(a, b)


def test_shape_errors_are_reported():
    X, dims, fks = _tiny_star(19)
    with pytest.raises(ValueError):
        O.join_predict(X, dims, fks, [np.zeros((9, 2))])           # joined width is 10
    with pytest.raises(ValueError):
        O.join_predict(X, dims, fks, [np.zeros((10, 4)), np.zeros((3, 1))])
    bad = [f.copy() for f in fks]
    bad[1][5] = 8                                                   # dim 1 has 8 rows
    with pytest.raises(ValueError):
        O.join_predict(X, dims, bad, [np.zeros((10, 2))])


# ------------------------------------------------------------------ group-by -------------

def _tiny_groupby(seed, n=200, rows=(7, 11, 5, 13), card=(3, 4), with_neg=False):
    r = _rng(seed)
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    if with_neg:
        fks[2][r.integers(0, n, size=9)] = -1
    codes = [r.integers(0, card[0], size=rows[0]).astype(np.int32),
             r.integers(0, card[1], size=rows[1]).astype(np.int32), None, None]
    masks = [None, (r.random(rows[1]) < 0.8).astype(np.uint8),
             (r.random(rows[2]) < 0.5).astype(np.uint8), (r.random(rows[3]) < 0.6).astype(np.uint8)]
    meas = [r.integers(1, 100001, size=n).astype(np.int32), r.integers(-50, 50, size=n).astype(np.int32)]
    fact_mask = (r.random(n) < 0.9).astype(np.uint8)
    return fks, list(rows), masks, codes, [card[0], card[1], 1, 1], fact_mask, meas


def _numpy_groupby(fks, rows, masks, codes, card, fact_mask, meas):
    n = fks[0].shape[0]
    s = np.ones(n, dtype=bool) if fact_mask is None else fact_mask.astype(bool)
    g = np.zeros(n, dtype=np.int64)
    for k in range(len(fks)):
        ok = fks[k] >= 0
        j = np.where(ok, fks[k], 0)
        s &= ok
        if masks[k] is not None:
            s &= masks[k][j].astype(bool)
        if codes[k] is not None:
            g = g * card[k] + codes[k][j]
    G = int(np.prod(card))
    sums = np.zeros((len(meas), G), dtype=np.int64)
    for m, v in enumerate(meas):
        np.add.at(sums[m], g[s], v[s].astype(np.int64))
    counts = np.bincount(g[s], minlength=G).astype(np.int64)
    return sums, counts


def test_groupby_matches_numpy_scatter_add_and_bincount():
    for seed, neg in ((20, False), (21, True)):
        args = _tiny_groupby(seed, with_neg=neg)
        sums, counts = O.groupby_sum(*args)
        ws, wc = _numpy_groupby(*args)
        np.testing.assert_array_equal(sums, ws)
        np.testing.assert_array_equal(counts, wc)
        sums4, counts4 = O.groupby_sum(*args, nthreads=4)
        np.testing.assert_array_equal(sums4, ws)
        np.testing.assert_array_equal(counts4, wc)


def test_groupby_matches_bruteforce_relational_query():
    r = _rng(22)
    fks, rows, masks, codes, card, fact_mask, meas = _tiny_groupby(23, n=60, rows=(4, 5, 3, 6))
    pks = [r.permutation(np.arange(10, 10 + 3 * a, 3)) for a in rows]
    dim_tables = []
    for k in range(4):
        t = [(int(pks[k][j]), {"code": None if codes[k] is None else int(codes[k][j]),
                               "ok": True if masks[k] is None else bool(masks[k][j])})
             for j in range(rows[k])]
        r.shuffle(t)
        dim_tables.append(t)
    fact_rows = [([int(pks[k][fks[k][i]]) for k in range(4)], [int(m[i]) for m in meas],
                  bool(fact_mask[i])) for i in range(60)]
    res = BF.filter_join_group_sum(fact_rows, dim_tables, ["code", "code", None, None],
                                   [lambda a: a["ok"]] * 4, 2)
    sums, counts = O.groupby_sum(fks, rows, masks, codes, card, fact_mask, meas)
    for a in range(card[0]):
        for b in range(card[1]):
            g = a * card[1] + b                   # last grouping dimension fastest
            if (a, b) in res:
                assert [int(sums[0, g]), int(sums[1, g])] == res[(a, b)][0]
                assert int(counts[g]) == res[(a, b)][1]
            else:
                assert counts[g] == 0 and sums[0, g] == 0 and sums[1, g] == 0
    assert sum(c for _, c in res.values()) == counts.sum()


def test_groupby_bigroup_closed_form_with_dense_indicator_matrices():
    """R = (I_a E_a)^T diag(s * v) (I_b E_b): selection vector, row-mapping matrices and
    group-mapping matrices all built densely."""
    fks, rows, masks, codes, card, fact_mask, meas = _tiny_groupby(24, n=32)
    n = 32
    s = fact_mask.astype(np.int64)
    for k in range(4):
        if masks[k] is not None:
            I = np.zeros((n, rows[k]), dtype=np.int64)
            I[np.arange(n), fks[k]] = 1
            s = s * (I @ masks[k].astype(np.int64))        # mask pushed through I_k
    IE = []
    for k in (0, 1):
        I = np.zeros((n, rows[k]), dtype=np.int64)
        I[np.arange(n), fks[k]] = 1
        E = np.zeros((rows[k], card[k]), dtype=np.int64)
        E[np.arange(rows[k]), codes[k]] = 1
        IE.append(I @ E)
    sums, counts = O.groupby_sum(fks, rows, masks, codes, card, fact_mask, meas)
    for m in range(2):
        R = IE[0].T @ np.diag(s * meas[m].astype(np.int64)) @ IE[1]
        np.testing.assert_array_equal(sums[m].reshape(card[0], card[1]), R)
    np.testing.assert_array_equal(counts.reshape(card[0], card[1]), IE[0].T @ np.diag(s) @ IE[1])


def test_groupby_invariants():
    fks, rows, masks, codes, card, fact_mask, meas = _tiny_groupby(25, n=500)
    sums, counts = O.groupby_sum(fks, rows, masks, codes, card, fact_mask, meas)
    s = fact_mask.astype(bool)
    for k in range(4):
        if masks[k] is not None:
            s &= masks[k][fks[k]].astype(bool)
    assert counts.sum() == s.sum()
    assert sums[0].sum() == meas[0][s].astype(np.int64).sum()
    # no masks, no grouping: a plain column sum in one group
    s1, c1 = O.groupby_sum(fks, rows, None, None, [1] * 4, None, meas)
    assert s1.shape == (2, 1) and c1[0] == 500
    assert s1[0, 0] == meas[0].astype(np.int64).sum() and s1[1, 0] == meas[1].astype(np.int64).sum()
    # a partition of one dimension's rows into two masks: results add up to the unmasked result
    part = (np.arange(rows[3]) % 2).astype(np.uint8)
    base = list(masks); base[3] = None
    a = list(base); a[3] = part
    b = list(base); b[3] = 1 - part
    sa, ca = O.groupby_sum(fks, rows, a, codes, card, fact_mask, meas)
    sb, cb = O.groupby_sum(fks, rows, b, codes, card, fact_mask, meas)
    s0, c0 = O.groupby_sum(fks, rows, base, codes, card, fact_mask, meas)
    np.testing.assert_array_equal(sa + sb, s0)
    np.testing.assert_array_equal(ca + cb, c0)
    # a bad code is rejected, not silently folded into another group
    bad = [c if c is None else c.copy() for c in codes]
    bad[1][0] = card[1]
    if (fks[1] == 0).any():
        with pytest.raises(ValueError):
            O.groupby_sum(fks, rows, None, bad, card, None, meas)


def test_groupby_paper_text_example():
    """Key domain {0,1,2,3,4,7}; groups {2}->0, {3,0}->1, {4,7}->2 (Section 2.4.1)."""
    S, R, want = [], [], {}
    for line in open(os.path.join(GOLDEN, "groupby_single_column_example.txt")):
        p = line.split()
        if not p or p[0] == "#":
            continue
        if p[0] == "S":
            S.append((int(p[1]), int(p[2])))
        elif p[0] == "R":
            R.append((int(p[1]), int(p[2])))
        elif p[0] == "G":
            want[int(p[1])] = (int(p[2]), int(p[3]))
    domain = sorted(set(k for k, _ in S) | set(k for k, _ in R))
    assert domain == [0, 1, 2, 3, 4, 7]
    row_of_key = {k: j for j, (k, _) in enumerate(S)}
    fk = np.array([row_of_key.get(k, -1) for k, _ in R], dtype=np.int32)   # no match -> dropped
    code = np.array([g for _, g in S], dtype=np.int32)
    val = np.array([v for _, v in R], dtype=np.int32)
    sums, counts = O.groupby_sum([fk], [len(S)], None, [code], [3], None, [val])
    for g, (s, c) in want.items():
        assert sums[0, g] == s and counts[g] == c
    # the LA form of the same example: MAT_R (values) * MAT_S^T, then the ones reduction
    MAT_R = np.zeros((len(R), len(domain)), dtype=np.int64)
    MAT_S = np.zeros((3, len(domain)), dtype=np.int64)
    for i, (k, v) in enumerate(R):
        MAT_R[i, domain.index(k)] = v
    for k, g in S:
        MAT_S[g, domain.index(k)] = 1
    np.testing.assert_array_equal(np.ones(len(R), dtype=np.int64) @ (MAT_R @ MAT_S.T), sums[0])
