"""Pins for the decision-tree part of the oracle (Section 3.3): plain tree traversal, a hand-worked
fixture, the dense matrix form, the identity of Eq. 2 and the reading that each dimension only
evaluates the nodes whose column it owns.  CPU only."""
import os

import numpy as np
import torch

from oracle import lq_oracle as O
from workloads import star as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _star(seed, n=200, c_f=0, rows=(7, 5, 9), cols=(3, 2, 4)):
    r = np.random.default_rng(seed)
    X = r.standard_normal((n, c_f)) if c_f else None
    dims = [r.standard_normal((a, b)) for a, b in zip(rows, cols)]
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    return X, dims, fks


def _traverse(tree, t):
    """Walk the linked tree: at node q go to the True child when t[feature] > threshold."""
    q = 0
    while q >= 0:
        go_true = t[int(tree.feature[q])] > float(tree.threshold[q])
        q = tree.true_child[q] if go_true else tree.false_child[q]
    return -q - 1


def test_matrix_form_reaches_the_leaf_a_plain_traversal_reaches():
    for seed, leaves, c_f in ((1, 2, 0), (2, 5, 0), (3, 16, 2), (4, 33, 0), (5, 7, 3)):
        X, dims, fks = _star(10 + seed, c_f=c_f)
        kw = c_f + 9
        tree = WL.make_tree(kw, leaves, seed)
        R, onehot, leaf = O.tree_predict(X, dims, fks, tree.feature, tree.threshold, tree.H)
        T = O.materialize(X, dims, fks)
        want = np.array([_traverse(tree, T[i]) for i in range(T.shape[0])])
        np.testing.assert_array_equal(leaf, want)
        assert (onehot.sum(axis=1) == 1).all()                 # exactly one leaf per tuple
        assert (onehot[np.arange(len(leaf)), leaf] == 1).all()
        # thresholds of both signs occur, so the ">" direction and the -1 entries are exercised
        assert (tree.threshold.numpy() < 0).any() and (tree.threshold.numpy() > 0).any() or leaves == 2


def test_hand_worked_three_leaf_tree():
    nodes, H, h, tuples = {}, {}, {}, []
    for line in open(os.path.join(GOLDEN, "tree_three_leaves_example.txt")):
        p = line.split()
        if not p or p[0] == "#":
            continue
        if p[0] == "N":
            nodes[int(p[1])] = (int(p[2]), float(p[3]))
        elif p[0] == "H":
            H[(int(p[1]), int(p[2]))] = int(p[3])
        elif p[0] == "h":
            h[int(p[1])] = int(p[2])
        elif p[0] == "T":
            tuples.append((float(p[1]), float(p[2]), int(p[3])))
    feature = np.array([nodes[q][0] for q in range(2)], dtype=np.int32)
    thr = np.array([nodes[q][1] for q in range(2)])
    Hm = np.zeros((2, 3), dtype=np.int8)
    for (q, j), e in H.items():
        Hm[q, j] = e
    assert (Hm[:, 1] == -1).all()                              # the paper's L2: both nodes on the False side
    # h as the fixture states it equals the number of +1 entries per column, not the column sum
    assert [h[j] for j in range(3)] == [int((Hm[:, j] == 1).sum()) for j in range(3)]
    assert [h[j] for j in range(3)] != [int(Hm[:, j].sum()) for j in range(3)]
    D = np.array([[a, b] for a, b, _ in tuples])
    fk = np.arange(len(tuples), dtype=np.int32)
    R, onehot, leaf = O.tree_predict(None, [D], [fk], feature, thr, Hm)
    assert leaf.tolist() == [w for _, _, w in tuples]
    np.testing.assert_array_equal(onehot, np.eye(3, dtype=np.uint8)[leaf])


def test_dense_matrix_form_with_numpy():
    """((T F > v) H) == h with F as a dense 0/1 column-selection matrix."""
    X, dims, fks = _star(20, c_f=2)
    tree = WL.make_tree(11, 9, 21)
    T = O.materialize(X, dims, fks)
    p = tree.n_nodes
    F = np.zeros((11, p))
    F[tree.feature.numpy(), np.arange(p)] = 1
    assert (F.sum(axis=0) == 1).all()
    Hm = tree.H.numpy().astype(np.int64)
    B = (T @ F > tree.threshold.numpy().astype(np.float64)).astype(np.int64)
    Rw = B @ Hm
    hw = (Hm == 1).sum(axis=0)
    R, onehot, leaf = O.tree_predict(X, dims, fks, tree.feature, tree.threshold, tree.H)
    np.testing.assert_array_equal(R, Rw)
    np.testing.assert_array_equal(onehot, (Rw == hw).astype(np.uint8))


def test_eq2_partial_tables_add_up_to_the_unfused_result():
    """sum_k I_k T_k (+ the fact table's own nodes) == (T F > v) H, exactly (integers)."""
    for c_f in (0, 3):
        X, dims, fks = _star(30 + c_f, n=300, c_f=c_f)
        kw = c_f + 9
        tree = WL.make_tree(kw, 12, 31)
        R, _, _ = O.tree_predict(X, dims, fks, tree.feature, tree.threshold, tree.H)
        Tk = O.tree_project(dims, c_f, tree.feature, tree.threshold, tree.H)
        S = sum(t[f] for t, f in zip(Tk, fks))
        if c_f:
            own = tree.feature.numpy() < c_f
            Bf = (X[:, tree.feature.numpy()[own]] > tree.threshold.numpy()[own].astype(np.float64))
            S = S + Bf.astype(np.int64) @ tree.H.numpy()[own].astype(np.int64)
        np.testing.assert_array_equal(S, R)


def test_leaf_is_reached_exactly_when_every_owner_agrees_on_all_of_its_path_nodes():
    """The statement behind the one-bit-per-leaf form of the pre-fused tables.  Agreement count of an
    owner (a dimension, or the fact table's own columns) for leaf j = its signed partial sum + its number
    of -1 entries in column j; it never exceeds the number of path nodes that owner has, and the counts
    of all owners reach the path length (R_j == h_j) iff each one reaches its own maximum.  Checked on
    the oracle's partial tables and its unfused result, for stars with and without fact columns, and for
    a matrix H that is not a tree (a leaf nobody reaches)."""
    for c_f, leaves, seed in ((0, 12, 40), (3, 12, 41), (2, 70, 42), (0, 3, 43)):
        X, dims, fks = _star(seed, n=400, c_f=c_f)
        tree = WL.make_tree(c_f + 9, leaves, seed + 100)
        H = tree.H.numpy().astype(np.int64)
        if seed == 43:
            H = np.concatenate([H, np.ones((H.shape[0], 1), dtype=np.int64)], axis=1)   # needs every node true
        Ht = torch.from_numpy(H.astype(np.int8))
        R, onehot, _ = O.tree_predict(X, dims, fks, tree.feature, tree.threshold, Ht)
        Tk = O.tree_project(dims, c_f, tree.feature, tree.threshold, Ht)
        feat, thr = tree.feature.numpy(), tree.threshold.numpy().astype(np.float64)
        every_owner_agrees = np.ones_like(onehot, dtype=bool)
        off = c_f
        for k, d in enumerate(dims):
            own = (feat >= off) & (feat < off + d.shape[1])
            neg, path = (H[own] == -1).sum(axis=0), (H[own] != 0).sum(axis=0)
            agree = Tk[k] + neg
            assert (agree >= 0).all() and (agree <= path).all()
            every_owner_agrees &= (agree == path)[fks[k]]
            off += d.shape[1]
        if c_f:
            # the fact table's own nodes, one at a time: the leaves that stay possible are those whose
            # path does not want the opposite outcome
            for q in np.flatnonzero(feat < c_f):
                bit = X[:, feat[q]] > thr[q]
                every_owner_agrees &= np.where(bit[:, None], H[q] >= 0, H[q] <= 0)
        np.testing.assert_array_equal(every_owner_agrees, onehot.astype(bool))
        if seed == 43:
            assert onehot[:, -1].sum() < len(onehot)         # the extra column is not always reached


def test_literal_per_dimension_predicate_double_counts_with_negative_thresholds():
    """Eq. 2 read literally evaluates (D_k M_k F > v) over ALL nodes in every dimension; a node of
    another table then sees 0 > v, which is true for v < 0.  The partial tables only add up when
    each dimension evaluates the nodes whose column it owns (what tree_project does)."""
    X, dims, fks = _star(40, n=150)
    offs = [0, 3, 5]
    for thresholds_negative in (True, False):
        tree = WL.make_tree(9, 8, 41)
        thr = tree.threshold.numpy().astype(np.float64)
        thr = -np.abs(thr) - 0.1 if thresholds_negative else np.abs(thr)
        R, _, _ = O.tree_predict(None, dims, fks, tree.feature, thr, tree.H)
        p = tree.n_nodes
        F = np.zeros((9, p)); F[tree.feature.numpy(), np.arange(p)] = 1
        Hm = tree.H.numpy().astype(np.int64)
        literal = 0
        for d, f, off in zip(dims, fks, offs):
            M = np.zeros((d.shape[1], 9)); M[np.arange(d.shape[1]), off + np.arange(d.shape[1])] = 1
            literal = literal + ((d @ M @ F > thr).astype(np.int64) @ Hm)[f]
        owned = sum(t[f] for t, f in zip(O.tree_project(dims, 0, tree.feature, thr, tree.H), fks))
        np.testing.assert_array_equal(owned, R)
        if thresholds_negative:
            assert (literal != R).any()
        else:
            np.testing.assert_array_equal(literal, R)


def test_path_matrices_that_are_no_trees_by_brute_force():
    """Eq. 2 for any H: column j of the result is 1 exactly when every node with a +1 in the column tests true and
    every node with a -1 tests false on the joined tuple, whatever the other columns say.  Several columns, or none,
    may then hold a 1; `leaf` is the first of them, -1 for none.  Checked tuple by tuple with plain Python loops on
    path matrices in which each column wants a few random nodes."""
    for seed, p, l, per, c_f in ((21, 6, 9, 2, 0), (22, 9, 20, 3, 2), (23, 4, 5, 1, 1), (24, 12, 30, 4, 0)):
        X, dims, fks = _star(40 + seed, n=150, c_f=c_f)
        kw = c_f + 9
        r = np.random.default_rng(seed)
        feature = r.integers(0, kw, size=p).astype(np.int32)
        thr = r.normal(0.0, 0.7, size=p)
        Hm = np.zeros((p, l), dtype=np.int8)
        for j in range(l):
            Hm[r.choice(p, size=per, replace=False), j] = r.choice([-1, 1], size=per)
        R, onehot, leaf = O.tree_predict(X, dims, fks, feature, thr, Hm)
        T = O.materialize(X, dims, fks)
        several = none = 0
        for i in range(T.shape[0]):
            hits = []
            for j in range(l):
                ok = True
                for q in range(p):
                    if Hm[q, j] == 0:
                        continue
                    test = T[i][int(feature[q])] > thr[q]
                    if test != (Hm[q, j] > 0):
                        ok = False
                if ok:
                    hits.append(j)
            assert onehot[i].tolist() == [1 if j in hits else 0 for j in range(l)]
            assert leaf[i] == (hits[0] if hits else -1)
            several += len(hits) > 1
            none += len(hits) == 0
        assert several > 0 and (none > 0 or per < 3)
