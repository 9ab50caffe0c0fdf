"""Pins for the group-discovery and result-ordering oracle: the paper's worked example, brute force
with Python sets and sorts, numpy's own unique / lexsort, and the invariants of the encoding.  CPU."""
import itertools
import os

import numpy as np

from oracle import domain_oracle as D
from oracle import lq_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "groupby_single_column_example.txt")


def _fixture():
    S, R, G = [], [], []
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0] == "#":
            continue
        {"S": S, "R": R, "G": G}[t[0]].append(tuple(int(x) for x in t[1:]))
    return S, R, G


def test_paper_example_groups_are_the_sorted_distinct_values():
    # Section 2.4.1: the values 0, 1, 2 are found as groups; keys {2}->0, {3,0}->1, {4,7}->2
    S, R, G = _fixture()
    attr = np.array([g for _, g in S])
    values, code = D.group_domain([attr])
    assert values.reshape(-1).tolist() == [0, 1, 2]
    by_key = {k: int(c) for (k, _), c in zip(S, code)}
    assert by_key == {2: 0, 3: 1, 0: 1, 4: 2, 7: 2}
    # the discovered codes drive the group-by oracle to the fixture's hand-added sums
    key_to_row = {k: i for i, (k, _) in enumerate(S)}
    fk = np.array([key_to_row.get(k, -1) for k, _ in R], dtype=np.int32)
    sums, counts = O.groupby_sum([fk], [len(S)], [None], [code.astype(np.int32)], [len(values)], None,
                                 [np.array([v for _, v in R], dtype=np.int32)])
    assert [(g, int(sums[0, g]), int(counts[g])) for g in range(3)] == G


def test_brute_force_sets_and_sorts():
    r = np.random.default_rng(5)
    for n_cols, rows, span in itertools.product((1, 2, 3, 4), (1, 2, 17, 300), (2, 9)):
        cols = [r.integers(-span, span, size=rows) for _ in range(n_cols)]
        values, code = D.group_domain(cols)
        tuples = list(zip(*[c.tolist() for c in cols]))
        want = sorted(set(tuples))
        assert [tuple(v) for v in values.tolist()] == want
        assert code.tolist() == [want.index(t) for t in tuples]


def test_agrees_with_numpy_unique():
    r = np.random.default_rng(6)
    a = r.integers(-1000, 1000, size=5000)
    values, code = D.group_domain([a])
    u, inv = np.unique(a, return_inverse=True)
    np.testing.assert_array_equal(values.reshape(-1), u)
    np.testing.assert_array_equal(code, inv)
    cols = [r.integers(0, 5, size=4000), r.integers(-3, 3, size=4000), r.integers(0, 2, size=4000)]
    values, code = D.group_domain(cols)
    u, inv = np.unique(np.stack(cols, axis=1), axis=0, return_inverse=True)
    np.testing.assert_array_equal(values, u)
    np.testing.assert_array_equal(code, inv.reshape(-1))


def test_invariants_and_edge_cases():
    r = np.random.default_rng(7)
    cols = [r.integers(-2**31, 2**31 - 1, size=999), r.integers(0, 3, size=999)]
    cols[0][::2] = cols[0][0]                                   # many duplicates in the leading column
    values, code = D.group_domain(cols)
    np.testing.assert_array_equal(values[code], np.stack(cols, axis=1))     # decoding restores every row
    assert code.min() == 0 and code.max() == len(values) - 1
    assert len(np.unique(code)) == len(values)                               # every group is used
    for a, b in zip(values[:-1].tolist(), values[1:].tolist()):
        assert a < b                                                         # strictly ascending tuples
    # order of the columns matters: the first one is the most significant
    v2, _ = D.group_domain(cols[::-1])
    assert v2[:, ::-1].tolist() != values.tolist()
    assert sorted(map(tuple, v2[:, ::-1].tolist())) == [tuple(v) for v in values.tolist()]
    # extremes of int32 order correctly; empty and constant columns
    values, code = D.group_domain([np.array([2**31 - 1, -2**31, 0, -1])])
    assert values.reshape(-1).tolist() == [-2**31, -1, 0, 2**31 - 1] and code.tolist() == [3, 0, 2, 1]
    values, code = D.group_domain([np.zeros(0, dtype=np.int32)])
    assert values.shape == (0, 1) and code.shape == (0,)
    values, code = D.group_domain([np.full(10, 7)])
    assert values.tolist() == [[7]] and code.tolist() == [0] * 10


def _lexsort_order(group_card, sums, counts, keys):
    G = len(counts)
    g = np.arange(G)
    cols = [g]                                                   # least significant: the group index
    for kind, index, desc in reversed(keys):
        if kind == D.KEY_GROUP_COLUMN:
            stride = int(np.prod(group_card[index + 1:]))
            v = (g // stride) % group_card[index]
        elif kind == D.KEY_SUM:
            v = sums[index]
        else:
            v = counts
        cols.append(-v if desc else v)
    order = np.lexsort(tuple(cols))
    return order[counts[order] > 0]


def test_order_groups_matches_numpy_lexsort():
    r = np.random.default_rng(8)
    card = [3, 4, 5]
    G = 60
    for trial in range(30):
        counts = r.integers(0, 4, size=G)
        sums = r.integers(-50, 50, size=(2, G)) * (counts > 0)
        n_keys = int(r.integers(0, 4))
        keys = [(int(r.integers(0, 3)), 0, bool(r.integers(0, 2))) for _ in range(n_keys)]
        keys = [(k, int(r.integers(0, 3 if k == 0 else 2)) if k != 2 else 0, d) for k, _, d in keys]
        got = D.order_groups(card, sums, counts, keys)
        np.testing.assert_array_equal(got, _lexsort_order(card, sums, counts, keys))


def test_order_groups_hand_worked():
    # 2 x 3 groups, group g = 3 a + b; counts mark g = 4 as empty
    counts = np.array([1, 2, 1, 5, 0, 1])
    sums = np.array([[10, 30, 30, -5, 0, 30]])
    assert D.order_groups([2, 3], sums, counts, []).tolist() == [0, 1, 2, 3, 5]
    assert D.order_groups([2, 3], sums, counts, [(D.KEY_SUM, 0, True)]).tolist() == [1, 2, 5, 0, 3]
    assert D.order_groups([2, 3], sums, counts, [(D.KEY_SUM, 0, False)]).tolist() == [3, 0, 1, 2, 5]
    assert D.order_groups([2, 3], sums, counts,
                          [(D.KEY_GROUP_COLUMN, 1, True), (D.KEY_COUNT, 0, False)]).tolist() == [2, 5, 1, 0, 3]
    assert D.order_groups([2, 3], sums, counts,
                          [(D.KEY_GROUP_COLUMN, 0, True), (D.KEY_SUM, 0, True)]).tolist() == [5, 3, 1, 2, 0]


def test_sorted_domain_makes_the_dense_result_ordered_by_the_grouping_attributes():
    # Section 2.5: with codes taken from the sorted domain, ascending group index IS ascending
    # (attribute of dimension 0, attribute of dimension 1) order; ordering by the columns is the identity
    r = np.random.default_rng(9)
    attr0, attr1 = r.integers(1990, 1999, size=40), r.integers(-5, 5, size=25)
    (v0, c0), (v1, c1) = D.group_domain([attr0]), D.group_domain([attr1])
    n = 3000
    fk0, fk1 = r.integers(0, 40, size=n).astype(np.int32), r.integers(0, 25, size=n).astype(np.int32)
    meas = r.integers(1, 100, size=n).astype(np.int32)
    card = [len(v0), len(v1)]
    sums, counts = O.groupby_sum([fk0, fk1], [40, 25], [None, None], [c0.astype(np.int32), c1.astype(np.int32)],
                                 card, None, [meas])
    order = D.order_groups(card, sums, counts, [(D.KEY_GROUP_COLUMN, 0, False), (D.KEY_GROUP_COLUMN, 1, False)])
    assert order.tolist() == [g for g in range(card[0] * card[1]) if counts[g] > 0]
    # and equals the relational answer: sort the joined tuples' distinct (attr0, attr1) pairs
    pairs = sorted(set(zip(attr0[fk0].tolist(), attr1[fk1].tolist())))
    assert [(int(v0[g // card[1], 0]), int(v1[g % card[1], 0])) for g in order] == pairs
    by_pair = {}
    for a, b, m in zip(attr0[fk0].tolist(), attr1[fk1].tolist(), meas.tolist()):
        by_pair[(a, b)] = by_pair.get((a, b), 0) + m
    assert [int(sums[0, g]) for g in order] == [by_pair[p] for p in pairs]
