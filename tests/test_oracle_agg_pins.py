"""Pins for the wider aggregate oracle: numpy boolean-mask evaluation, reduction to the plain
group-by-sum oracle, dense linear-algebra form with a Hadamard product, hand-worked numbers.  CPU."""
import numpy as np

from oracle import lq_oracle as O


def _inputs(seed, n=400, rows=(6, 9, 4), card=(3, 4, 1)):
    r = np.random.default_rng(seed)
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    fks[2][r.integers(0, n, size=7)] = -1
    codes = [r.integers(0, card[0], size=rows[0]).astype(np.int32), r.integers(0, card[1], size=rows[1]).astype(np.int32), None]
    masks = [None, (r.random(rows[1]) < 0.7).astype(np.uint8), (r.random(rows[2]) < 0.6).astype(np.uint8)]
    cols = {name: r.integers(lo, hi, size=n).astype(np.int32)
            for name, lo, hi in (("price", 1, 100_000), ("disc", 0, 11), ("qty", 1, 51), ("cost", 1, 60_000))}
    return fks, list(rows), masks, codes, list(card), cols


def test_matches_numpy_boolean_mask_evaluation():
    fks, rows, masks, codes, card, c = _inputs(1)
    preds = [(c["disc"], 1, 3), (c["qty"], -10, 24)]
    meas = [("mul", c["price"], c["disc"]), ("sub", c["price"], c["cost"]), ("col", c["qty"], None)]
    sums, mins, maxs, counts = O.groupby_agg(fks, rows, masks, codes, card, preds, meas)
    keep = (c["disc"] >= 1) & (c["disc"] <= 3) & (c["qty"] <= 24)
    g = np.zeros(len(keep), dtype=np.int64)
    for k in range(3):
        ok = fks[k] >= 0
        j = np.where(ok, fks[k], 0)
        keep &= ok
        if masks[k] is not None:
            keep &= masks[k][j].astype(bool)
        if codes[k] is not None:
            g = g * card[k] + codes[k][j]
    vals = [c["price"].astype(np.int64) * c["disc"], c["price"].astype(np.int64) - c["cost"], c["qty"].astype(np.int64)]
    for m, v in enumerate(vals):
        for grp in range(12):
            sel = keep & (g == grp)
            assert sums[m, grp] == v[sel].sum()
            assert counts[grp] == sel.sum()
            if sel.any():
                assert mins[m, grp] == v[sel].min() and maxs[m, grp] == v[sel].max()
            else:
                assert mins[m, grp] == np.iinfo(np.int64).max and maxs[m, grp] == np.iinfo(np.int64).min


def test_reduces_to_the_plain_group_by_sum():
    fks, rows, masks, codes, card, c = _inputs(2)
    s0, c0 = O.groupby_sum(fks, rows, masks, codes, card, None, [c["price"], c["qty"]])
    s1, _, _, c1 = O.groupby_agg(fks, rows, masks, codes, card, [], [("col", c["price"], None), ("col", c["qty"], None)])
    np.testing.assert_array_equal(s0, s1)
    np.testing.assert_array_equal(c0, c1)
    # a range predicate is the same thing as a fact mask
    fm = ((c["disc"] >= 2) & (c["disc"] <= 5)).astype(np.uint8)
    s2, c2 = O.groupby_sum(fks, rows, masks, codes, card, fm, [c["price"]])
    s3, _, _, c3 = O.groupby_agg(fks, rows, masks, codes, card, [(c["disc"], 2, 5)], [("col", c["price"], None)])
    np.testing.assert_array_equal(s2, s3)
    np.testing.assert_array_equal(c2, c3)


def test_dense_linear_algebra_form_with_hadamard_measure():
    """sum(price * disc) grouped by one dimension: (I E)^T (s * price * disc), all dense."""
    r = np.random.default_rng(3)
    n, rows, card = 40, 5, 3
    fk = r.integers(0, rows, size=n).astype(np.int32)
    code = r.integers(0, card, size=rows).astype(np.int32)
    price, disc = r.integers(1, 100, size=n).astype(np.int32), r.integers(0, 10, size=n).astype(np.int32)
    s = ((disc >= 3) & (disc <= 7)).astype(np.int64)
    I = np.zeros((n, rows), dtype=np.int64); I[np.arange(n), fk] = 1
    E = np.zeros((rows, card), dtype=np.int64); E[np.arange(rows), code] = 1
    want = (I @ E).T @ (s * price.astype(np.int64) * disc)
    sums, _, _, counts = O.groupby_agg([fk], [rows], None, [code], [card], [(disc, 3, 7)], [("mul", price, disc)])
    np.testing.assert_array_equal(sums[0], want)
    np.testing.assert_array_equal(counts, (I @ E).T @ s)


def test_hand_worked_rows():
    """Rows (key, price, disc): (0,10,2) (1,7,5) (0,3,2) (1,100,9) (0,50,0); predicate 1 <= disc <= 5;
    dimension rows 0,1 -> groups 1,0.  Kept: rows 0,1,2.  Group 1: 10*2 + 3*2 = 26 (min 6, max 20, count 2);
    group 0: 7*5 = 35 (count 1)."""
    fk = np.array([0, 1, 0, 1, 0], dtype=np.int32)
    price = np.array([10, 7, 3, 100, 50], dtype=np.int32)
    disc = np.array([2, 5, 2, 9, 0], dtype=np.int32)
    sums, mins, maxs, counts = O.groupby_agg([fk], [2], None, [np.array([1, 0], dtype=np.int32)], [2],
                                             [(disc, 1, 5)], [("mul", price, disc)])
    assert sums.tolist() == [[35, 26]] and counts.tolist() == [1, 2]
    assert mins.tolist() == [[35, 6]] and maxs.tolist() == [[35, 20]]


def test_products_do_not_wrap_at_32_bits():
    fk = np.zeros(3, dtype=np.int32)
    a = np.array([2**31 - 1, -2**31, 2**31 - 1], dtype=np.int32)
    b = np.array([2**31 - 1, 2**31 - 1, -2**31], dtype=np.int32)
    sums, mins, maxs, _ = O.groupby_agg([fk], [1], None, None, [1], [], [("mul", a, b), ("sub", a, b)])
    assert sums[0, 0] == (2**31 - 1) ** 2 + 2 * (-2**31) * (2**31 - 1)
    assert sums[1, 0] == 0 + (-2**31 - (2**31 - 1)) + (2**31 - 1 + 2**31)
    assert maxs[0, 0] == (2**31 - 1) ** 2 and mins[1, 0] == -2**32 + 1


def test_avg_is_the_exact_mean_of_the_group_rounded_once():
    """AVG against the mean computed exactly (Python fractions over the surviving rows of each group, rounded to
    fp64 once): sums stay below 2^53, so SUM / COUNT in fp64 is that same correctly rounded quotient; a group
    without rows gives NaN; hand-worked: values 1, 2, 4 -> 7/3."""
    from fractions import Fraction
    r = np.random.default_rng(9)
    n, rows, card = 5_000, (13, 9), (13, 3)
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    codes = [r.integers(0, c, size=a).astype(np.int32) for a, c in zip(rows, card)]
    codes[1][:] = np.arange(9) % 2                                   # code 2 of the second table never occurs
    masks = [None, (r.random(9) < 0.7).astype(np.uint8)]
    a, b = r.integers(-10**5, 10**5, size=n).astype(np.int32), r.integers(1, 50, size=n).astype(np.int32)
    sums, _, _, counts = O.groupby_agg(fks, rows, masks, codes, card, [], [("mul", a, b), ("col", a, None)])
    avgs = O.group_avg(sums, counts)
    exact = {}
    for i in range(n):
        if not masks[1][fks[1][i]]:
            continue
        g = int(codes[0][fks[0][i]]) * 3 + int(codes[1][fks[1][i]])
        exact.setdefault(g, []).append((int(a[i]) * int(b[i]), int(a[i])))
    for g in range(39):
        if g not in exact:
            assert counts[g] == 0 and np.isnan(avgs[:, g]).all()
        else:
            for m in range(2):
                want = float(Fraction(sum(v[m] for v in exact[g]), len(exact[g])))
                assert avgs[m, g] == want
    assert np.isnan(avgs[:, 2::3]).all() and len(exact) >= 10          # code 2 never occurs; many groups do
    hand = O.group_avg(np.array([[7, -9, 0]]), np.array([3, 2, 0]))
    assert hand[0, 0] == 7 / 3 and hand[0, 1] == -4.5 and np.isnan(hand[0, 2])
