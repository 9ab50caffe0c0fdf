"""GPU parity of the wider aggregate query (fact range predicates, product / difference measures,
SUM / MIN / MAX / COUNT) against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

from oracle import lq_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _case(seed, n, rows, card, big=False):
    r = np.random.default_rng(seed)
    K = len(rows)
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    if n:
        fks[-1][r.integers(0, n, size=max(1, n // 97))] = -1
    codes = [r.integers(0, card[k], size=rows[k]).astype(np.int32) if card[k] > 1 else None for k in range(K)]
    masks = [None] + [(r.random(rows[k]) < 0.6).astype(np.uint8) for k in range(1, K)]
    hi = 2**31 - 1 if big else 100_000
    cols = {"price": r.integers(-hi if big else 1, hi, size=n).astype(np.int32), "disc": r.integers(0, 11, size=n).astype(np.int32),
            "qty": r.integers(1, 51, size=n).astype(np.int32), "cost": r.integers(-hi if big else 1, hi, size=n).astype(np.int32)}
    return fks, list(rows), masks, codes, list(card), cols


def _check(lq, fks, rows, masks, codes, card, preds, meas):
    want = O.groupby_agg(fks, rows, masks, codes, card, preds, meas)
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    got = lq.lq_groupby_agg([dev(f) for f in fks], rows, [dev(m) for m in masks], [dev(c) for c in codes], card,
                            [(dev(c), lo, hi) for c, lo, hi in preds], [(op, dev(a), dev(b)) for op, a, b in meas])
    torch.cuda.synchronize()
    for name, w in zip(("sum", "min", "max", "count"), want):
        np.testing.assert_array_equal(got[name].cpu().numpy(), w, err_msg=name)
    return want


@pytest.mark.parametrize("n", [0, 1, 5, 1_023, 4_099, 300_001])
def test_product_and_difference_measures_with_fact_predicates(lq, n):
    fks, rows, masks, codes, card, c = _case(n + 1, n, (7, 40, 13), (7, 5, 1))
    preds = [(c["disc"], 1, 3), (c["qty"], 1, 24)]
    meas = [("mul", c["price"], c["disc"]), ("sub", c["price"], c["cost"]), ("col", c["qty"], None)]
    _check(lq, fks, rows, masks, codes, card, preds, meas)


def test_single_join_no_grouping_shape(lq):
    """One join, fact predicates, SUM of a product, no GROUP BY (the shape of the benchmark's group 1)."""
    fks, rows, masks, codes, card, c = _case(50, 500_003, (2_556,), (1,))
    masks = [(np.arange(2_556) % 7 == 3).astype(np.uint8)]
    want = _check(lq, fks, rows, masks, [None], [1], [(c["disc"], 1, 3), (c["qty"], 1, 24)], [("mul", c["price"], c["disc"])])
    assert want[3][0] > 1_000


def test_four_joins_difference_measure_shape(lq):
    """Four joins, two masks, GROUP BY two dimensions, SUM(a - b) (the shape of the benchmark's group 4)."""
    fks, rows, masks, codes, card, c = _case(51, 400_001, (2_556, 30_000, 2_000, 200_000), (7, 25, 1, 1))
    _check(lq, fks, rows, masks, codes, card, [], [("sub", c["price"], c["cost"])])


def test_full_range_int32_values_do_not_wrap(lq):
    fks, rows, masks, codes, card, c = _case(52, 50_001, (5, 9), (5, 3), big=True)
    _check(lq, fks, rows, masks, codes, card, [(c["disc"], 0, 10)], [("mul", c["price"], c["cost"]), ("sub", c["price"], c["cost"])])


def test_tables_too_large_for_lds_and_optional_outputs(lq):
    fks, rows, masks, codes, card, c = _case(53, 200_003, (300_000, 250_000), (4, 3))
    want = O.groupby_agg(fks, rows, masks, codes, card, [], [("col", c["price"], None)])
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    got = lq.lq_groupby_agg([dev(f) for f in fks], rows, [dev(m) for m in masks], [dev(x) for x in codes], card, [],
                            [("col", dev(c["price"]), None)], want=("sum", "count"))
    torch.cuda.synchronize()
    assert got["min"] is None and got["max"] is None
    np.testing.assert_array_equal(got["sum"].cpu().numpy(), want[0])
    np.testing.assert_array_equal(got["count"].cpu().numpy(), want[3])


def test_more_groups_than_lds_accumulators(lq):
    """25 x 25 x 250 groups with SUM / MIN / MAX / COUNT of a product and a difference: the outputs
    themselves accumulate (device-wide atomics), empty groups keep 0 / INT64_MAX / INT64_MIN."""
    fks, rows, masks, codes, card, c = _case(60, 700_001, (2_556, 30_000, 2_000, 200_000), (25, 25, 250, 1))
    want = _check(lq, fks, rows, masks, codes, card, [(c["qty"], 1, 40)],
                  [("mul", c["price"], c["disc"]), ("sub", c["price"], c["cost"])])
    empty = want[3] == 0
    assert empty.any() and (want[1][:, empty] == np.iinfo(np.int64).max).all() and (want[2][:, empty] == np.iinfo(np.int64).min).all()


def test_many_groups_full_range_values_and_one_hot_group(lq):
    fks, rows, masks, codes, card, c = _case(61, 400_003, (300, 301), (300, 301), big=True)
    fks[0][:] = 7                                  # one dimension row for everyone: 301 populated groups of 90,300
    _check(lq, fks, rows, masks, codes, card, [], [("mul", c["price"], c["cost"]), ("col", c["price"], None)])


def test_avg_from_sums_and_counts(lq):
    """AVG = SUM / COUNT in fp64, bit for bit the oracle's quotient; NaN exactly where a group has no rows; also on
    the accumulators-in-memory form (more than 8,192 accumulators) and with sums beyond 2^53."""
    for seed, n, rows, card, big in ((70, 300_001, (7, 40, 13), (7, 5, 1), False), (71, 200_003, (300, 301), (300, 301), True)):
        fks, rws, masks, codes, cd, c = _case(seed, n, rows, card, big=big)
        meas = [("mul", c["price"], c["cost"]), ("col", c["qty"], None)]
        want = O.groupby_agg(fks, rws, masks, codes, cd, [], meas)
        want_avg = O.group_avg(want[0], want[3])
        dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
        got = lq.lq_groupby_agg([dev(f) for f in fks], rws, [dev(m) for m in masks], [dev(x) for x in codes], cd, [],
                                [(op, dev(a), dev(b)) for op, a, b in meas], want=("sum", "count"))
        avg = lq.lq_group_avg(got["sum"], got["count"])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(avg.cpu().numpy(), want_avg)             # NaN == NaN in this comparison
        assert np.isnan(want_avg).any() == (want[3] == 0).any()


def test_long_scan_of_the_specialised_aggregate(lq):
    """More than eight steps per thread (over 16.8M fact rows): the specialised scan then consumes its measure
    columns at once instead of one step late; two joins, two predicates, a product, ragged row count."""
    fks, rows, masks, codes, card, c = _case(80, 20_000_003, (2_556, 300), (7, 1))
    _check(lq, fks, rows, masks, codes, card, [(c["disc"], 1, 3), (c["qty"], 1, 24)], [("mul", c["price"], c["disc"])])


@pytest.mark.parametrize("ops,want", [
    ((("sub", 0, 1),), ("sum", "count")),            # SUM(a - b): the profit measure of the fourth query group
    ((("col", 0, None),), ("sum",)),
    ((("col", 0, None), ("col", 2, None)), ("sum", "count")),
], ids=["sub", "col", "two_cols"])
def test_many_group_sums_without_predicates_take_the_plain_group_by(lq, ops, want):
    """Sums and counts without fact predicates over more groups than LDS holds: with the default (large) workspace the
    call runs the plain group-by's bucketed form, with the small one the aggregate's own scan; both equal the oracle."""
    import ctypes
    r = np.random.default_rng(77 + len(ops))
    n = 400_003
    rows, card = [300, 260, 900], [250, 240, 1]
    fks = [r.integers(0, a, size=n).astype(np.int32) for a in rows]
    fks[1][::97] = -1
    codes = [r.integers(0, card[k], size=rows[k]).astype(np.int32) if card[k] > 1 else None for k in range(3)]
    masks = [None, None, (r.random(rows[2]) < 0.6).astype(np.uint8)]
    cols = [r.integers(-50_000, 100_000, size=n).astype(np.int32) for _ in range(3)]
    meas = [(op, cols[a], None if b is None else cols[b]) for op, a, b in ops]
    ref = O.groupby_agg(fks, rows, masks, codes, card, [], meas)
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    d_fks, d_masks, d_codes = [dev(f) for f in fks], [dev(m) for m in masks], [dev(c) for c in codes]
    d_meas = [(op, dev(a), dev(b)) for op, a, b in meas]
    rows_c = (ctypes.c_int64 * 3)(*rows); card_c = (ctypes.c_int32 * 3)(*card)
    small = torch.empty(int(lq.binding._lib.lq_groupby_agg_workspace_bytes(3, rows_c, card_c, len(meas))), dtype=torch.uint8,
                        device="cuda")
    for kw in ({}, {"ws": small}):
        out = lq.lq_groupby_agg(d_fks, rows, d_masks, d_codes, card, [], d_meas, want=want, **kw)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out["sum"].cpu().numpy(), ref[0])
        if "count" in want:
            np.testing.assert_array_equal(out["count"].cpu().numpy(), ref[3])
