"""GPU parity of the masked star-join group-by against the int64 oracle: bit-exact."""
import numpy as np
import pytest
import torch

from oracle import lq_oracle as O
from tests.helpers import cpu_list, to_dev
from workloads import star as WL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _oracle(w, nthreads=8):
    return O.groupby_sum(cpu_list(w.fks), w.dim_rows, cpu_list(w.dim_mask), cpu_list(w.dim_code),
                         w.group_card, None if w.fact_mask is None else w.fact_mask.cpu(),
                         cpu_list(w.measures), nthreads=nthreads)


def _gpu(lq, w, **kw):
    sums, counts = lq.lq_masked_groupby_sum(w.fks, w.dim_rows, w.dim_mask, w.dim_code, w.group_card,
                                            w.fact_mask, w.measures, **kw)
    torch.cuda.synchronize()
    return sums.cpu().numpy(), None if counts is None else counts.cpu().numpy()


def _check(lq, w, **kw):
    ws, wc = _oracle(w)
    w = to_dev(w)
    s, c = _gpu(lq, w, **kw)
    np.testing.assert_array_equal(s, ws)
    np.testing.assert_array_equal(c, wc)
    return w, ws, wc


def _random_groupby(seed, n, rows, card, n_measures=2, fact_mask=True, neg=False, sel=(0.8, 0.5, 0.6)):
    r = np.random.default_rng(seed)
    K = len(rows)
    fks = [torch.from_numpy(r.integers(0, a, size=n).astype(np.int32)) for a in rows]
    if neg:
        fks[K - 1][torch.from_numpy(r.integers(0, n, size=max(1, n // 50)))] = -1
    codes = [torch.from_numpy(r.integers(0, card[k], size=rows[k]).astype(np.int32)) if card[k] > 1 else None
             for k in range(K)]
    masks = [None] + [torch.from_numpy((r.random(rows[k]) < sel[(k - 1) % len(sel)]).astype(np.uint8))
                      for k in range(1, K)]
    meas = [torch.from_numpy(r.integers(-100_000, 100_001, size=n).astype(np.int32)) for _ in range(n_measures)]
    fm = torch.from_numpy((r.random(n) < 0.9).astype(np.uint8)) if fact_mask else None
    return WL.GroupByWorkload("rand", n, fks, list(rows), masks, codes, list(card), fm, meas)


def test_config3_both_variants_full_size(lq):
    for variant in ("A", "B"):
        w = WL.c3_groupby(variant=variant)
        w, ws, wc = _check(lq, w)
        populated = int((wc > 0).sum())
        assert populated == (175 if variant == "A" else 35)
        frac = wc.sum() / w.n
        assert (0.015 < frac < 0.035) if variant == "A" else (0.002 < frac < 0.02)
        # twice more: integer atomics make the result independent of scheduling
        for _ in range(2):
            s, c = _gpu(lq, w)
            np.testing.assert_array_equal(s, ws)
            np.testing.assert_array_equal(c, wc)


def test_config3_two_measures(lq):
    _check(lq, WL.c3_groupby(n=1_000_003, n_measures=2))


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 1023, 4096, 4099, 100_001])
def test_ragged_sizes(lq, n):
    _check(lq, _random_groupby(10 + n, n, (7, 11, 5, 13), (3, 4, 1, 1)))


def test_negative_keys_drop_rows(lq):
    _check(lq, _random_groupby(30, 50_001, (9, 40, 33), (5, 1, 1), neg=True))


def test_no_grouping_is_a_plain_masked_sum(lq):
    w = _random_groupby(31, 70_003, (50, 60), (1, 1), n_measures=1)
    w, ws, wc = _check(lq, w)
    assert ws.shape == (1, 1)


def test_no_masks_no_fact_mask_counts_every_row(lq):
    w = _random_groupby(32, 33_333, (6, 9), (6, 9), fact_mask=False)
    w.dim_mask = [None, None]
    w, ws, wc = _check(lq, w)
    assert wc.sum() == 33_333


def test_empty_and_full_selections(lq):
    w = _random_groupby(33, 20_000, (10, 20, 30), (2, 5, 1))
    w.dim_mask[2] = torch.zeros(30, dtype=torch.uint8)
    w, ws, wc = _check(lq, w)
    assert wc.sum() == 0 and ws.sum() == 0
    w = _random_groupby(34, 20_000, (10, 20, 30), (2, 5, 1), fact_mask=False)
    w.dim_mask = [torch.ones(r, dtype=torch.uint8) for r in (10, 20, 30)]
    w, ws, wc = _check(lq, w)
    assert wc.sum() == 20_000


def test_three_grouping_dimensions_and_wide_codes(lq):
    # 3 grouping dimensions; one with cardinality > 255 (16-bit side table)
    _check(lq, _random_groupby(35, 60_000, (400, 30, 8, 50), (300, 3, 2, 1), n_measures=1))
    _check(lq, _random_groupby(36, 60_000, (40, 30, 8), (10, 10, 8), n_measures=4))


def test_both_sides_of_the_lds_accumulator_limit(lq):
    # 64 x 64 = 4,096 groups with one measure: (M + 1) * G = 8,192 accumulators, the most a workgroup keeps
    # in LDS; with two measures the same groups need 12,288 and the output arrays accumulate instead
    _check(lq, _random_groupby(43, 300_001, (500, 700, 20), (64, 64, 1), n_measures=1))
    _check(lq, _random_groupby(44, 300_001, (500, 700, 20), (64, 64, 1), n_measures=2))
    w = to_dev(_random_groupby(44, 1_000, (500, 700), (65_535, 65_535), n_measures=2))
    with pytest.raises(lq.LQError) as e:                     # more than 2^30 groups
        lq.lq_masked_groupby_sum(w.fks, w.dim_rows, w.dim_mask, w.dim_code, w.group_card, w.fact_mask, w.measures,
                                 sums=torch.empty((2, 1), dtype=torch.int64, device="cuda"),
                                 counts=torch.empty((1,), dtype=torch.int64, device="cuda"),
                                 ws=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == "LQ_ERR_UNSUPPORTED"


def test_side_tables_too_large_for_lds_are_read_from_memory(lq):
    # 400,000 + 300,000 byte-coded rows exceed the 160 KB of LDS
    _check(lq, _random_groupby(37, 300_007, (400_000, 300_000, 1_000), (7, 5, 1), n_measures=1))


def test_mixed_residency_small_tables_in_lds_large_ones_in_memory(lq):
    # byte table of 500,000 rows and bitmap of 2,000,000 rows stay in memory, the 3,000-row byte
    # table lives in LDS; memory tables are only consulted for rows the LDS predicates let through
    _check(lq, _random_groupby(41, 200_003, (500_000, 3_000, 2_000_000), (7, 5, 1), n_measures=2))
    # one large bitmap in memory, everything else in LDS (the 16x-scaled star-schema shape)
    _check(lq, _random_groupby(42, 150_001, (2_556, 100_000, 32_000, 1_500_000), (7, 25, 1, 1), n_measures=1,
                               fact_mask=False))


def test_unaligned_columns_take_the_scalar_path(lq):
    w = _random_groupby(38, 40_001, (20, 30), (4, 5))
    ws, wc = _oracle(w)
    w = to_dev(w)
    # shift every column by one element so that no pointer is 16-byte aligned
    def shift(t):
        buf = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda")
        buf[1:] = t
        return buf[1:]
    w.fks = [shift(f) for f in w.fks]
    w.measures = [shift(m) for m in w.measures]
    w.fact_mask = shift(w.fact_mask)
    s, c = _gpu(lq, w)
    np.testing.assert_array_equal(s, ws)
    np.testing.assert_array_equal(c, wc)


def test_counts_are_optional_and_outputs_are_overwritten(lq):
    w = _random_groupby(39, 10_000, (5, 6), (5, 6))
    ws, wc = _oracle(w)
    w = to_dev(w)
    sums = torch.full((2, 30), 123456789, dtype=torch.int64, device="cuda")
    s, c = _gpu(lq, w, sums=sums, want_counts=False)
    assert c is None
    np.testing.assert_array_equal(s, ws)


def test_check_fks_flag(lq):
    w = to_dev(_random_groupby(40, 9_000, (5, 6), (5, 6)))
    _gpu(lq, w, flags=lq.LQ_CHECK_FKS)
    w.fks[1][77] = 6
    with pytest.raises(lq.LQError) as e:
        _gpu(lq, w, flags=lq.LQ_CHECK_FKS)
    assert e.value.status == "LQ_ERR_FK_RANGE"
    w.fks[1][77] = -5                                        # negative = no match: allowed
    _gpu(lq, w, flags=lq.LQ_CHECK_FKS)


def test_check_flag_also_covers_the_group_codes(lq):
    """A code outside [0, group_card) on a dimension row that passes its mask would address an accumulator
    that does not exist: the checked call reports it (outputs untouched); the same code on a row that its
    mask filters out is never looked up and is fine."""
    w = _random_groupby(41, 9_000, (50, 60), (5, 6), sel=(1.0,))
    want_s, want_c = _oracle(w)
    w = to_dev(w)
    sums = torch.full((2, 30), 7, dtype=torch.int64, device="cuda")
    for bad in (6, 1 << 20, -1):
        code = w.dim_code[1].clone()
        code[17] = bad
        w2 = WL.GroupByWorkload("bad", w.n, w.fks, w.dim_rows, w.dim_mask, [w.dim_code[0], code], w.group_card,
                                w.fact_mask, w.measures)
        with pytest.raises(lq.LQError) as e:
            _gpu(lq, w2, sums=sums, flags=lq.LQ_CHECK_FKS)
        assert e.value.status == "LQ_ERR_SHAPE" and "group code" in str(e.value)
        torch.cuda.synchronize()
        assert (sums == 7).all()
    # the offending row filtered out by its mask: accepted, and the result is the oracle's for that mask
    mask = w.dim_mask[1].clone()
    mask[17] = 0
    code = w.dim_code[1].clone()
    code[17] = 1 << 20
    w3 = WL.GroupByWorkload("masked", w.n, w.fks, w.dim_rows, [w.dim_mask[0], mask], [w.dim_code[0], code],
                            w.group_card, w.fact_mask, w.measures)
    s, c = _gpu(lq, w3, flags=lq.LQ_CHECK_FKS)
    code_ok = w.dim_code[1].clone()
    w4 = WL.GroupByWorkload("masked_ok", w.n, cpu_list(w.fks), w.dim_rows, cpu_list([w.dim_mask[0], mask]),
                            cpu_list([w.dim_code[0], code_ok]), w.group_card, w.fact_mask.cpu(), cpu_list(w.measures))
    ws, wc = _oracle(w4)
    np.testing.assert_array_equal(s, ws)
    np.testing.assert_array_equal(c, wc)


def test_call_on_a_side_stream_keeps_its_temporaries(lq):
    """The binding allocates the workspace and the outputs itself; the kernels run on the caller's stream.
    Allocating and overwriting on the default stream right after the call must not hand those blocks out
    again while the side stream still uses them."""
    w = WL.c3_groupby(n=2_000_003)
    want_s, want_c = _oracle(w)
    w = to_dev(w)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    for _ in range(3):
        s, c = lq.lq_masked_groupby_sum(w.fks, w.dim_rows, w.dim_mask, w.dim_code, w.group_card, w.fact_mask,
                                        w.measures, stream=side)
        junk = [torch.full((1 << 18,), -1, dtype=torch.int64, device="cuda") for _ in range(16)]
        small = [torch.full((175,), -1, dtype=torch.int64, device="cuda") for _ in range(64)]
        side.synchronize()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(s.cpu().numpy(), want_s)
        np.testing.assert_array_equal(c.cpu().numpy(), want_c)
        del junk, small


def test_reuse_side_tables_skips_the_dimension_pass_and_gives_the_same_result(lq):
    # first call encodes the dimension side into the workspace; the following ones reuse it over
    # other fact rows, another fact mask and other measures
    w = _random_groupby(45, 120_001, (2_556, 3_000, 500_000), (7, 25, 1))
    ws_, wc_ = _oracle(w)
    w = to_dev(w)
    ws = torch.empty(lq.lq_groupby_workspace_bytes(w.dim_rows, w.group_card, len(w.measures)),
                     dtype=torch.uint8, device="cuda")
    s, c = _gpu(lq, w, ws=ws, flags=lq.LQ_CHECK_FKS)
    np.testing.assert_array_equal(s, ws_)
    for _ in range(2):
        s, c = _gpu(lq, w, ws=ws, flags=lq.LQ_REUSE_SIDE_TABLES | lq.LQ_CHECK_FKS)
        np.testing.assert_array_equal(s, ws_)
        np.testing.assert_array_equal(c, wc_)
    w2 = _random_groupby(46, 77_777, (2_556, 3_000, 500_000), (7, 25, 1))
    w2.dim_mask = [None if m is None else m.cpu() for m in w.dim_mask]
    w2.dim_code = [None if m is None else m.cpu() for m in w.dim_code]
    ws2, wc2 = _oracle(w2)
    w2 = to_dev(w2)
    w2.dim_mask, w2.dim_code = w.dim_mask, w.dim_code            # the very same device arrays
    s, c = _gpu(lq, w2, ws=ws, flags=lq.LQ_REUSE_SIDE_TABLES)
    np.testing.assert_array_equal(s, ws2)
    np.testing.assert_array_equal(c, wc2)


# ---------------------------------------------------------------- more groups than LDS accumulators
# The multi-column group-by of Section 2.4.2 multiplies the cardinalities of its grouping attributes:
# above 8,192 accumulators the output arrays themselves accumulate (device-wide atomics).

def _many_groups(seed, n, rows, card, n_measures, sel=None, fact_mask=False, hot=False, neg=False):
    r = np.random.default_rng(seed)
    K = len(rows)
    fks = [torch.from_numpy(r.integers(0, a, size=n).astype(np.int32)) for a in rows]
    if hot and n:        # most fact rows point at the same few dimension rows: many lanes hit one group
        for f, a in zip(fks, rows):
            f[torch.from_numpy(r.random(n) < 0.7)] = int(r.integers(0, a))
    if neg and n:
        fks[K - 1][torch.from_numpy(r.integers(0, n, size=max(1, n // 50)))] = -1
    codes = [torch.from_numpy(r.integers(0, card[k], size=rows[k]).astype(np.int32)) if card[k] > 1 else None
             for k in range(K)]
    masks = [None if sel is None or sel[k] is None else torch.from_numpy((r.random(rows[k]) < sel[k]).astype(np.uint8))
             for k in range(K)]
    meas = [torch.from_numpy(r.integers(-100_000, 100_001, size=n).astype(np.int32)) for _ in range(n_measures)]
    fm = torch.from_numpy((r.random(n) < 0.9).astype(np.uint8)) if fact_mask else None
    return WL.GroupByWorkload("many_groups", n, fks, list(rows), masks, codes, list(card), fm, meas)


@pytest.mark.parametrize("n_measures", [1, 4])
def test_three_grouping_attributes_25_25_250(lq, n_measures):
    # 156,250 groups; the fourth dimension only filters (about 2.4 % of the fact rows survive)
    w = _many_groups(300 + n_measures, 1_500_003, (2_556, 30_000, 2_000, 200_000), (25, 25, 250, 1), n_measures,
                     sel=(None, 0.2, None, 0.12))
    w, ws, wc = _check(lq, w)
    assert ws.shape == (n_measures, 156_250) and 10_000 < (wc > 0).sum() < 156_250      # most groups stay empty


@pytest.mark.parametrize("n_measures", [1, 4])
def test_one_million_groups_every_row_survives(lq, n_measures):
    # 1000 x 1000 groups (16-bit codes), no predicate: 2M atomics per measure, every group about twice
    w = _many_groups(310 + n_measures, 2_000_001, (5_000, 70_000), (1_000, 1_000), n_measures)
    w, ws, wc = _check(lq, w)
    assert wc.sum() == w.n and (wc > 0).sum() > 800_000


def test_many_groups_with_a_few_hot_ones(lq):
    # 70 % of the rows fall into one group: the lanes of a wavefront are merged before the atomic
    w = _many_groups(320, 3_000_017, (300, 300), (300, 300), 2, hot=True, fact_mask=True)
    w, ws, wc = _check(lq, w)
    assert wc.max() > 0.4 * wc.sum()


@pytest.mark.parametrize("n", [0, 1, 5, 63, 64, 65, 1_023, 4_099])
def test_many_groups_ragged_sizes_negative_keys_fact_mask(lq, n):
    _check(lq, _many_groups(330 + n, n, (70, 110, 50, 13), (30, 40, 9, 1), 2, sel=(None, 0.8, 0.5, 0.6),
                            fact_mask=True, neg=True))


def test_many_groups_unaligned_columns_counts_optional_and_flags(lq):
    w = _many_groups(340, 300_001, (700, 1_100, 40_000), (100, 120, 1), 1, sel=(None, None, 0.5))
    ws_, wc_ = _oracle(w)
    w = to_dev(w)
    # columns that start 4 bytes past a 16-byte boundary: the one-row-per-lane form of the scan
    off = lambda t: torch.cat([torch.zeros(1, dtype=t.dtype, device="cuda"), t])[1:]
    w.fks = [off(f) for f in w.fks]
    w.measures = [off(m) for m in w.measures]
    s, c = _gpu(lq, w)
    np.testing.assert_array_equal(s, ws_)
    np.testing.assert_array_equal(c, wc_)
    sums = torch.full((1, 12_000), 99, dtype=torch.int64, device="cuda")
    s, c = _gpu(lq, w, sums=sums, want_counts=False)
    assert c is None
    np.testing.assert_array_equal(s, ws_)
    # checked call, then the same query again on the encoded side tables
    ws = torch.empty(lq.lq_groupby_workspace_bytes(w.dim_rows, w.group_card, 1), dtype=torch.uint8, device="cuda")
    s, c = _gpu(lq, w, ws=ws, flags=lq.LQ_CHECK_FKS)
    np.testing.assert_array_equal(s, ws_)
    s, c = _gpu(lq, w, ws=ws, flags=lq.LQ_REUSE_SIDE_TABLES)
    np.testing.assert_array_equal(s, ws_)
    np.testing.assert_array_equal(c, wc_)
    w.fks[0][123] = 700
    with pytest.raises(lq.LQError) as e:
        _gpu(lq, w, ws=ws, flags=lq.LQ_CHECK_FKS)
    assert e.value.status == "LQ_ERR_FK_RANGE"


@pytest.mark.parametrize("rows,card,sel,n_measures", [
    ((2_556, 30_000, 2_000, 200_000), (25, 25, 250, 1), (None, 0.2, None, 0.12), 2),     # all side tables in LDS
    ((400_000, 300, 250, 900_000), (200, 200, 3, 1), (0.5, None, None, 0.3), 1),         # a code table and a bitmap stay in memory
    ((300, 250), (250, 250), (None, 0.9), 2),                                            # two grouping tables only
    ((400_000, 300_000, 900, 700_000), (200, 150, 3, 1), (None, 0.8, None, 0.5), 2),     # two code tables and a bitmap in memory
    ((400_000, 300_000), (20, 15), (0.9, None), 1),                                      # the same with accumulators in LDS
], ids=["lds_tables_m2", "tables_in_memory", "two_tables_m2", "two_code_tables_in_memory", "two_code_tables_in_memory_lds_acc"])
def test_many_groups_on_the_specialised_scan(lq, rows, card, sel, n_measures):
    # aligned columns, no fact mask, byte codes and bitmaps, one or two measures: the compile-time specialised scan
    w = _many_groups(350 + len(rows) + n_measures, 777_777, rows, card, n_measures, sel=sel, neg=True)
    _check(lq, w)


def test_many_groups_through_buckets_and_through_atomics(lq):
    """The two forms of the many-groups group-by on the same query: with the small workspace the survivors go through
    device-wide atomics, with lq_groupby_bucket_workspace_bytes they are sorted into buckets first; both equal the oracle.
    Also with most rows in a few groups (a bucket runs out of slots and the rest takes the atomics) and with a workspace
    one byte short of the bucketed form."""
    for seed, hot, nm in ((350, False, 1), (351, True, 2), (352, False, 2)):
        # (grouping attributes of at most 255 values: side tables of bytes, the specialised scan in both forms)
        w = _many_groups(seed, 2_000_003, (300, 280, 5_000), (250, 240, 1), nm, sel=(None, None, 0.7), hot=hot)
        ws_, wc_ = _oracle(w)
        w = to_dev(w)
        small = lq.lq_groupby_workspace_bytes(w.dim_rows, w.group_card, nm)
        big = lq.lq_groupby_bucket_workspace_bytes(w.n, w.dim_rows, w.group_card, nm)
        assert big > small + 2 * 4 * (1 + nm) * w.n
        for size in (small, big - 1, big):
            ws = torch.empty(size, dtype=torch.uint8, device="cuda")
            s, c = _gpu(lq, w, ws=ws)
            np.testing.assert_array_equal(s, ws_, err_msg=f"seed {seed}, workspace {size}")
            np.testing.assert_array_equal(c, wc_, err_msg=f"seed {seed}, workspace {size}")
    # the bucketed form does not apply: few accumulators, three measures
    assert lq.lq_groupby_bucket_workspace_bytes(1_000_000, [300, 280], [30, 28], 1) == 0
    assert lq.lq_groupby_bucket_workspace_bytes(1_000_000, [300, 280], [250, 240], 3) == \
        lq.lq_groupby_bucket_workspace_bytes(1_000_000, [300, 280], [250, 240], 2)
    assert lq.lq_groupby_bucket_workspace_bytes(0, [300, 280], [250, 240], 1) == 0


@pytest.mark.parametrize("n", [1, 5, 1_023, 4_099, 70_001])
def test_bucketed_many_groups_ragged_sizes_and_negative_keys(lq, n):
    # no fact mask, aligned columns: the specialised scan, with the default (large) workspace the bucketed form
    _check(lq, _many_groups(360 + n, n, (70, 110, 50, 130), (70, 110, 3, 1), 2, sel=(None, 0.8, 0.5, 0.6), neg=True))


@pytest.mark.parametrize("card,n_measures", [
    ((91, 91), 1),                  # 8,281 groups: just past the LDS limit at one measure, buckets of 32 groups
    ((65, 64), 2),                  # 4,160 groups x 3 accumulators: buckets of 16
    ((200, 173, 87), 1),            # 3.0e6 groups, not a multiple of the bucket size (4,096 groups each)
    ((255, 255, 255), 2),           # 1.66e7 groups: 8,097 buckets of 2,048, close to the most the form takes
    ((255, 255, 255, 3), 1),        # 5.0e7 groups: more buckets than the form takes, the atomic form runs
], ids=["8281x1", "4160x2", "3.0e6x1", "1.66e7x2", "5.0e7x1"])
def test_bucketed_many_groups_bucket_geometries(lq, card, n_measures):
    # (grouping attributes of at most 255 values each: the side tables the specialised scan takes)
    rows = tuple(c + 5 for c in card) + (40,)
    w = _many_groups(370 + card[0] + len(card), 200_003, rows, tuple(card) + (1,), n_measures,
                     sel=(None,) * len(card) + (0.9,))
    _check(lq, w)


@pytest.mark.parametrize("n", [3, 4_098, 600_001])
@pytest.mark.parametrize("card,n_measures", [
    ((7, 25), 2),                   # accumulators in LDS
    ((), 1),                        # no grouping: a filtered sum
    ((200, 173), 1),                # 34,600 groups: buckets (atomics with the small workspace)
    ((250, 240), 3),                # three measures over many groups: two bucketed calls
    ((1_000, 9), 2),                # a 16-bit code table
], ids=["lds", "one_group", "buckets", "buckets_m3", "wide_codes"])
def test_fact_mask_on_the_specialised_scan(lq, card, n_measures, n):
    """The fact table's own selection vector (one byte per fact row, Section 2.2) on the compile-time specialised
    scans: accumulators in LDS, through buckets and through atomics, ragged sizes, rows dropped by a negative key as
    well.  (A mask that is not 4-byte aligned takes the generic scan: test_unaligned_columns_take_the_scalar_path.)"""
    rows = tuple(c + 3 for c in card) + (60,)
    w = _many_groups(390 + len(card) + n_measures, n, rows, tuple(card) + (1,), n_measures,
                     sel=(None,) * len(card) + (0.8,), fact_mask=True, neg=True)
    assert w.fact_mask is not None and (n < 100 or int(w.fact_mask.sum()) < n)
    w, ws_, wc_ = _check(lq, w)
    if len(card) == 2 and card[0] * card[1] > 8_192 and n_measures <= 2:
        small = torch.empty(lq.lq_groupby_workspace_bytes(w.dim_rows, w.group_card, n_measures), dtype=torch.uint8, device="cuda")
        s, c = _gpu(lq, w, ws=small)
        np.testing.assert_array_equal(s, ws_)
        np.testing.assert_array_equal(c, wc_)


def test_bucketed_many_groups_all_rows_in_one_group(lq):
    # every row in one group: its bucket fills up and the rest goes through the merged atomics
    w = _many_groups(380, 1_000_003, (300, 300), (300, 300), 1)
    for f in w.fks:
        f[:] = 7
    w, ws, wc = _check(lq, w)
    assert (wc > 0).sum() == 1 and wc.max() == 1_000_003


@pytest.mark.parametrize("card,n_measures,sel", [
    ((300, 9), 2, (None, None, 0.5)),            # 2,700 groups x 3 accumulators: LDS form with a 16-bit code table
    ((1_000, 7), 1, (None, None, 0.3)),          # 7,000 groups x 2: past the LDS limit (a brand x year query)
    ((1_000, 250), 2, (0.9, None, None)),        # 250,000 groups, two measures, a masked grouping table
    ((40_000, 3), 1, (None, None, None)),        # a 16-bit table too large for LDS, every row survives
], ids=["lds_2700x3", "7000x2", "250000x3", "table_in_memory"])
def test_grouping_attributes_of_more_than_255_values_on_the_specialised_scan(lq, card, n_measures, sel):
    """Code tables of 16-bit entries on the specialised scan (no fact mask, aligned columns), in its LDS form, through
    atomics (small workspace) and through buckets (default workspace)."""
    rows = (card[0] + 17, card[1] + 3, 900)
    w = _many_groups(390 + card[0] % 97, 300_007, rows, tuple(card) + (1,), n_measures, sel=sel, neg=True)
    ws_, wc_ = _oracle(w)
    w = to_dev(w)
    small = torch.empty(lq.lq_groupby_workspace_bytes(w.dim_rows, w.group_card, n_measures), dtype=torch.uint8, device="cuda")
    for kw in ({}, {"ws": small}):
        s, c = _gpu(lq, w, **kw)
        np.testing.assert_array_equal(s, ws_)
        np.testing.assert_array_equal(c, wc_)
