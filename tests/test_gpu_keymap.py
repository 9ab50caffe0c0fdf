"""GPU parity of the key -> row mapping (Algorithm 1's domain generation + row-matching matrix)
against the MM-Join oracle: bit-exact, including the COO form of I and its use by the group-by."""
import numpy as np
import pytest
import torch

from oracle import lq_oracle as O
from oracle import mmjoin_oracle as MJ

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _keys(seed, r, n, miss=0.05, lo=-2**31, hi=2**31 - 1):
    g = np.random.default_rng(seed)
    pool = np.unique(g.integers(lo, hi, size=int(r * 1.3) + 8, dtype=np.int64))
    g.shuffle(pool)
    key_S = pool[:r].astype(np.int32)
    extra = pool[r:]
    key_R = g.choice(key_S, size=n).astype(np.int32) if r else np.zeros(n, dtype=np.int32)
    if len(extra) and n:
        m = g.random(n) < miss
        key_R[m] = g.choice(extra, size=int(m.sum())).astype(np.int32)
    return key_S, key_R


@pytest.mark.parametrize("r,n", [(1, 1), (1, 100), (7, 1_000), (2_556, 100_003), (30_000, 200_001), (200_000, 1_000_000), (2_000, 1_200_003), (8_000, 1_100_000)])
def test_lookup_and_compaction_match_algorithm_1(lq, r, n):
    key_S, key_R = _keys(r + n, r, n)
    fk_w, rows_w, cols_w = MJ.key_to_row(key_R, key_S)
    table = lq.lq_keymap_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
    fk = lq.lq_keymap_lookup(table, torch.from_numpy(key_R).cuda())
    rows, cols, nnz = lq.lq_compact_matches(fk)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(fk.cpu().numpy(), fk_w)
    m = int(nnz.item())
    assert m == len(rows_w)
    np.testing.assert_array_equal(rows[:m].cpu().numpy(), rows_w)
    np.testing.assert_array_equal(cols[:m].cpu().numpy(), cols_w)


def test_extreme_key_values_and_no_matches(lq):
    key_S = np.array([-2**31, 2**31 - 1, 0, -1, 1], dtype=np.int32)
    key_R = np.array([0, -1, 2**31 - 1, -2**31, 5, 1, 1, -7], dtype=np.int32)
    table = lq.lq_keymap_build(torch.from_numpy(key_S).cuda())
    fk = lq.lq_keymap_lookup(table, torch.from_numpy(key_R).cuda())
    assert fk.cpu().tolist() == [2, 3, 1, 0, -1, 4, 4, -1]
    none = lq.lq_keymap_lookup(table, torch.full((1000,), 77, dtype=torch.int32, device="cuda"))
    rows, cols, nnz = lq.lq_compact_matches(none)
    assert int(nnz.item()) == 0 and (none == -1).all()
    rows, cols, nnz = lq.lq_compact_matches(torch.empty(0, dtype=torch.int32, device="cuda"))
    assert int(nnz.item()) == 0


def test_duplicate_dimension_keys_are_reported(lq):
    keys = torch.tensor([5, 9, 5, 3], dtype=torch.int32, device="cuda")
    with pytest.raises(lq.LQError) as e:
        lq.lq_keymap_build(keys, flags=lq.LQ_CHECK_KEYS)
    assert e.value.status == "LQ_ERR_DUPLICATE_KEY"


def test_incremental_insert_equals_rebuild(lq):
    """Updating a cached domain: keys of new dimension rows are inserted into the existing map."""
    key_S, key_R = _keys(99, 50_000, 300_000, miss=0.2)
    full = lq.lq_keymap_build(torch.from_numpy(key_S).cuda())
    part = lq.lq_keymap_build(torch.from_numpy(key_S[:30_000]).cuda(), max_keys=50_000)
    kr = torch.from_numpy(key_R).cuda()
    before = lq.lq_keymap_lookup(part, kr)
    lq.lq_keymap_insert(part, torch.from_numpy(key_S[30_000:]).cuda(), 30_000, flags=lq.LQ_CHECK_KEYS)
    after = lq.lq_keymap_lookup(part, kr)
    want = lq.lq_keymap_lookup(full, kr)
    torch.cuda.synchronize()
    assert torch.equal(after, want)
    fk_w, _, _ = MJ.key_to_row(key_R, key_S[:30_000])
    np.testing.assert_array_equal(before.cpu().numpy(), fk_w)


def test_mapped_keys_feed_the_group_by(lq):
    """End to end on raw key values: map four key columns, then aggregate; unmatched keys drop out."""
    g = np.random.default_rng(5)
    n, rows_k, card = 200_003, (50, 400, 30), (5, 7, 1)
    keys_S, keys_R = zip(*[_keys(200 + k, r, n, miss=0.1) for k, r in enumerate(rows_k)])
    codes = [g.integers(0, c, size=r).astype(np.int32) if c > 1 else None for r, c in zip(rows_k, card)]
    masks = [None, None, (g.random(30) < 0.5).astype(np.uint8)]
    meas = g.integers(1, 1000, size=n).astype(np.int32)
    fks_w = [MJ.key_to_row(kr, ks)[0] for kr, ks in zip(keys_R, keys_S)]
    want_s, want_c = O.groupby_sum(fks_w, list(rows_k), masks, codes, list(card), None, [meas])
    fks = [lq.lq_keymap_lookup(lq.lq_keymap_build(torch.from_numpy(ks).cuda()), torch.from_numpy(kr).cuda())
           for kr, ks in zip(keys_R, keys_S)]
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    s, c = lq.lq_masked_groupby_sum(fks, list(rows_k), [dev(m) for m in masks], [dev(x) for x in codes],
                                    list(card), None, [dev(meas)])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(s.cpu().numpy(), want_s)
    np.testing.assert_array_equal(c.cpu().numpy(), want_c)


def _is_direct(table):
    return int(table[12:16].view(torch.int32).item()) == 1


def _dense_keys(seed, r, n, base, fill=0.7, miss=0.05):
    """r distinct keys out of a window of r / fill consecutive integers starting at `base`, shuffled."""
    g = np.random.default_rng(seed)
    window = np.arange(int(r / fill) + 1, dtype=np.int64) + base
    g.shuffle(window)
    key_S = window[:r].astype(np.int32)
    key_R = g.choice(window, size=n).astype(np.int32)              # some hit the gaps: no match
    m = g.random(n) < miss
    key_R[m] = (base - 1 - g.integers(0, 1000, size=int(m.sum()))).astype(np.int32)   # and some lie outside the window
    return key_S, key_R


@pytest.mark.parametrize("r,n,base", [(1, 10, 5), (2_556, 1_300_001, 19920101), (2_000, 100_003, 1), (30_000, 1_200_000, 1),
                                      (200_000, 1_000_003, -150_000), (8_192, 1_048_576, -2**31 + 1000)])
def test_dense_key_ranges_use_the_direct_form(lq, r, n, base):
    key_S, key_R = _dense_keys(r + n, r, n, base)
    fk_w, rows_w, cols_w = MJ.key_to_row(key_R, key_S)
    table = lq.lq_keymap_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
    assert _is_direct(table)
    fk = lq.lq_keymap_lookup(table, torch.from_numpy(key_R).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(fk.cpu().numpy(), fk_w)
    # unaligned key columns take the one-key-per-thread path
    kr = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    kr[1:] = torch.from_numpy(key_R)
    np.testing.assert_array_equal(lq.lq_keymap_lookup(table, kr[1:]).cpu().numpy(), fk_w)


def test_sparse_key_ranges_use_the_hashed_form(lq):
    key_S, key_R = _keys(17, 5_000, 1_100_000)
    table = lq.lq_keymap_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
    assert not _is_direct(table)
    fk_w, _, _ = MJ.key_to_row(key_R, key_S)
    np.testing.assert_array_equal(lq.lq_keymap_lookup(table, torch.from_numpy(key_R).cuda()).cpu().numpy(), fk_w)


def test_direct_form_duplicates_and_inserts(lq):
    keys = torch.tensor([5, 9, 5, 3], dtype=torch.int32, device="cuda")
    with pytest.raises(lq.LQError) as e:
        lq.lq_keymap_build(keys, flags=lq.LQ_CHECK_KEYS)
    assert e.value.status == "LQ_ERR_DUPLICATE_KEY"
    # surrogate keys 1..r, new dimension rows appended with the next keys: inside the window
    key_S = np.arange(1, 40_001, dtype=np.int32)
    g = np.random.default_rng(3)
    key_R = g.integers(-5, 40_020, size=500_000).astype(np.int32)
    part = lq.lq_keymap_build(torch.from_numpy(key_S[:25_000]).cuda(), max_keys=40_000)
    assert _is_direct(part)
    lq.lq_keymap_insert(part, torch.from_numpy(key_S[25_000:]).cuda(), 25_000, flags=lq.LQ_CHECK_KEYS)
    fk_w, _, _ = MJ.key_to_row(key_R, key_S)
    np.testing.assert_array_equal(lq.lq_keymap_lookup(part, torch.from_numpy(key_R).cuda()).cpu().numpy(), fk_w)
    # a key far outside the window cannot be added to a direct map: reported, the map stays usable
    with pytest.raises(lq.LQError) as e:
        lq.lq_keymap_insert(part, torch.tensor([2_000_000_000], dtype=torch.int32, device="cuda"), 40_000,
                            flags=lq.LQ_CHECK_KEYS)
    assert e.value.status == "LQ_ERR_WORKSPACE"
    np.testing.assert_array_equal(lq.lq_keymap_lookup(part, torch.from_numpy(key_R).cuda()).cpu().numpy(), fk_w)


# ---------------------------------------------------------------- 64-bit keys

def _keys64(seed, r, n, dense, miss=0.1):
    g = np.random.default_rng(seed)
    if dense:
        base = int(g.choice([-2**62, -7, 0, 10**15, 2**63 - 1 - 3 * r]))
        pool = base + g.permutation(int(r * 1.4) + 1).astype(np.int64)
    else:
        pool = np.unique(g.integers(-2**63 + 1, 2**63 - 1, size=int(r * 1.4) + 8, dtype=np.int64))
        g.shuffle(pool)
    key_S = pool[:r].copy()
    extra = pool[r:]
    key_R = g.choice(key_S, size=n)
    if len(extra) and n:
        m = g.random(n) < miss
        key_R[m] = g.choice(extra, size=int(m.sum()))
    return key_S, key_R


@pytest.mark.parametrize("dense", [True, False])
@pytest.mark.parametrize("r,n", [(1, 3), (9, 1_001), (2_556, 100_003), (30_000, 400_000), (200_000, 1_000_001)])
def test_int64_keys_match_algorithm_1(lq, r, n, dense):
    key_S, key_R = _keys64(r + n + dense, r, n, dense)
    fk_w, rows_w, cols_w = MJ.key_to_row(key_R, key_S)
    table = lq.lq_keymap64_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
    assert _is_direct(table) == (dense and r > 1 or (r == 1))
    fk = lq.lq_keymap64_lookup(table, torch.from_numpy(key_R).cuda())
    rows, cols, nnz = lq.lq_compact_matches(fk)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(fk.cpu().numpy(), fk_w)
    m = int(nnz.item())
    assert m == len(rows_w)
    np.testing.assert_array_equal(rows[:m].cpu().numpy(), rows_w)
    np.testing.assert_array_equal(cols[:m].cpu().numpy(), cols_w)
    # unaligned key column: one key per thread
    kr = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    kr[1:] = torch.from_numpy(key_R)
    np.testing.assert_array_equal(lq.lq_keymap64_lookup(table, kr[1:]).cpu().numpy(), fk_w)


def test_int64_extremes_duplicates_inserts_and_the_reserved_key(lq):
    key_S = np.array([2**63 - 1, -2**63 + 1, 0, -1, 1, 2**40], dtype=np.int64)
    key_R = np.array([0, -1, 2**63 - 1, -2**63 + 1, 5, 1, 2**40, -2**63], dtype=np.int64)
    table = lq.lq_keymap64_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
    assert lq.lq_keymap64_lookup(table, torch.from_numpy(key_R).cuda()).cpu().tolist() == [2, 3, 0, 1, -1, 4, 5, -1]
    with pytest.raises(lq.LQError) as e:
        lq.lq_keymap64_build(torch.tensor([5, 9, 5, 2**50], dtype=torch.int64, device="cuda"), flags=lq.LQ_CHECK_KEYS)
    assert e.value.status == "LQ_ERR_DUPLICATE_KEY"
    with pytest.raises(lq.LQError) as e:
        lq.lq_keymap64_build(torch.tensor([-2**63, 2**62], dtype=torch.int64, device="cuda"), flags=lq.LQ_CHECK_KEYS)
    assert e.value.status == "LQ_ERR_UNSUPPORTED"
    # incremental update of a hashed and of a direct map
    for dense in (False, True):
        ks, kr = _keys64(77 + dense, 40_000, 300_000, dense, miss=0.2)
        part = lq.lq_keymap64_build(torch.from_numpy(ks[:25_000]).cuda(), max_keys=40_000)
        try:
            lq.lq_keymap64_insert(part, torch.from_numpy(ks[25_000:]).cuda(), 25_000, flags=lq.LQ_CHECK_KEYS)
        except lq.LQError as err:                       # a direct map may have to be rebuilt for keys outside its window
            assert dense and err.status == "LQ_ERR_WORKSPACE"
            part = lq.lq_keymap64_build(torch.from_numpy(ks).cuda(), flags=lq.LQ_CHECK_KEYS)
        fk_w, _, _ = MJ.key_to_row(kr, ks)
        np.testing.assert_array_equal(lq.lq_keymap64_lookup(part, torch.from_numpy(kr).cuda()).cpu().numpy(), fk_w)
