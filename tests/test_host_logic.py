"""CPU-only checks: the C-ABI library loads, exports every declared symbol, and its host-side
validation rejects bad arguments before anything is enqueued (no GPU needed: every call here
fails validation, so no kernel is launched and no device pointer is dereferenced)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lq.h")
LIB = os.path.join(ROOT, "paper_2306_08367_amd", "liblq.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="liblq.so not built")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    names = declared_functions()
    assert {"lq_project_dims", "lq_fused_join_predict", "lq_materialized_join_predict",
            "lq_masked_groupby_sum", "lq_workspace_bytes", "lq_groupby_workspace_bytes",
            "lq_stream_copy", "lq_last_error", "lq_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in lq.h but not exported"


def _binding():
    from paper_2306_08367_amd import binding
    return binding


def test_struct_layout_matches_the_header():
    b = _binding()
    # void* (8) + int64 (8) + int32 (4) + pad (4) + int64 (8) + int32 (4) + pad (4)
    assert ctypes.sizeof(b.lq_mat) == 40
    assert b.lq_mat.ld.offset == 24 and b.lq_mat.dtype.offset == 32
    assert b.lq_star.fact.offset == 8 and b.lq_star.n_dims.offset == 48
    assert b.lq_star.dims.offset == 56 and b.lq_star.fks.offset == 64
    assert b.lq_model.W.offset == 8 and b.lq_model.bias.offset == 16


FAKE = 0x10000   # non-NULL, aligned; never dereferenced because validation fails first


def _star_model(b, n=10, c_f=2, dims=((5, 3),), l=(4,), dtype=0, w_rows=None):
    K = len(dims)
    dims_arr = (b.lq_mat * max(1, K))()
    for k, (r, c) in enumerate(dims):
        dims_arr[k] = b.lq_mat(FAKE, r, c, c, dtype)
    fks = (ctypes.c_void_p * max(1, K))(*([FAKE] * K))
    star = b.lq_star(n, b.lq_mat(FAKE, n, c_f, max(c_f, 1), dtype), K, dims_arr, fks)
    kw = c_f + sum(c for _, c in dims)
    W = (b.lq_mat * len(l))()
    rows = kw if w_rows is None else w_rows
    for j, lo in enumerate(l):
        W[j] = b.lq_mat(FAKE, rows, lo, lo, dtype)
        rows = lo
    bias = (ctypes.c_void_p * len(l))()
    model = b.lq_model(len(l), W, bias)
    return star, model, (dims_arr, fks, W, bias)


def test_project_dims_rejects_bad_arguments():
    b = _binding()
    lib = b._lib
    star, model, keep = _star_model(b, w_rows=4)            # joined width is 5
    P = (b.lq_mat * 1)(b.lq_mat(FAKE, 5, 4, 4, 0))
    assert lib.lq_project_dims(ctypes.byref(star), ctypes.byref(model), P, None) == 2
    assert "joined width" in b.lq_last_error()
    star, model, keep = _star_model(b)
    P = (b.lq_mat * 1)(b.lq_mat(FAKE, 6, 4, 4, 0))           # wrong row count
    assert lib.lq_project_dims(ctypes.byref(star), ctypes.byref(model), P, None) == 2
    P = (b.lq_mat * 1)(b.lq_mat(FAKE, 5, 4, 4, 1))           # bf16 P for an f32 model
    assert lib.lq_project_dims(ctypes.byref(star), ctypes.byref(model), P, None) == 3
    assert lib.lq_project_dims(None, ctypes.byref(model), P, None) == 1
    P = (b.lq_mat * 1)(b.lq_mat(None, 5, 4, 4, 0))
    assert lib.lq_project_dims(ctypes.byref(star), ctypes.byref(model), P, None) == 1
    star, model, keep = _star_model(b, l=(4, 3, 2))
    keep[2][2].rows = 5                                       # layer widths do not chain
    assert lib.lq_project_dims(ctypes.byref(star), ctypes.byref(model), P, None) == 2


def test_fused_rejects_bad_arguments():
    b = _binding()
    lib = b._lib
    star, model, keep = _star_model(b)
    P = (b.lq_mat * 1)(b.lq_mat(FAKE, 5, 4, 4, 0))
    Y = b.lq_mat(FAKE, 10, 3, 3, 0)                           # l_out is 4
    args = (ctypes.byref(star), ctypes.byref(model), P, ctypes.byref(Y), None, 0, 0, None)
    assert lib.lq_fused_join_predict(*args) == 2
    Y = b.lq_mat(FAKE, 10, 4, 4, 1)                           # bf16 Y for an f32 model
    args = (ctypes.byref(star), ctypes.byref(model), P, ctypes.byref(Y), None, 0, 0, None)
    assert lib.lq_fused_join_predict(*args) == 3
    Y = b.lq_mat(FAKE, 10, 4, 2, 0)                           # ld < cols
    args = (ctypes.byref(star), ctypes.byref(model), P, ctypes.byref(Y), None, 0, 0, None)
    assert lib.lq_fused_join_predict(*args) == 2
    Y = b.lq_mat(FAKE, 10, 4, 4, 0)
    args = (ctypes.byref(star), ctypes.byref(model), P, ctypes.byref(Y), None, 0, b.LQ_CHECK_FKS, None)
    assert lib.lq_fused_join_predict(*args) == 4              # key check needs a workspace
    star.n_dims = 9
    args = (ctypes.byref(star), ctypes.byref(model), P, ctypes.byref(Y), None, 0, 0, None)
    assert lib.lq_fused_join_predict(*args) == 2
    assert b.lq_last_error() != ""


def test_materialized_rejects_small_or_missing_workspace():
    b = _binding()
    lib = b._lib
    star, model, keep = _star_model(b)
    Y = b.lq_mat(FAKE, 10, 4, 4, 0)
    assert lib.lq_materialized_join_predict(ctypes.byref(star), ctypes.byref(model), ctypes.byref(Y),
                                            None, 0, 0, None) == 4
    assert lib.lq_materialized_join_predict(ctypes.byref(star), ctypes.byref(model), ctypes.byref(Y),
                                            0x10000, 1024, 0, None) == 4
    need = lib.lq_workspace_bytes(b.LQ_CALL_MATERIALIZED, ctypes.byref(star), ctypes.byref(model), 256)
    assert need >= 256 * 5 * 4
    assert lib.lq_workspace_bytes(99, ctypes.byref(star), ctypes.byref(model), 256) == 0


def test_groupby_rejects_bad_arguments():
    b = _binding()
    lib = b._lib
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    fks = (vp * 2)(FAKE, FAKE)
    rows = (i64 * 2)(10, 20)
    codes = (vp * 2)(FAKE, FAKE)
    meas = (vp * 1)(FAKE)

    def call(card, n_meas=1, ws=FAKE, ws_bytes=1 << 20, sums=FAKE, K=2):
        return lib.lq_masked_groupby_sum(100, K, fks, rows, None, codes, (i32 * 2)(*card), None,
                                         n_meas, meas, sums, None, ws, ws_bytes, 0, None)
    assert call((65_535, 65_535)) == 6                        # more than 2^30 groups
    assert b.lq_groupby_workspace_bytes([10, 20], [65_535, 65_535], 1) == 0
    # above 8,192 accumulators the outputs themselves accumulate: the workspace only holds the side tables
    assert 0 < b.lq_groupby_workspace_bytes([10, 20], [100, 100], 1) < b.lq_groupby_workspace_bytes([10, 20], [60, 60], 1)
    assert call((0, 5)) == 2
    assert call((5, 5), n_meas=0) == 2
    assert call((5, 5), n_meas=5) == 2
    assert call((5, 5), ws=None) == 4
    assert call((5, 5), ws_bytes=16) == 4
    assert call((5, 5), sums=None) == 1
    assert call((5, 5), K=9) == 2
    assert b.lq_groupby_workspace_bytes([10, 20], [5, 5], 1) >= 60


def test_stream_copy_rejects_misaligned():
    b = _binding()
    assert b._lib.lq_stream_copy(0x10008, 0x20000, 64, None) == 2
    assert b._lib.lq_stream_copy(0x10000, 0x20000, 60, None) == 2
    assert b._lib.lq_stream_copy(None, 0x20000, 64, None) == 1
    assert b._lib.lq_stream_copy(None, None, 0, None) == 0


def test_tree_entry_points_reject_bad_arguments():
    b = _binding()
    lib = b._lib
    assert b.lq_tree_table_ld(64) == 64 and b.lq_tree_table_ld(65) == 80 and b.lq_tree_table_ld(0) == 0
    star, model, keep = _star_model(b)
    tree = b.lq_tree(3, 4, FAKE, FAKE, FAKE)
    tables = (ctypes.c_void_p * 1)(FAKE)
    assert lib.lq_tree_project_dims(ctypes.byref(star), ctypes.byref(tree), tables, None, None) == 1
    bad = b.lq_tree(0, 4, FAKE, FAKE, FAKE)
    assert lib.lq_tree_project_dims(ctypes.byref(star), ctypes.byref(bad), tables, FAKE, None) == 2
    bad = b.lq_tree(3, 4, None, FAKE, FAKE)
    assert lib.lq_tree_project_dims(ctypes.byref(star), ctypes.byref(bad), tables, FAKE, None) == 1
    keep[0][0].dtype = 1                                      # bf16 dimension table
    assert lib.lq_tree_project_dims(ctypes.byref(star), ctypes.byref(tree), tables, FAKE, None) == 3
    keep[0][0].dtype = 0
    # fused: neither output requested; misaligned target
    assert lib.lq_fused_join_tree(ctypes.byref(star), ctypes.byref(tree), tables, FAKE, None, None, 0,
                                  None, 0, None) == 1
    assert lib.lq_fused_join_tree(ctypes.byref(star), ctypes.byref(tree), tables, FAKE + 8, FAKE, None, 0,
                                  None, 0, None) == 1
    # materialised: workspace too small
    assert lib.lq_materialized_join_tree(ctypes.byref(star), ctypes.byref(tree), FAKE, None, FAKE, 1024, 0,
                                         None) == 4
    assert lib.lq_tree_workspace_bytes(ctypes.byref(star), ctypes.byref(tree), 256) >= 256 * 5 * 4
    # leaf masks: word count; size of the fact-side buffer (header 16 B, column + threshold per node,
    # rounded to 16, then two words per node and mask word, then the per-leaf lists: l + 1 offsets rounded
    # to 16 and room for 64 entries of 16 bytes per leaf); missing or misaligned arguments
    assert b.lq_tree_mask_words(1) == 1 and b.lq_tree_mask_words(64) == 1 and b.lq_tree_mask_words(65) == 2
    assert b.lq_tree_mask_words(0) == 0
    assert b.lq_tree_fact_mask_bytes(3, 4) == 48 + 3 * 16 + 32 + 4 * 1024
    assert b.lq_tree_fact_mask_bytes(63, 65) == 528 + 63 * 32 + 272 + 65 * 1024
    assert b.lq_tree_fact_mask_bytes(0, 4) == 0
    assert lib.lq_tree_fact_masks(-1, ctypes.byref(tree), FAKE, None) == 2
    assert lib.lq_tree_fact_masks(2, ctypes.byref(tree), None, None) == 1
    assert lib.lq_tree_fact_masks(2, ctypes.byref(tree), FAKE + 8, None) == 1
    masks = (ctypes.c_void_p * 1)(FAKE)
    # incremental refresh: dimension and row range are checked against the star (dims[0] has 5 rows)
    refresh = lambda dim, first, count, tb=tables, mk=masks: lib.lq_tree_project_dim_rows(
        ctypes.byref(star), ctypes.byref(tree), tb, mk, dim, first, count, None)
    assert refresh(-1, 0, 1) == 2 and refresh(1, 0, 1) == 2
    assert refresh(0, 3, 3) == 2 and refresh(0, -1, 2) == 2 and refresh(0, 6, 0) == 2
    assert refresh(0, 5, 0) == 0                              # an empty range at the end: nothing to do
    assert refresh(0, 0, 1, tb=(ctypes.c_void_p * 1)(FAKE + 8)) == 1
    assert refresh(0, 0, 1, mk=(ctypes.c_void_p * 1)(FAKE + 4)) == 1
    # a fact table with columns of its own needs the fact-side buffer
    assert lib.lq_fused_join_tree_masks(ctypes.byref(star), ctypes.byref(tree), masks, None, FAKE, None, 0, None) == 1
    assert lib.lq_fused_join_tree_masks(ctypes.byref(star), ctypes.byref(tree), masks, FAKE + 8, FAKE, None, 0, None) == 1
    star0, _, keep0 = _star_model(b, c_f=0)
    assert lib.lq_tree_compress_tables(ctypes.byref(star0), ctypes.byref(tree), tables, None, None) == 1
    assert lib.lq_fused_join_tree_masks(ctypes.byref(star0), ctypes.byref(tree), masks, None, None, None, 0, None) == 1
    odd = (ctypes.c_void_p * 1)(FAKE + 4)
    assert lib.lq_fused_join_tree_masks(ctypes.byref(star0), ctypes.byref(tree), odd, None, FAKE, None, 0, None) == 1


def test_keymap_entry_points_reject_bad_arguments():
    b = _binding()
    lib = b._lib
    assert b.lq_keymap_bytes(0) == 256 + 16 and b.lq_keymap_bytes(1000) == 256 + 2048 * 8
    assert b.lq_keymap_bytes(-1) == 0
    nbytes = b.lq_keymap_bytes(1000)
    assert lib.lq_keymap_build(None, nbytes, FAKE, 10, 0, None) == 4
    assert lib.lq_keymap_build(FAKE, nbytes, FAKE, 2000, 0, None) == 4      # sized for 1000 keys
    assert lib.lq_keymap_build(FAKE + 8, nbytes, FAKE, 10, 0, None) == 4    # misaligned buffer
    assert lib.lq_keymap_insert(FAKE, nbytes, None, 10, 0, 0, None) == 1
    assert lib.lq_keymap_insert(FAKE, nbytes, FAKE, 10, 2**31, 0, None) == 2
    assert lib.lq_keymap_lookup(FAKE, nbytes, None, 10, FAKE, None) == 1
    assert lib.lq_keymap_lookup(FAKE, 8, FAKE, 10, FAKE, None) == 4
    assert lib.lq_compact_matches(FAKE, 10, FAKE, FAKE, None, FAKE, 4096, None) == 1
    assert lib.lq_compact_matches(FAKE, 10, FAKE, FAKE, FAKE, FAKE, 8, None) == 4
    assert lib.lq_compact_workspace_bytes(10) >= 16


def test_fusion_advice_is_the_complexity_model_of_the_paper():
    """Equal column counts and three dimensions: the ratio must be Eq. 3, k/l + k^2/(3 i l) + k/sum r."""
    b = _binding()
    i, c, l = 600_000 * 4, 16, 8
    rows = (80_000, 8_000, 2_555)
    k = 3 * c
    adv = b.lq_fusion_advice(i, 0, [(r, c) for r in rows], [l], queries_per_update=1.0)
    eq3 = k / l + k * k / (3 * i * l) + k / sum(rows)
    assert abs(adv["ratio"] - eq3) <= 1e-12 * eq3
    assert adv["ratio_leading_term"] == k / l
    assert adv["cost_fusion"] == i * l * sum(rows)
    assert adv["cost_prefusion"] == sum(rows) * c * l
    assert adv["memory_growth"] == l / c and adv["fuse"] == 1
    # an output wider than the joined table: fusing loses and the pre-fused tables grow (Q6)
    wide = b.lq_fusion_advice(3_000, 0, [(2_000, 8)] * 3, [4096], queries_per_update=1.0)
    assert wide["memory_growth"] == 512 and wide["ratio"] < 1 and wide["fuse"] == 0
    # the trend the paper reports: the ratio grows with k and shrinks with l
    r1 = b.lq_fusion_advice(i, 0, [(r, 32) for r in rows], [8])["ratio"]
    r2 = b.lq_fusion_advice(i, 0, [(r, 32) for r in rows], [64])["ratio"]
    assert r1 > adv["ratio"] > r2 * 0 and r1 > r2

def test_fusion_decision_follows_what_the_kernels_move_not_the_dense_model():
    """The paper's dense cost ratio falls below 1 as soon as l > k; with one key per fact row the fused
    join stage of this library is still ahead there (its gathers come out of the caches, the non-fused
    pipeline writes and re-reads T), so the flag must not be the sign of (ratio - 1)."""
    b = _binding()
    rows = (60_000, 8_000, 2_555)
    for cols, l in (((8, 4, 4), 32), ((8, 4, 4), 64), ((12, 12, 8), 64)):
        adv = b.lq_fusion_advice(2_400_000, 0, list(zip(rows, cols)), [l], queries_per_update=1.0)
        assert adv["ratio"] < 1 and adv["fuse"] == 1, (cols, l, adv)
        assert adv["seconds_no_fusion"] > adv["seconds_fused"] > 0 and adv["seconds_prefusion"] > 0
        # the decision is exactly the stated inequality, for any update frequency
        for q in (1e-3, 0.5, 1.0, 100.0):
            a = b.lq_fusion_advice(2_400_000, 0, list(zip(rows, cols)), [l], queries_per_update=q)
            assert a["fuse"] == int(q * (a["seconds_no_fusion"] - a["seconds_fused"]) > a["seconds_prefusion"])
        # dimension tables that change before a single query has run never pay for their pre-fusion
        assert b.lq_fusion_advice(2_400_000, 0, list(zip(rows, cols)), [l], queries_per_update=1e-3)["fuse"] == 0
    # more fact rows only scale the per-query terms; more dimension rows only the pre-fusion
    a1 = b.lq_fusion_advice(1_000_000, 4, [(10_000, 32)] * 3, [64, 1])
    a2 = b.lq_fusion_advice(2_000_000, 4, [(10_000, 32)] * 3, [64, 1])
    assert a2["seconds_prefusion"] == a1["seconds_prefusion"] and a2["seconds_fused"] > 1.9 * a1["seconds_fused"] - 1e-5
    a3 = b.lq_fusion_advice(1_000_000, 4, [(20_000, 32)] * 3, [64, 1])
    assert a3["seconds_prefusion"] > a1["seconds_prefusion"] and a3["seconds_fused"] == a1["seconds_fused"]


def test_groupby_agg_rejects_bad_arguments():
    b = _binding()
    lib = b._lib
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    fks = (vp * 1)(FAKE)
    rows = (i64 * 1)(10)
    card = (i32 * 1)(5)
    codes = (vp * 1)(FAKE)
    preds = (b.lq_range_pred * 1)(b.lq_range_pred(FAKE, 0, 3))
    meas = (b.lq_measure * 1)(b.lq_measure(1, FAKE, None))            # product without a second column

    def call(n_preds=1, n_meas=1, m=meas, sums=FAKE, ws=FAKE, ws_bytes=1 << 22):
        return lib.lq_groupby_agg(100, 1, fks, rows, None, codes, card, n_preds, preds, n_meas, m, sums, None, None,
                                  None, ws, ws_bytes, 0, None)
    assert call() == 1
    ok = (b.lq_measure * 1)(b.lq_measure(7, FAKE, FAKE))
    assert call(m=ok) == 2                                            # unknown op
    ok = (b.lq_measure * 1)(b.lq_measure(0, FAKE, None))
    assert call(m=ok, n_preds=5) == 2
    assert call(m=ok, n_meas=0) == 2
    assert call(m=ok, sums=None) == 1                                 # no output requested
    assert call(m=ok, ws=None) == 4
    assert call(m=ok, ws_bytes=64) == 4
    assert lib.lq_groupby_agg_workspace_bytes(1, rows, card, 1) > 0


def test_group_domain_and_order_groups_reject_bad_arguments():
    b = _binding()
    lib = b._lib
    vp = ctypes.c_void_p
    cols = (vp * 4)(FAKE, FAKE, FAKE, FAKE)
    card = ctypes.c_int32(-1)
    need = lib.lq_group_domain_workspace_bytes(1000)
    assert need >= 256 + 2 * 2048 * 4 + 65536 * 4 and lib.lq_group_domain_workspace_bytes(-1) == 0
    args = lambda **kw: dict(dict(rows=1000, n_cols=1, cols=cols, max_card=100, code=FAKE, values=FAKE,
                                  card=ctypes.byref(card), ws=FAKE, ws_bytes=need), **kw)
    call = lambda a: lib.lq_group_domain(a["rows"], a["n_cols"], a["cols"], a["max_card"], a["code"], a["values"],
                                         a["card"], a["ws"], a["ws_bytes"], None)
    assert call(args(n_cols=0)) == 2 and call(args(n_cols=5)) == 2
    assert call(args(max_card=0)) == 2 and call(args(max_card=65536)) == 2
    assert call(args(rows=-1)) == 2
    assert call(args(cols=None)) == 1 and call(args(card=None)) == 1 and call(args(code=None)) == 1
    assert call(args(ws=None)) == 4 and call(args(ws_bytes=need - 1)) == 4 and call(args(ws=FAKE + 8)) == 4
    assert call(args(rows=0, code=None, values=None, ws_bytes=lib.lq_group_domain_workspace_bytes(0))) == 0
    assert card.value == 0                                        # an empty table has no groups; nothing is launched

    gc = (ctypes.c_int32 * 2)(7, 25)
    keys = (b.lq_sort_key * 2)(b.lq_sort_key(b.LQ_KEY_GROUP_COLUMN, 0, 0), b.lq_sort_key(b.LQ_KEY_SUM, 0, 1))
    order = lambda **kw: lib.lq_order_groups(*[dict(dict(n=2, gc=gc, m=1, sums=FAKE, counts=FAKE, nk=2, keys=keys,
                                                           order=FAKE, n_out=FAKE), **kw)[x]
                                               for x in ("n", "gc", "m", "sums", "counts", "nk", "keys", "order", "n_out")], None)
    assert order(n=9) == 2 and order(nk=5) == 2 and order(m=5) == 2
    assert order(counts=None) == 1 and order(order=None) == 1 and order(n_out=None) == 1 and order(keys=None) == 1
    assert order(sums=None) == 2                                   # a key asks for a sum that is not given
    assert order(m=0) == 2                                         # ... or for a measure that does not exist
    assert order(gc=(ctypes.c_int32 * 2)(8192, 2)) == 6            # more than 8,192 groups
    assert order(gc=(ctypes.c_int32 * 2)(0, 2)) == 2
    bad = (b.lq_sort_key * 2)(b.lq_sort_key(b.LQ_KEY_GROUP_COLUMN, 2, 0), b.lq_sort_key(9, 0, 0))
    assert order(keys=bad) == 2
    assert order(counts=FAKE + 4) == 2


def test_keymap64_entry_points_reject_bad_arguments():
    b = _binding()
    lib = b._lib
    assert b.lq_keymap64_bytes(0) == 256 + 2 * 12 and b.lq_keymap64_bytes(1000) == 256 + 2048 * 12
    assert b.lq_keymap64_bytes(-1) == 0
    nbytes = b.lq_keymap64_bytes(1000)
    assert lib.lq_keymap64_build(None, nbytes, FAKE, 10, 0, None) == 4
    assert lib.lq_keymap64_build(FAKE, nbytes, FAKE, 2000, 0, None) == 4       # sized for 1000 keys
    assert lib.lq_keymap64_build(FAKE, nbytes, FAKE + 4, 10, 0, None) == 1     # keys not 8-byte aligned
    assert lib.lq_keymap64_insert(FAKE, nbytes, None, 10, 0, 0, None) == 1
    assert lib.lq_keymap64_insert(FAKE, nbytes, FAKE, 10, 2**31, 0, None) == 2
    assert lib.lq_keymap64_lookup(FAKE, nbytes, None, 10, FAKE, None) == 1
    assert lib.lq_keymap64_lookup(FAKE, 8, FAKE, 10, FAKE, None) == 4


def test_bucket_workspace_sizes_follow_the_rows_and_the_groups():
    """lq_groupby_bucket_workspace_bytes: 0 where the bucketed form does not apply, otherwise the small workspace plus
    two slots of 4 (1 + measures) bytes per fact row (plus 1,024 slots per bucket and the counters)."""
    b = _binding()
    rows, card = [300, 280], [250, 240]                       # 60,000 groups
    small = b.lq_groupby_workspace_bytes(rows, card, 1)
    for n in (1, 1_000, 2_000_003):
        big = b.lq_groupby_bucket_workspace_bytes(n, rows, card, 1)
        assert big > small + 2 * 8 * n
        assert big < small + 2 * 8 * n + 8_192 * (4 + 1_026 * 8) + 4_096
    assert b.lq_groupby_bucket_workspace_bytes(1_000, rows, card, 2) > b.lq_groupby_bucket_workspace_bytes(1_000, rows, card, 1)
    assert b.lq_groupby_bucket_workspace_bytes(1_000, rows, [30, 28], 1) == 0        # 840 groups: LDS accumulators
    # three or four measures run as two calls of two measures: the size of those
    assert b.lq_groupby_bucket_workspace_bytes(1_000, rows, card, 3) == b.lq_groupby_bucket_workspace_bytes(1_000, rows, card, 2)
    assert b.lq_groupby_bucket_workspace_bytes(1_000, rows, [60, 40], 4) == 0        # 2,400 groups: two measures fit LDS
    assert b.lq_groupby_bucket_workspace_bytes(0, rows, card, 1) == 0
    assert b.lq_groupby_bucket_workspace_bytes(1 << 31, rows, card, 1) == 0
    assert b.lq_groupby_bucket_workspace_bytes(1_000, [70_000, 70_000], [65_535, 16_000], 1) == 0   # more than 8,192 buckets


def test_fused_workspace_grows_with_the_chunk_only_for_models_of_two_or_more_layers():
    import torch
    b = _binding()
    W1 = [torch.zeros((40, 1_000)), torch.zeros((1_000, 300)), torch.zeros((300, 2))]
    assert b.lq_workspace_bytes(b.LQ_CALL_FUSED, 40, W1[:1], 4_096) == 256
    assert b.lq_workspace_bytes(b.LQ_CALL_FUSED, 40, W1, 0) == 256
    # two activation buffers as wide as the widest hidden layer (1,000 floats), rows rounded up to 256
    assert b.lq_workspace_bytes(b.LQ_CALL_FUSED, 40, W1, 4_000) == 256 + 2 * 4_096 * 4_000
    Wb = [w.to(torch.bfloat16) for w in W1]
    assert b.lq_workspace_bytes(b.LQ_CALL_FUSED, 40, Wb, 256) == 256 + 2 * 256 * 2_000


def test_tree_mask_rows_have_an_even_number_of_words_from_three_on():
    b = _binding()
    got = [b.lq_tree_mask_words(l) for l in (0, 1, 64, 65, 128, 129, 192, 193, 256, 257, 1_024, 1_025)]
    assert got == [0, 1, 1, 2, 2, 4, 4, 4, 4, 6, 16, 18]
