"""GPU parity of the decision-tree fusion (Section 3.3, Eq. 2) against the oracle: bit-exact
(every decision is a comparison of an fp32 table value with an fp32 threshold, and the rest is
integer arithmetic)."""
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


def _case(name, n, c_f, rows, cols, leaves, seed, tree_cols=None):
    w = WL.make_predict(name, n, c_f, rows, cols, (1,), seed=seed)
    kw = c_f + sum(cols)
    tree = WL.make_tree(kw, leaves, seed + 1, cols=tree_cols)
    return w, tree


def _run(lq, w, tree, onehot=True):
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, w.c_f, f, t, H)
    leaf, oh = lq.lq_fused_join_tree(w.X, w.fks, tables, target, f, t, H, want_onehot=onehot)
    leaf_m, oh_m = lq.lq_materialized_join_tree(w.X, w.dims, w.fks, f, t, H, want_onehot=onehot, chunk_rows=1024)
    torch.cuda.synchronize()
    return tables, target, leaf, oh, leaf_m, oh_m


CASES = [
    # name, n, c_f, dim_rows, dim_cols, leaves
    ("two_leaves", 1_000, 0, (10, 7), (3, 2), 2),
    ("five_leaves", 5_003, 0, (50, 70, 30), (4, 4, 4), 5),
    ("sixteen", 4_099, 0, (100, 200), (8, 8), 16),
    ("setting1_like", 20_011, 0, (800, 160, 255), (43, 43, 42), 64),
    ("hundred_leaves", 3_333, 0, (64, 64, 64, 64), (5, 5, 5, 5), 100),
    ("wide_256", 2_049, 0, (300, 200), (16, 16), 256),
    ("very_wide_1500", 1_025, 0, (120, 90), (32, 32), 1_500),
    ("wide_384_six_mask_words", 1_531, 0, (200, 100), (16, 16), 384),
    ("wide_1024_three_tables", 1_101, 0, (150, 90, 60), (20, 20, 20), 1_024),
    ("wide_2048_one_table", 515, 0, (333,), (40,), 2_048),
    ("wide_600_three_tables", 777, 0, (1_000, 37, 300), (20, 30, 10), 600),
    ("wide_4096_two_tables", 301, 0, (50, 40), (12, 12), 4_096),
    ("wide_2704_five_tables", 259, 0, (20, 30, 10, 25, 9), (5, 5, 5, 5, 5), 2_704),
    ("fact_columns", 2_500, 3, (40, 60), (4, 4), 24),
    ("fact_columns_4_aligned", 5_111, 4, (40, 60, 25), (4, 4, 3), 64),
    ("fact_columns_8_wide_tree", 3_001, 8, (90, 60), (6, 6), 200),
    ("fact_columns_12", 2_777, 12, (50,), (8,), 48),
    ("fact_columns_5_very_wide_tree", 1_333, 5, (70, 30), (10, 10), 700),
    ("fact_columns_9_two_mask_words", 2_311, 9, (70, 30), (5, 5), 100),
    ("fact_columns_20_mostly_fact_nodes", 3_100, 20, (40,), (3,), 40),
    ("fact_columns_only", 4_321, 6, (), (), 40),
    ("fact_columns_4_wide_1024", 1_203, 4, (150, 90), (20, 20), 1_024),
    ("fact_columns_12_wide_384", 1_777, 12, (64, 32, 16), (5, 5, 5), 384),
    ("fact_columns_only_wide_256", 2_049, 7, (), (), 256),
    ("fact_columns_only_1100_leaves", 1_501, 3, (), (), 1_100),      # more fact-side nodes than the byte-table join lists
    ("one_row", 1, 0, (5,), (3,), 4),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_tree_paths_match_oracle(lq, case):
    name, n, c_f, rows, cols, leaves = case
    w, tree = _case(name, n, c_f, rows, cols, leaves, WL.SEED0 + 500 + leaves)
    R, onehot, leaf = O.tree_predict(w.X, w.dims, w.fks, tree.feature, tree.threshold, tree.H)
    Tk = O.tree_project(w.dims, c_f, tree.feature, tree.threshold, tree.H)
    w = to_dev(w)
    tables, target, g_leaf, g_oh, m_leaf, m_oh = _run(lq, w, tree)
    # pre-fused tables: agreement counts = signed partial sums + the table's own -1 entries per leaf
    Hn = tree.H.numpy().astype(np.int64)
    feat = tree.feature.numpy()
    off = c_f
    for k, d in enumerate(w.dims):
        own = (feat >= off) & (feat < off + d.shape[1])
        neg = (Hn[own] == -1).sum(axis=0)
        np.testing.assert_array_equal(tables[k].cpu().numpy()[:, :leaves].astype(np.int64), Tk[k] + neg)
        assert (tables[k].cpu().numpy()[:, leaves:] == 0).all()
        off += d.shape[1]
    np.testing.assert_array_equal(target.cpu().numpy()[:leaves], (Hn != 0).sum(axis=0))
    assert (target.cpu().numpy()[leaves:] == 0xFF).all()
    np.testing.assert_array_equal(g_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(g_oh.cpu().numpy(), onehot)
    np.testing.assert_array_equal(m_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(m_oh.cpu().numpy(), onehot)
    assert (onehot.sum(axis=1) == 1).all()
    _check_masks(lq, w, tree, tables, Tk, leaf, onehot)


def _fact_side(lq, w, tree):
    """Keyword arguments for the join on the masks when the fact table has columns, after checking the
    packed buffer: count, column, threshold and the two mask rows of every node that tests a fact column
    (test true: the leaves whose path does not want it false; test false: those that do not want it true)."""
    if w.c_f == 0:
        return {}
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    buf = lq.lq_tree_fact_masks(w.c_f, f, t, H)
    torch.cuda.synchronize()
    Hn = tree.H.numpy().astype(np.int64)
    feat = tree.feature.numpy()
    p, leaves = Hn.shape
    words = lq.lq_tree_mask_words(leaves)
    assert buf.numel() == lq.lq_tree_fact_mask_bytes(p, leaves)
    raw = buf.cpu().numpy()
    nodes = np.flatnonzero(feat < w.c_f)
    assert int(raw[:4].view(np.int32)[0]) == len(nodes)
    np.testing.assert_array_equal(raw[16:16 + 4 * p].view(np.int32)[:len(nodes)], feat[nodes])
    np.testing.assert_array_equal(raw[16 + 4 * p:16 + 8 * p].view(np.float32)[:len(nodes)], tree.threshold.numpy()[nodes])
    start = (16 + 8 * p + 15) // 16 * 16
    got = raw[start:start + 16 * words * len(nodes)].view(np.uint64).reshape(len(nodes), words, 2)
    for which, keep in ((0, Hn[nodes] >= 0), (1, Hn[nodes] <= 0)):
        padded = np.zeros((len(nodes), words * 64), dtype=np.uint8)
        padded[:, :leaves] = keep
        want = np.packbits(padded.reshape(-1, words, 64), axis=2, bitorder="little").view(np.uint64).reshape(-1, words)
        np.testing.assert_array_equal(got[:, :, which], want)
    return {"X": w.X, "fact_masks": buf}


def _check_masks(lq, w, tree, tables, Tk, leaf, onehot):
    """Leaf masks: bit j of a row = (its table entry equals the number of nodes the dimension owns on
    the path to leaf j), from the oracle's tables; the join on the masks gives the oracle's leaves."""
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    Hn = tree.H.numpy().astype(np.int64)
    feat = tree.feature.numpy()
    leaves = Hn.shape[1]
    words = lq.lq_tree_mask_words(leaves)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H, c_f=w.c_f)
    fact = _fact_side(lq, w, tree)
    g_leaf, g_oh = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, want_onehot=True, **fact)
    g_leaf_only, none = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, **fact)
    torch.cuda.synchronize()
    off = w.c_f
    for k, d in enumerate(w.dims):
        own = (feat >= off) & (feat < off + d.shape[1])
        neg = (Hn[own] == -1).sum(axis=0)
        own_len = (Hn[own] != 0).sum(axis=0)
        bits = (Tk[k] + neg == own_len)                                  # [r_k x leaves]
        padded = np.zeros((bits.shape[0], words * 64), dtype=np.uint8)
        padded[:, :leaves] = bits
        want = np.packbits(padded.reshape(-1, words, 64), axis=2, bitorder="little").view(np.uint64).reshape(-1, words)
        got = masks[k].cpu().numpy().view(np.uint64)
        np.testing.assert_array_equal(got, want)
        off += d.shape[1]
    assert none is None
    np.testing.assert_array_equal(g_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(g_leaf_only.cpu().numpy(), leaf)
    np.testing.assert_array_equal(g_oh.cpu().numpy(), onehot)


def test_tree_on_a_subset_of_columns_and_leaf_only_output(lq):
    # the tree only tests columns of dimension 1; dimension 0 contributes all-zero tables
    w, tree = _case("subset", 6_007, 0, (30, 40), (6, 6), 12, WL.SEED0 + 600, tree_cols=range(6, 12))
    _, _, leaf = O.tree_predict(w.X, w.dims, w.fks, tree.feature, tree.threshold, tree.H)
    w = to_dev(w)
    tables, target, g_leaf, g_oh, m_leaf, _ = _run(lq, w, tree, onehot=False)
    assert g_oh is None
    assert (tables[0] == 0).all()
    np.testing.assert_array_equal(g_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(m_leaf.cpu().numpy(), leaf)


def test_degenerate_matrices_without_a_matching_leaf_give_minus_one(lq):
    """H need not come from a tree: a leaf that needs a node both true (+1) elsewhere is fine, but a
    column can also be unreachable for some rows; then no leaf matches and the index is -1."""
    w = WL.make_predict("degenerate", 2_000, 0, (20,), (2,), (1,), seed=WL.SEED0 + 601)
    feature = torch.tensor([0, 1], dtype=torch.int32)
    thr = torch.tensor([0.0, 0.0])
    H = torch.tensor([[1], [1]], dtype=torch.int8)            # one "leaf" that needs both nodes true
    _, onehot, leaf = O.tree_predict(w.X, w.dims, w.fks, feature, thr, H)
    assert (leaf == -1).any() and (leaf == 0).any()
    w = to_dev(w)
    tables, target = lq.lq_tree_project_dims(w.dims, 0, feature.cuda(), thr.cuda(), H.cuda())
    g_leaf, g_oh = lq.lq_fused_join_tree(None, w.fks, tables, target, feature.cuda(), thr.cuda(), H.cuda(),
                                         want_onehot=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(g_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(g_oh.cpu().numpy(), onehot)
    masks = lq.lq_tree_compress_tables(w.dims, tables, feature.cuda(), thr.cuda(), H.cuda())
    k_leaf, k_oh = lq.lq_fused_join_tree_masks(w.fks, masks, feature.cuda(), thr.cuda(), H.cuda(), want_onehot=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(k_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(k_oh.cpu().numpy(), onehot)


def test_check_fks_flag_on_the_tree_calls(lq):
    w, tree = _case("fk_check", 3_000, 0, (30, 40), (6, 6), 12, WL.SEED0 + 602)
    _, _, leaf = O.tree_predict(w.X, w.dims, w.fks, tree.feature, tree.threshold, tree.H)
    w = to_dev(w)
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, 0, f, t, H)
    good, _ = lq.lq_fused_join_tree(None, w.fks, tables, target, f, t, H, flags=lq.LQ_CHECK_FKS)
    good_m, _ = lq.lq_materialized_join_tree(None, w.dims, w.fks, f, t, H, flags=lq.LQ_CHECK_FKS)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(good.cpu().numpy(), leaf)
    np.testing.assert_array_equal(good_m.cpu().numpy(), leaf)
    bad = [w.fks[0].clone(), w.fks[1]]
    bad[0][1234] = 30                                   # one past the last row of dimension 0
    for call in (lambda: lq.lq_fused_join_tree(None, bad, tables, target, f, t, H, flags=lq.LQ_CHECK_FKS),
                 lambda: lq.lq_materialized_join_tree(None, w.dims, bad, f, t, H, flags=lq.LQ_CHECK_FKS)):
        with pytest.raises(lq.LQError) as e:
            call()
        assert e.value.status == "LQ_ERR_FK_RANGE"
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H)
    with pytest.raises(lq.LQError) as e:
        lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, flags=lq.LQ_CHECK_FKS)
    assert e.value.status == "LQ_ERR_UNSUPPORTED"


def test_tree_full_size_setting1_shape(lq):
    """Cardinality setting 1 at scale factor 8 (4.8M fact rows; dimensions 80,000 / 16,000 / 2,555),
    128 joined columns, 64 leaves: oracle on a row sample, fused vs non-fused over all rows."""
    n = 4_800_000
    w = WL.make_predict("tree_s1_sf8", n, 0, (80_000, 16_000, 2_555), (43, 43, 42), (1,), seed=WL.SEED0 + 700,
                        device="cuda")
    tree = WL.make_tree(128, 64, WL.SEED0 + 701)
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, 0, f, t, H)
    leaf, _ = lq.lq_fused_join_tree(None, w.fks, tables, target, f, t, H)
    leaf_m, _ = lq.lq_materialized_join_tree(None, w.dims, w.fks, f, t, H, chunk_rows=1 << 20)
    torch.cuda.synchronize()
    assert torch.equal(leaf, leaf_m)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H)
    leaf_k, _ = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H)
    torch.cuda.synchronize()
    assert torch.equal(leaf, leaf_k)
    rows = WL.sample_rows(n)
    sub = WL.take_rows(w, rows)
    _, _, want = O.tree_predict(None, sub.dims, sub.fks, tree.feature, tree.threshold, tree.H)
    np.testing.assert_array_equal(leaf[rows.cuda()].cpu().numpy(), want)
    assert len(np.unique(want)) > 20                      # the rows really spread over the leaves


@pytest.mark.parametrize("c_f,padded", [(4, False), (5, False), (3, True), (12, True)], ids=["cf4", "cf5", "cf3_strided", "cf12_strided"])
def test_masks_with_fact_columns_at_a_size_that_keeps_tables_in_lds(lq, c_f, padded):
    """Above 2^20 fact rows the mask join keeps small tables in LDS; here with nodes on the fact
    table's own columns as well (register and re-read forms, contiguous and strided X)."""
    n = (1 << 20) + 4_099
    w, tree = _case("masks_lds_fact", n, c_f, (3_000, 500, 40_000), (5, 4, 6), 64, WL.SEED0 + 610 + c_f)
    _, _, leaf = O.tree_predict(w.X, w.dims, w.fks, tree.feature, tree.threshold, tree.H)
    w = to_dev(w)
    if padded:                                            # rows of X 4 (c_f + 3) bytes apart: not 16-byte pieces
        wide = torch.zeros((n, c_f + 3), device="cuda")
        wide[:, :c_f] = w.X
        w.X = wide[:, :c_f]
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, H)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H, c_f=c_f)
    fact = _fact_side(lq, w, tree)
    got, _ = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, **fact)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), leaf)
    assert len(np.unique(leaf)) > 20


def test_masks_need_the_fact_side_when_the_fact_table_has_columns(lq):
    w, tree = _case("masks_no_fact_side", 1_000, 2, (30,), (4,), 8, WL.SEED0 + 620)
    w = to_dev(w)
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, _ = lq.lq_tree_project_dims(w.dims, 2, f, t, H)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H, c_f=2)
    with pytest.raises(lq.LQError) as e:
        lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, X=w.X)
    assert e.value.status == "LQ_ERR_NULL"


@pytest.mark.parametrize("leaves,c_f", [(24, 0), (64, 3), (300, 0), (2_000, 2)], ids=["l24", "l64_fact", "l300", "l2000_fact"])
def test_incremental_refresh_of_tree_tables_and_masks(lq, leaves, c_f):
    """Section 3.2: the pre-fused tables are constants only until a dimension row changes.  Refreshing a
    row range must give what a full pre-fusion (the oracle's) gives for the changed table, and must not
    touch other rows (every pre-fusion kernel: bit-mask form, per-leaf node lists)."""
    w, tree = _case("tree_refresh", 3_001, c_f, (500, 90), (6, 5), leaves, WL.SEED0 + 640 + leaves)
    w = to_dev(w)
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, H)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H, c_f=c_f)
    g = torch.Generator().manual_seed(WL.SEED0 + 641)
    for dim, first, count in ((0, 37, 101), (1, 0, 90), (0, 499, 1), (1, 45, 0)):
        w.dims[dim][first:first + count] = torch.randn((count, w.dims[dim].shape[1]), generator=g).cuda()
        before = [tb.clone() for tb in tables], [m.clone() for m in masks]
        lq.lq_tree_project_dim_rows(w.dims, c_f, tables, masks, f, t, H, dim, first, count)
        torch.cuda.synchronize()
        for k in range(2):                      # rows outside the range: untouched
            keep = torch.ones(tables[k].shape[0], dtype=torch.bool, device="cuda")
            if k == dim:
                keep[first:first + count] = False
            assert torch.equal(tables[k][keep], before[0][k][keep]) and torch.equal(masks[k][keep], before[1][k][keep])
    cpu = cpu_list(w.dims)
    Tk = O.tree_project(cpu, c_f, tree.feature, tree.threshold, tree.H)
    _, onehot, leaf = O.tree_predict(None if w.X is None else w.X.cpu(), cpu, cpu_list(w.fks), tree.feature, tree.threshold, tree.H)
    Hn = tree.H.numpy().astype(np.int64)
    feat = tree.feature.numpy()
    off = c_f
    for k, d in enumerate(cpu):
        own = (feat >= off) & (feat < off + d.shape[1])
        np.testing.assert_array_equal(tables[k].cpu().numpy()[:, :leaves].astype(np.int64), Tk[k] + (Hn[own] == -1).sum(axis=0))
        off += d.shape[1]
    got, _ = lq.lq_fused_join_tree(w.X, w.fks, tables, target, f, t, H)
    fact = _fact_side(lq, w, tree)
    got_k, oh_k = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, want_onehot=True, **fact)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), leaf)
    np.testing.assert_array_equal(got_k.cpu().numpy(), leaf)
    np.testing.assert_array_equal(oh_k.cpu().numpy(), onehot)
    # tables only (no masks given)
    lq.lq_tree_project_dim_rows(w.dims, c_f, tables, None, f, t, H, 0, 10, 20)
    with pytest.raises(lq.LQError) as e:
        lq.lq_tree_project_dim_rows(w.dims, c_f, tables, masks, f, t, H, 1, 80, 11)
    assert e.value.status == "LQ_ERR_SHAPE"


def test_mask_join_with_more_fact_side_nodes_than_the_lds_list_holds(lq):
    """H need not be a tree.  200 nodes, all on the 8 fact columns and one dimension column, 48 "leaves"
    that each want 4 nodes: above 2^20 rows the mask join keeps the first 128 fact-side nodes in LDS and
    reads the others from memory.  All three joins against the oracle on a row sample, and against each
    other on every row."""
    n, c_f, p, l = (1 << 20) + 333, 8, 200, 48
    w = WL.make_predict("masks_many_fact_nodes", n, c_f, (700,), (1,), (1,), seed=WL.SEED0 + 660, device="cuda")
    g = np.random.default_rng(WL.SEED0 + 661)
    feature = torch.from_numpy(g.integers(0, c_f + 1, size=p).astype(np.int32))
    feature[150:] = torch.from_numpy(g.integers(0, c_f, size=p - 150).astype(np.int32))    # the tail: fact columns only
    thr = torch.from_numpy(g.normal(0.0, 0.7, size=p).astype(np.float32))
    Hn = np.zeros((p, l), dtype=np.int8)
    for j in range(l):
        qs = np.concatenate([g.choice(150, size=2, replace=False), 150 + g.choice(50, size=2, replace=False)])
        Hn[qs, j] = g.choice([-1, 1], size=4)                                              # two wanted nodes beyond the first 128
    H = torch.from_numpy(Hn)
    f, t, Hd = feature.cuda(), thr.cuda(), H.cuda()
    assert int((feature < c_f).sum()) > 128
    tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, Hd)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, Hd, c_f=c_f)
    fmask = lq.lq_tree_fact_masks(c_f, f, t, Hd)
    leaf_b, _ = lq.lq_fused_join_tree(w.X, w.fks, tables, target, f, t, Hd)
    leaf_k, oh_k = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, want_onehot=True, X=w.X, fact_masks=fmask)
    leaf_l, _ = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, X=w.X, fact_masks=fmask)
    torch.cuda.synchronize()
    assert torch.equal(leaf_b, leaf_k) and torch.equal(leaf_b, leaf_l)
    rows = WL.sample_rows(n)
    sub = WL.take_rows(w, rows)
    _, onehot, want = O.tree_predict(sub.X, sub.dims, sub.fks, feature, thr, H)
    np.testing.assert_array_equal(leaf_l[rows.cuda()].cpu().numpy(), want)
    np.testing.assert_array_equal(oh_k[rows.cuda()].cpu().numpy(), onehot)
    assert (want >= 0).any() and (want == -1).any() and (onehot.sum(axis=1) > 1).any()


def _fact_lists(lq, buf, p, leaves):
    """The per-leaf lists of fact-side nodes at the end of the packed buffer: (complete?, offsets, entries)."""
    raw = buf.cpu().numpy()
    words = lq.lq_tree_mask_words(leaves)
    off = (16 + 8 * p + 15) // 16 * 16 + p * words * 16
    ent = off + (4 * (leaves + 1) + 15) // 16 * 16
    head = raw[:16].view(np.int32)
    offsets = raw[off:off + 4 * (leaves + 1)].view(np.int32)
    entries = raw[ent:ent + 16 * min(int(head[2]), 64 * leaves)].view(np.uint32).reshape(-1, 4)
    return int(head[1]), int(head[2]), offsets, entries


@pytest.mark.parametrize("kind", ["lists_and_not_a_tree", "chain_past_the_room_for_lists", "small_past_the_room_for_lists"])
def test_mask_join_walks_the_fact_side_nodes_of_each_candidate_leaf(lq, kind):
    """From four mask words on, the join with fact columns checks the lowest leaf the tables left possible against
    the fact-side nodes on its own path, read from per-leaf lists in the packed buffer (64 entries per leaf on
    average), and takes out all leaves that the first failed test excludes; a tree whose lists do not fit (a chain
    of 259 tests, all on fact columns) is joined node by node instead.  With an H that is no tree several leaves
    are reached per row: the one-hot rows hold all of them."""
    c_f, n = (12 if kind.startswith("small") else 5), 5_003
    w = WL.make_predict("masks_fact_lists_" + kind, n, c_f, (300,), (2,), (1,), seed=WL.SEED0 + 670)
    g = np.random.default_rng(WL.SEED0 + 671)
    if kind == "lists_and_not_a_tree":
        p, l = 120, 300
        feature = g.integers(0, c_f + 2, size=p).astype(np.int32)
        thr = g.normal(0.0, 0.7, size=p).astype(np.float32)
        Hn = np.zeros((p, l), dtype=np.int8)
        for j in range(l):
            Hn[g.choice(p, size=8, replace=False), j] = g.choice([-1, 1], size=8)
    elif kind == "small_past_the_room_for_lists":
        # 40 "leaves" that each want 70 of 80 tests that always come out true, and 4 of 20 real ones: on a fact table
        # of more than 8 columns small trees take the walk too, and fall back to the general kernel here
        p, l = 100, 40
        feature = g.integers(0, c_f, size=p).astype(np.int32)
        thr = g.normal(0.0, 0.7, size=p).astype(np.float32)
        thr[:80] = -1e30
        Hn = np.zeros((p, l), dtype=np.int8)
        for j in range(l):
            Hn[g.choice(80, size=70, replace=False), j] = 1
            Hn[80 + g.choice(20, size=4, replace=False), j] = g.choice([-1, 1], size=4)
    else:
        p, l = 259, 260
        feature = g.integers(0, c_f, size=p).astype(np.int32)
        thr = g.normal(1.8, 0.5, size=p).astype(np.float32)
        Hn = np.zeros((p, l), dtype=np.int8)
        for j in range(l):                                   # leaf j: tests 0 .. j - 1 false, test j true (the last: all false)
            Hn[:min(j, p), j] = -1
            if j < p:
                Hn[j, j] = 1
    feature, thr, H = torch.from_numpy(feature), torch.from_numpy(thr), torch.from_numpy(Hn)
    _, onehot, want = O.tree_predict(w.X, w.dims, w.fks, feature, thr, H)
    w = to_dev(w)
    f, t, Hd = feature.cuda(), thr.cuda(), H.cuda()
    assert lq.lq_tree_mask_words(l) >= 4 or c_f > 8
    tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, Hd)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, Hd, c_f=c_f)
    fmask = lq.lq_tree_fact_masks(c_f, f, t, Hd)
    leaf_k, oh_k = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, want_onehot=True, X=w.X, fact_masks=fmask)
    leaf_l, _ = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, X=w.X, fact_masks=fmask)
    none, oh_o = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, want_onehot=True, want_leaf=False, X=w.X, fact_masks=fmask)
    torch.cuda.synchronize()
    complete, total, offsets, entries = _fact_lists(lq, fmask, p, l)
    on_fact = feature.numpy() < c_f
    per_leaf = ((Hn != 0) & on_fact[:, None]).sum(axis=0)
    assert total == per_leaf.sum()
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(per_leaf)]))
    if kind == "lists_and_not_a_tree":
        assert complete == 1
        for j in (0, 1, 63, 64, 127, 128, l - 1):
            qs = np.flatnonzero((Hn[:, j] != 0) & on_fact)
            got = entries[offsets[j]:offsets[j + 1]]
            np.testing.assert_array_equal(got[:, 0], feature.numpy()[qs])
            np.testing.assert_array_equal(got[:, 1], (Hn[qs, j] < 0).astype(np.uint32))
            np.testing.assert_array_equal(got[:, 2], thr.numpy()[qs].view(np.uint32))
            np.testing.assert_array_equal(got[:, 3], np.cumsum(on_fact)[qs] - 1)         # place among the fact-side nodes
        assert (onehot.sum(axis=1) > 1).any() and (want == -1).any()
    elif kind == "small_past_the_room_for_lists":
        assert complete == 0 and total > 64 * l
        assert (onehot.sum(axis=1) > 1).any() and (want == -1).any() and len(np.unique(want)) >= 10
    else:
        assert complete == 0 and total > 64 * l
        assert len(np.unique(want)) >= 10 and (onehot.sum(axis=1) == 1).all()
    assert none is None
    np.testing.assert_array_equal(leaf_k.cpu().numpy(), want)
    np.testing.assert_array_equal(leaf_l.cpu().numpy(), want)
    np.testing.assert_array_equal(oh_k.cpu().numpy(), onehot)
    np.testing.assert_array_equal(oh_o.cpu().numpy(), onehot)


@pytest.mark.parametrize("l", [8_193, 16_384], ids=["l8193", "l16384"])
def test_fact_side_nodes_with_more_leaves_than_the_byte_join_lists_in_lds(lq, l):
    """The byte-table join prepares the fact side of the tree in LDS: the table-only target of every leaf, and per-leaf
    node lists up to 8,192 leaves; past that it reads a column of H for every leaf the tables leave possible.  Up to the
    largest tree the calls take (16,384 leaves): 40 nodes on three fact columns and one table, l columns of H that want
    three nodes each; all joins against the oracle."""
    c_f, p, n = 3, 40, 301
    w = WL.make_predict("many_leaves_fact", n, c_f, (50,), (4,), (1,), seed=WL.SEED0 + 680)
    g = np.random.default_rng(WL.SEED0 + 681 + l)
    feature = torch.from_numpy(g.integers(0, c_f + 4, size=p).astype(np.int32))
    thr = torch.from_numpy(g.normal(0.0, 0.7, size=p).astype(np.float32))
    Hn = np.zeros((p, l), dtype=np.int8)
    picks = np.argsort(g.random((l, p)), axis=1)[:, :3]
    Hn[picks, np.arange(l)[:, None]] = g.choice(np.array([-1, 1], dtype=np.int8), size=(l, 3))
    H = torch.from_numpy(Hn)
    _, onehot, want = O.tree_predict(w.X, w.dims, w.fks, feature, thr, H)
    assert (onehot.sum(axis=1) > 1).any()
    w = to_dev(w)
    f, t, Hd = feature.cuda(), thr.cuda(), H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, Hd)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, Hd, c_f=c_f)
    fmask = lq.lq_tree_fact_masks(c_f, f, t, Hd)
    leaf_b, oh_b = lq.lq_fused_join_tree(w.X, w.fks, tables, target, f, t, Hd, want_onehot=True)
    leaf_k, oh_k = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, want_onehot=True, X=w.X, fact_masks=fmask)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(leaf_b.cpu().numpy(), want)
    np.testing.assert_array_equal(oh_b.cpu().numpy(), onehot)
    np.testing.assert_array_equal(leaf_k.cpu().numpy(), want)
    np.testing.assert_array_equal(oh_k.cpu().numpy(), onehot)


def test_more_than_32767_nodes_most_of_them_on_no_path(lq):
    """The matrix form allows nodes that lie on no leaf's path (all-zero rows of H).  Past 32,767 nodes the
    pre-fusion walks the columns of H directly instead of building per-leaf node lists."""
    w, tree = _case("many_nodes", 1_003, 0, (40, 50), (6, 6), 12, WL.SEED0 + 610)
    p, l = tree.H.shape
    extra = 33_000 - p
    r = np.random.default_rng(610)
    feature = torch.cat([tree.feature, torch.from_numpy(r.integers(0, 12, size=extra).astype(np.int32))])
    thr = torch.cat([tree.threshold, torch.from_numpy(r.normal(size=extra).astype(np.float32))])
    H = torch.cat([tree.H, torch.zeros((extra, l), dtype=torch.int8)])
    perm = torch.from_numpy(r.permutation(33_000))              # the tree's own nodes end up anywhere
    feature, thr, H = feature[perm].contiguous(), thr[perm].contiguous(), H[perm].contiguous()
    _, onehot, leaf = O.tree_predict(w.X, w.dims, w.fks, feature, thr, H)
    assert (leaf >= 0).all()
    w = to_dev(w)
    f, t, Hd = feature.cuda(), thr.cuda(), H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, 0, f, t, Hd)
    g_leaf, g_oh = lq.lq_fused_join_tree(None, w.fks, tables, target, f, t, Hd, want_onehot=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(g_leaf.cpu().numpy(), leaf)
    np.testing.assert_array_equal(g_oh.cpu().numpy(), onehot)
    # the tables themselves: agreement counts = the oracle's signed partial sums + the table's own -1 entries per leaf
    Pw = O.tree_project([d.cpu() for d in w.dims], 0, feature, thr, H)
    Hn, feat, off = H.numpy().astype(np.int64), feature.numpy(), 0
    for k, d in enumerate(w.dims):
        own = (feat >= off) & (feat < off + d.shape[1])
        neg = (Hn[own] == -1).sum(axis=0)
        np.testing.assert_array_equal(tables[k][:, :l].cpu().numpy().astype(np.int64), Pw[k] + neg)
        off += d.shape[1]
