"""The entry points enqueue plain kernels only (no memset nodes, no allocation, no host sync unless a
check flag is given), so a caller may record them into a HIP graph.  Each graph is replayed several
times with eager work and synchronisation in between and compared with the eager result every time."""
import pytest
import torch

from tests.helpers import to_dev
from workloads import star as WL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _capture(fn):
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        fn()                                  # warm-up on the capture stream (kernel attributes are set here)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        fn()
    return graph


def test_group_by_replays_match_eager(lq):
    g = to_dev(WL.c3_groupby(n=500_003))
    ws = torch.empty(lq.lq_groupby_workspace_bytes(g.dim_rows, g.group_card, 1), dtype=torch.uint8, device="cuda")
    sums = torch.empty((1, g.G), dtype=torch.int64, device="cuda")
    counts = torch.empty((g.G,), dtype=torch.int64, device="cuda")

    def call():
        lq.lq_masked_groupby_sum(g.fks, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, None, g.measures,
                                 sums=sums, counts=counts, ws=ws)
    call()
    torch.cuda.synchronize()
    ref_s, ref_c = sums.clone(), counts.clone()
    graph = _capture(call)
    for _ in range(4):
        sums.fill_(-1); counts.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(sums, ref_s) and torch.equal(counts, ref_c)
        call()                                 # eager work between replays
        torch.cuda.synchronize()


def test_prefusion_and_fused_predict_replays_match_eager(lq):
    w = to_dev(WL.make_predict("graph", 100_003, 4, (1_000, 5_000, 300), (32, 32, 32), (64, 1),
                               seed=WL.SEED0 + 5, w_sigma=(0.1, 0.1)))
    P = [torch.empty((d.shape[0], 64), device="cuda") for d in w.dims]
    Y = torch.empty((w.n, 1), device="cuda")

    def call():
        lq.lq_project_dims(w.dims, w.weights[0], w.c_f, P=P)
        lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, Y=Y)
    call()
    torch.cuda.synchronize()
    ref = Y.clone()
    graph = _capture(call)
    for _ in range(3):
        Y.fill_(7.0)
        for p in P:
            p.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, ref)
        call()
        torch.cuda.synchronize()


def test_raw_keys_to_ordered_aggregate_replays_match_eager(lq):
    """Key lookup -> group-by with reused side tables -> ORDER BY, recorded as one graph."""
    import numpy as np
    r = np.random.default_rng(12)
    n, rows = 300_007, (2_556, 3_000)
    keys_S = [torch.from_numpy((r.permutation(a) + 1).astype(np.int32)).cuda() for a in rows]
    keys_R = [torch.from_numpy(r.integers(0, a + 40, size=n).astype(np.int32)).cuda() for a in rows]
    maps = [lq.lq_keymap_build(k) for k in keys_S]
    codes = [torch.from_numpy(r.integers(0, c, size=a).astype(np.int32)).cuda() for a, c in zip(rows, (7, 25))]
    meas = [torch.from_numpy(r.integers(1, 1000, size=n).astype(np.int32)).cuda()]
    fks = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in rows]
    ws = torch.empty(lq.lq_groupby_workspace_bytes(rows, (7, 25), 1), dtype=torch.uint8, device="cuda")
    sums = torch.empty((1, 175), dtype=torch.int64, device="cuda")
    counts = torch.empty((175,), dtype=torch.int64, device="cuda")
    order = torch.empty(175, dtype=torch.int32, device="cuda")
    n_out = torch.empty(1, dtype=torch.int32, device="cuda")
    keys = [(lq.LQ_KEY_GROUP_COLUMN, 0, False), (lq.LQ_KEY_SUM, 0, True)]
    lq.lq_masked_groupby_sum(fks, rows, None, codes, (7, 25), None, meas, sums=sums, counts=counts, ws=ws)  # encodes the side tables

    def call():
        for m, kr, fk in zip(maps, keys_R, fks):
            lq.lq_keymap_lookup(m, kr, fk=fk)
        lq.lq_masked_groupby_sum(fks, rows, None, codes, (7, 25), None, meas, sums=sums, counts=counts, ws=ws,
                                 flags=lq.LQ_REUSE_SIDE_TABLES)
        lq.lq_order_groups((7, 25), sums, counts, keys, order=order, n_out=n_out)
    call()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (sums, counts, order, n_out, fks[0], fks[1])]
    assert int(n_out.item()) > 100 and int((fks[1] < 0).sum()) > 0
    graph = _capture(call)
    for _ in range(3):
        for t in (sums, counts, order, n_out, fks[0], fks[1]):
            t.fill_(-3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((sums, counts, order, n_out, fks[0], fks[1]), ref):
            assert torch.equal(got, want)
        call()
        torch.cuda.synchronize()


@pytest.mark.parametrize("leaves", [300, 257], ids=["rows_written_whole", "rows_cleared_then_set"])
def test_tree_mask_join_with_fact_columns_replays_match_eager(lq, leaves):
    """Leaf numbers and one-hot rows of a tree that tests fact columns: the call clears the one-hot rows with a
    fill kernel where it sets them byte by byte (257 leaves), and launches both forms of the fact side."""
    c_f = 5
    w = to_dev(WL.make_predict("graph_tree_fact", 70_001, c_f, (300, 200), (6, 6), (1,), seed=WL.SEED0 + 910))
    tree = WL.make_tree(c_f + 12, leaves, WL.SEED0 + 911)
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, H)
    masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H, c_f=c_f)
    fmask = lq.lq_tree_fact_masks(c_f, f, t, H)
    torch.cuda.synchronize()
    out = {}

    def call():
        out["leaf"], out["onehot"] = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, want_onehot=True, X=w.X,
                                                                  fact_masks=fmask)
    call()
    torch.cuda.synchronize()
    ref_leaf, ref_oh = out["leaf"].clone(), out["onehot"].clone()
    assert int(ref_oh.sum()) == w.n
    graph = _capture(call)                      # (the outputs of the captured call live in the graph's memory pool)
    g_leaf, g_oh = out["leaf"], out["onehot"]
    for _ in range(4):
        g_leaf.fill_(-7); g_oh.fill_(9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_leaf, ref_leaf) and torch.equal(g_oh, ref_oh)
        call()                                  # eager work between replays
        torch.cuda.synchronize()


def test_bucketed_group_by_with_a_fact_mask_replays_match_eager(lq):
    """More groups than LDS accumulators, a fact mask, the bucketed form: outputs and bucket counters are cleared by
    a kernel of the call."""
    import numpy as np
    r = np.random.default_rng(920)
    n, rows, card = 400_003, (300, 280, 5_000), (250, 240, 1)
    fks = [torch.from_numpy(r.integers(0, a, size=n).astype(np.int32)).cuda() for a in rows]
    codes = [torch.from_numpy(r.integers(0, c, size=a).astype(np.int32)).cuda() if c > 1 else None for a, c in zip(rows, card)]
    masks = [None, None, torch.from_numpy((r.random(rows[2]) < 0.7).astype(np.uint8)).cuda()]
    meas = [torch.from_numpy(r.integers(-1000, 100_000, size=n).astype(np.int32)).cuda()]
    fm = torch.from_numpy((r.random(n) < 0.8).astype(np.uint8)).cuda()
    G = 250 * 240
    ws = torch.empty(lq.lq_groupby_bucket_workspace_bytes(n, rows, card, 1), dtype=torch.uint8, device="cuda")
    sums = torch.empty((1, G), dtype=torch.int64, device="cuda")
    counts = torch.empty((G,), dtype=torch.int64, device="cuda")

    def call():
        lq.lq_masked_groupby_sum(fks, rows, masks, codes, card, fm, meas, sums=sums, counts=counts, ws=ws)
    call()
    torch.cuda.synchronize()
    ref_s, ref_c = sums.clone(), counts.clone()
    assert 0 < int(ref_c.sum()) < n
    graph = _capture(call)
    for _ in range(4):
        sums.fill_(-1); counts.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(sums, ref_s) and torch.equal(counts, ref_c)
        call()
        torch.cuda.synchronize()
