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
