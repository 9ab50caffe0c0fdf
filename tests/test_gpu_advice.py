"""The fuse / do-not-fuse flag of lq_fusion_advice against what this library measures on the GPU: the 28
k x l cells of the linear-operator sweep (cardinality setting 1 at sf 4, Table 4 / Table 5: k = 2^4..2^7,
l = 2^1..2^7).  Wherever the measured difference between the two pipelines exceeds 20 %, the flag must
have the sign of (non-fused - fused - pre-fusion / q), for q = 1 (dimension tables change before every
query) and for pre-fusion paid once and amortised away.  Timing cells closer than 20 % are not judged."""
import pytest
import torch

pytestmark = pytest.mark.gpu

ROWS = (60_000, 8_000, 2_555)
SPLIT = {16: (8, 4, 4), 32: (12, 12, 8), 64: (24, 20, 20), 128: (44, 44, 40)}
N = 2_400_000


def _median_ms(fn, iters=7, warmup=2):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); fn(); b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b))
    return sorted(ts)[len(ts) // 2]


def test_fuse_flag_agrees_with_the_measured_sweep():
    import paper_2306_08367_amd as lq
    from workloads import star as WL
    dev = torch.device("cuda:0")
    ws = None
    judged, wrong = 0, []
    for k_in, cols in SPLIT.items():
        for l_out in (2, 4, 8, 16, 32, 64, 128):
            w = WL.make_predict("advice", N, 0, ROWS, cols, (l_out,), seed=WL.SEED0 + 5000 + k_in, device=dev)
            P = lq.lq_project_dims(w.dims, w.weights[0], 0)
            Y = torch.empty((N, l_out), dtype=torch.float32, device=dev)
            need = lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, k_in, w.weights, 1 << 21)
            if ws is None or ws.numel() < need:
                ws = torch.empty(need, dtype=torch.uint8, device=dev)
            fused = _median_ms(lambda: lq.lq_fused_join_predict(None, w.fks, P, w.weights, None, Y=Y))
            pre = _median_ms(lambda: lq.lq_project_dims(w.dims, w.weights[0], 0, P=P))
            mat = _median_ms(lambda: lq.lq_materialized_join_predict(None, w.dims, w.fks, w.weights, None, Y=Y, ws=ws),
                             iters=5, warmup=1)
            for q, pre_share in ((1.0, pre), (1e9, 0.0)):
                adv = lq.lq_fusion_advice(N, 0, list(zip(ROWS, cols)), [l_out], queries_per_update=q)
                a, b = mat, fused + pre_share
                if abs(a - b) <= 0.2 * max(a, b):
                    continue
                judged += 1
                if adv["fuse"] != int(a > b):
                    wrong.append((k_in, l_out, q, round(fused, 4), round(pre, 4), round(mat, 4), adv["fuse"]))
            del w, P, Y
    assert judged >= 30, f"only {judged} cells had a measured gap above 20 %"
    assert not wrong, f"flag disagrees with the measurement in (k, l, q, fused ms, pre-fusion ms, non-fused ms, flag): {wrong}"
