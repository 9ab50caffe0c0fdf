"""Randomised differential run, GPU library against the oracles, on seeded random valid shapes of every
entry point: a bounded slice (a fixed list of seeds per entry point, about a minute in all) of the long
randomised runs the kernels were developed against.  Every case is compared with `oracle/` only, to the
same bars as the other parity tests (1e-4 fp32, 2e-2 bf16, integers bit for bit); a test stops at its
first mismatch and names the seed and the shape."""
import numpy as np
import pytest
import torch

from oracle import domain_oracle as DO
from oracle import lq_oracle as O
from oracle import mmjoin_oracle as MJ
from tests.helpers import TOL_BF16, TOL_F32, assert_close, to_dev
from workloads import star as WL

pytestmark = pytest.mark.gpu

SEED = 20230608


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _seeds(kind, count):
    return [int(s) for s in np.random.default_rng(SEED + kind).integers(0, 2 ** 31, size=count)]


def test_random_stars_and_models(lq):
    first = [1, 2, 3, 4, 6, 8, 12, 16, 20, 24, 32, 37, 48, 64, 72, 100, 128, 200, 256, 260, 516, 768, 1024, 2048]
    later = [1, 2, 3, 4, 5, 8, 16, 17, 24, 33, 48, 64]
    for seed in _seeds(0, 1200):
        r = np.random.default_rng(seed)
        bf = r.random() < 0.3
        K = int(r.integers(0, 9))
        c_f = int(r.choice([0, 0, 1, 3, 4, 5, 8, 9, 12, 16, 20]))
        if K == 0 and c_f == 0:
            c_f = 4
        rows = [int(r.integers(1, 300)) for _ in range(K)]
        cols = [int(r.integers(1, 20)) for _ in range(K)]
        nl = int(r.integers(1, 3 if bf else 5))
        layers = [int(r.choice(first))] + [int(r.choice(later)) for _ in range(nl - 1)]
        if bf:
            layers[0] = max(8, layers[0] // 8 * 8) if layers[0] > 64 else layers[0]
        n = int(r.choice([63, 64, 65, 255, 257, 1000, 4097, 20011]))
        if layers[0] >= 512 or bf:
            # (bf16: the 2e-2 bar is a per-element bound on rounding noise -- P and Y each round once to 2^-9 --
            # whose largest deviation grows with the number of outputs; a few thousand rows keep it well inside)
            n = min(n, 4097)
        desc = f"seed={seed} bf16={bf} n={n} c_f={c_f} rows={rows} cols={cols} layers={layers}"
        k = c_f + sum(cols)
        sig = [1.0 / np.sqrt(max(k, 1))] + [1.0 / np.sqrt(a) for a in layers[:-1]]
        w = WL.make_predict("random", n, c_f, rows, cols, layers, seed=seed,
                            dtype=torch.bfloat16 if bf else torch.float32, w_sigma=sig, bias=bool(r.integers(0, 2)))
        want = O.join_predict(w.X, w.dims, w.fks, w.weights, w.biases, nthreads=8)
        w = to_dev(w)
        tol = TOL_BF16 if bf else TOL_F32
        for pd, yd in ([(torch.bfloat16, torch.bfloat16), (torch.float32, torch.float32)] if bf else [(torch.float32,) * 2]):
            P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=pd)
            Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=yd)
            Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases, y_dtype=yd,
                                                 chunk_rows=int(r.choice([256, 1024, 8192])))
            torch.cuda.synchronize()
            assert_close(Y, want, tol, f"fused, {desc}")
            assert_close(Ym, want, tol, f"non-fused, {desc}")


def test_random_deeper_models(lq):
    """fp32 models of two to six layers with first layers of 20 .. 256 columns on one to eight tables: the shapes of the
    matrix-core kernel (one or two column parts, one to four tables prefetched and up to four more gathered inside
    the step, up to 64 fact columns, later layers up to 128 wide)."""
    first = [20, 24, 32, 36, 48, 64, 72, 100, 128, 132, 200, 256]
    later = [1, 2, 3, 4, 5, 8, 16, 17, 24, 33, 48, 64, 100, 128, 130, 200, 256]
    for seed in _seeds(7, 400):
        r = np.random.default_rng(seed)
        K = int(r.integers(1, 9))
        c_f = int(r.choice([0, 0, 1, 3, 4, 5, 8, 9, 12, 16, 20, 33, 64]))
        rows = [int(r.integers(1, 400)) for _ in range(K)]
        cols = [int(r.integers(1, 12)) for _ in range(K)]
        nl = int(r.integers(2, 7))
        layers = [int(r.choice(first))] + [int(r.choice(later)) for _ in range(nl - 1)]
        n = int(r.choice([1, 15, 16, 17, 63, 64, 65, 255, 1000, 4097]))
        k = c_f + sum(cols)
        sig = [1.0 / np.sqrt(max(k, 1))] + [1.4 / np.sqrt(a) for a in layers[:-1]]
        desc = f"seed={seed} n={n} c_f={c_f} rows={rows} cols={cols} layers={layers}"
        w = WL.make_predict("random_deep", n, c_f, rows, cols, layers, seed=seed, w_sigma=sig, bias=bool(r.integers(0, 2)))
        want = O.join_predict(w.X, w.dims, w.fks, w.weights, w.biases, nthreads=8)
        w = to_dev(w)
        P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
        Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
        torch.cuda.synchronize()
        assert_close(Y, want, TOL_F32, f"fused, {desc}")


def test_random_models_on_one_or_two_fact_rows_are_exact_on_small_integers(lq):
    for seed in _seeds(7, 100):
        r = np.random.default_rng(seed)
        K = int(r.integers(1, 5))
        rows = [int(r.integers(1, 50)) for _ in range(K)]
        cols = [int(r.integers(1, 6)) for _ in range(K)]
        layers = [int(r.choice([1, 4, 16, 64, 128, 512])), int(r.choice([1, 2, 4]))][: int(r.integers(1, 3))]
        n, c_f = int(r.integers(1, 3)), int(r.choice([0, 4]))
        w = WL.make_predict("random_exact", n, c_f, rows, cols, layers, seed=seed, integer_valued=True, bias=True)
        want = O.join_predict(w.X, w.dims, w.fks, w.weights, w.biases)
        assert np.abs(want).max() < 2 ** 23
        w = to_dev(w)
        P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
        Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(Y.cpu().double().numpy(), want, err_msg=f"seed={seed} n={n} rows={rows} layers={layers}")


def test_random_group_bys_and_aggregates(lq):
    for seed in _seeds(1, 500):
        r = np.random.default_rng(seed)
        K = int(r.integers(1, 6))
        n = int(r.choice([0, 1, 3, 4, 1023, 4099, 100003]))
        rows = [int(r.choice([1, 5, 100, 3000, 70000, 400000])) for _ in range(K)]
        many = r.random() < 0.3                                   # more groups than LDS accumulators
        card = [int(r.choice([1, 2, 30, 120, 300] if many else [1, 1, 2, 5, 7])) for _ in range(K)]
        card = [min(c, a) for c, a in zip(card, rows)]
        while np.prod(card, dtype=np.int64) * (13 if not many else 1) > (8192 if not many else 4_000_000):
            card[int(r.integers(0, K))] = 1
        fks = [torch.from_numpy(r.integers(-1 if r.random() < 0.3 else 0, a, size=n).astype(np.int32)) for a in rows]
        codes = [torch.from_numpy(r.integers(0, c, size=a).astype(np.int32)) if c > 1 else None for a, c in zip(rows, card)]
        masks = [torch.from_numpy((r.random(a) < 0.6).astype(np.uint8)) if r.random() < 0.6 else None for a in rows]
        M = int(r.integers(1, 5))
        meas = [torch.from_numpy(r.integers(-1000, 100000, size=n).astype(np.int32)) for _ in range(M)]
        fm = torch.from_numpy((r.random(n) < 0.8).astype(np.uint8)) if r.random() < 0.4 else None
        desc = f"seed={seed} n={n} rows={rows} card={card} M={M} fact_mask={fm is not None} masks={[m is not None for m in masks]}"
        ws, wc = O.groupby_sum(fks, rows, masks, codes, card, fm, meas)
        dv = lambda t: None if t is None else t.cuda()
        s, c = lq.lq_masked_groupby_sum([dv(f) for f in fks], rows, [dv(m) for m in masks], [dv(x) for x in codes], card,
                                        dv(fm), [dv(m) for m in meas])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(s.cpu().numpy(), ws, err_msg=desc)
        np.testing.assert_array_equal(c.cpu().numpy(), wc, err_msg=desc)
        if M <= 2 and n > 0:
            preds = [(meas[0], int(r.integers(-1000, 100)), int(r.integers(100, 100000)))]
            ms = [("mul" if M > 1 else "col", meas[0], meas[1] if M > 1 else None)]
            npy = lambda t: None if t is None else t.numpy()
            want = O.groupby_agg([f.numpy() for f in fks], rows, [npy(m) for m in masks], [npy(x) for x in codes], card,
                                 [(p[0].numpy(), p[1], p[2]) for p in preds], [(o, a.numpy(), npy(b)) for o, a, b in ms])
            got = lq.lq_groupby_agg([dv(f) for f in fks], rows, [dv(m) for m in masks], [dv(x) for x in codes], card,
                                    [(dv(p[0]), p[1], p[2]) for p in preds], [(o, dv(a), dv(b)) for o, a, b in ms])
            torch.cuda.synchronize()
            for name, wv in zip(("sum", "min", "max", "count"), want):
                np.testing.assert_array_equal(got[name].cpu().numpy(), wv, err_msg=f"{name}, {desc}")


def test_random_trees(lq):
    for seed in _seeds(2, 300):
        r = np.random.default_rng(seed)
        K = int(r.integers(0, 5))
        c_f = int(r.choice([0, 0, 2, 3, 4, 8, 11]))
        if K == 0 and c_f == 0:
            c_f = 5
        rows = [int(r.integers(1, 500)) for _ in range(K)]
        cols = [int(r.integers(1, 12)) for _ in range(K)]
        leaves = int(r.choice([2, 3, 7, 16, 17, 48, 64, 65, 100, 128, 129, 200, 256, 257, 300, 384, 512, 640, 1024, 1100]))
        n = int(r.choice([1, 7, 64, 1000, 4099]))
        desc = f"seed={seed} n={n} c_f={c_f} rows={rows} cols={cols} leaves={leaves}"
        w = WL.make_predict("random_tree", n, c_f, rows, cols, (1,), seed=seed)
        tree = WL.make_tree(c_f + sum(cols), leaves, seed + 1)
        _, oh, leaf = O.tree_predict(w.X, w.dims, w.fks, tree.feature, tree.threshold, tree.H)
        w = to_dev(w)
        f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
        tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, H)
        gl, go = lq.lq_fused_join_tree(w.X, w.fks, tables, target, f, t, H, want_onehot=True)
        ml, mo = lq.lq_materialized_join_tree(w.X, w.dims, w.fks, f, t, H, want_onehot=True, chunk_rows=512)
        masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, H, c_f=c_f)
        kw = {"X": w.X, "fact_masks": lq.lq_tree_fact_masks(c_f, f, t, H)} if c_f else {}
        kl, ko = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, want_onehot=True, **kw)
        kl2, _ = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, H, **kw)
        torch.cuda.synchronize()
        for got_leaf, got_oh, what in ((gl, go, "byte tables"), (ml, mo, "non-fused"), (kl, ko, "leaf masks"), (kl2, None, "leaf masks, leaf only")):
            np.testing.assert_array_equal(got_leaf.cpu().numpy(), leaf, err_msg=f"{what}, {desc}")
            if got_oh is not None:
                np.testing.assert_array_equal(got_oh.cpu().numpy(), oh, err_msg=f"{what} one-hot, {desc}")
        if K > 0:   # change rows of one table, refresh them, compare with a full pre-fusion
            dim = int(r.integers(0, K))
            first_row = int(r.integers(0, rows[dim]))
            cnt = int(r.integers(0, rows[dim] - first_row + 1))
            w.dims[dim][first_row:first_row + cnt] = torch.randn((cnt, cols[dim]), device="cuda")
            lq.lq_tree_project_dim_rows(w.dims, c_f, tables, masks, f, t, H, dim, first_row, cnt)
            t2, _ = lq.lq_tree_project_dims(w.dims, c_f, f, t, H)
            m2 = lq.lq_tree_compress_tables(w.dims, t2, f, t, H, c_f=c_f)
            torch.cuda.synchronize()
            for k in range(K):
                assert torch.equal(tables[k], t2[k]) and torch.equal(masks[k], m2[k]), f"refresh differs, {desc}"


def test_random_path_matrices_that_are_no_trees(lq):
    """H in its matrix form (Section 3.3.1) with any set of wanted outcomes per column, and chains of tests: several
    leaves or none are reached per row, fact-side lists of any length.  Byte-table join, mask join with leaf and
    one-hot rows together and each alone, against the oracle."""
    for seed in _seeds(7, 250):
        r = np.random.default_rng(seed)
        K = int(r.choice([0, 1, 1, 2, 3, 5]))
        c_f = int(r.choice([0, 2, 4, 7, 9, 12, 20]))
        if K == 0 and c_f == 0:
            c_f = 3
        rows = [int(r.integers(1, 400)) for _ in range(K)]
        cols = [int(r.integers(1, 9)) for _ in range(K)]
        n = int(r.choice([1, 63, 65, 257, 1000, 4099]))
        kw = c_f + sum(cols)
        if r.random() < 0.7:
            p, l = int(r.integers(1, 150)), int(r.choice([1, 5, 48, 64, 70, 130, 200, 260, 400]))
            per = int(r.integers(1, min(p, 9) + 1))
            thr = r.normal(0, 0.7, size=p).astype(np.float32)
            Hn = np.zeros((p, l), dtype=np.int8)
            for j in range(l):
                Hn[r.choice(p, size=per, replace=False), j] = r.choice([-1, 1], size=per)
        else:
            p = int(r.choice([5, 70, 130, 200]))
            l = p + 1
            thr = r.normal(1.5, 0.6, size=p).astype(np.float32)
            Hn = np.zeros((p, l), dtype=np.int8)
            for j in range(l):                           # leaf j: tests before j false, test j true
                Hn[:min(j, p), j] = -1
                if j < p:
                    Hn[j, j] = 1
        feature = torch.from_numpy(r.integers(0, kw, size=p).astype(np.int32))
        thr, H = torch.from_numpy(thr), torch.from_numpy(Hn)
        desc = f"seed={seed} n={n} c_f={c_f} rows={rows} cols={cols} p={p} l={l}"
        w = WL.make_predict("random_matrix", n, c_f, rows, cols, (1,), seed=seed)
        _, oh, leaf = O.tree_predict(w.X, w.dims, w.fks, feature, thr, H)
        w = to_dev(w)
        f, t, Hd = feature.cuda(), thr.cuda(), H.cuda()
        tables, target = lq.lq_tree_project_dims(w.dims, c_f, f, t, Hd)
        masks = lq.lq_tree_compress_tables(w.dims, tables, f, t, Hd, c_f=c_f)
        fact = {"X": w.X, "fact_masks": lq.lq_tree_fact_masks(c_f, f, t, Hd)} if c_f else {}
        gl, go = lq.lq_fused_join_tree(w.X, w.fks, tables, target, f, t, Hd, want_onehot=True)
        kl, ko = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, want_onehot=True, **fact)
        kl2, _ = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, **fact)
        _, ko2 = lq.lq_fused_join_tree_masks(w.fks, masks, f, t, Hd, want_leaf=False, want_onehot=True, **fact)
        torch.cuda.synchronize()
        for got_leaf, got_oh, what in ((gl, go, "byte tables"), (kl, ko, "leaf masks"), (kl2, None, "leaf masks, leaf only"),
                                       (None, ko2, "leaf masks, one-hot only")):
            if got_leaf is not None:
                np.testing.assert_array_equal(got_leaf.cpu().numpy(), leaf, err_msg=f"{what}, {desc}")
            if got_oh is not None:
                np.testing.assert_array_equal(got_oh.cpu().numpy(), oh, err_msg=f"{what} one-hot, {desc}")


def test_random_key_maps(lq):
    for seed in _seeds(3, 300):
        r = np.random.default_rng(seed)
        wide = r.random() < 0.35                                     # 64-bit key values
        rr = int(r.choice([1, 2, 7, 100, 2556, 8192, 30000, 70000]))
        n = int(r.choice([1, 5, 1000, 100003, 600001]))
        lo, hi = (-2 ** 63 + 1, 2 ** 63 - 1) if wide else (-2 ** 31, 2 ** 31 - 1)
        dense = r.random() < 0.6
        if dense:
            base = int(r.choice([lo, -5, 0, 1, 19920101, hi - 5 * rr]))
            span = min(int(rr * r.choice([1.0, 1.5, 3.9, 4.5, 9.0])) + 1, hi - base)
            pool = base + r.permutation(span)[:rr].astype(np.int64)
        else:
            pool = np.unique(r.integers(lo, hi, size=rr * 2 + 8, dtype=np.int64))
            r.shuffle(pool)
            pool = pool[:rr]
        rr = len(pool)
        kt = np.int64 if wide else np.int32
        key_S = pool.astype(kt)
        key_R = r.choice(key_S, size=n).astype(kt)
        m = r.random(n) < 0.2
        key_R[m] = r.integers(lo, hi, size=int(m.sum()), dtype=np.int64).astype(kt)
        desc = f"seed={seed} 64-bit={wide} r={rr} n={n} dense={dense}"
        fk_w, rows_w, cols_w = MJ.key_to_row(key_R, key_S)
        if wide:
            tab = lq.lq_keymap64_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
            fk = lq.lq_keymap64_lookup(tab, torch.from_numpy(key_R).cuda())
        else:
            split = int(r.integers(1, rr + 1))
            tab = lq.lq_keymap_build(torch.from_numpy(key_S[:split]).cuda(), max_keys=rr)
            if split < rr:
                try:
                    lq.lq_keymap_insert(tab, torch.from_numpy(key_S[split:]).cuda(), split, flags=lq.LQ_CHECK_KEYS)
                except lq.LQError as e:            # a direct map only takes keys inside its window: rebuild with all keys
                    assert e.status == "LQ_ERR_WORKSPACE", desc
                    tab = lq.lq_keymap_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
            fk = lq.lq_keymap_lookup(tab, torch.from_numpy(key_R).cuda())
        rws, cls, nnz = lq.lq_compact_matches(fk)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(fk.cpu().numpy(), fk_w, err_msg=desc)
        mm = int(nnz.item())
        assert mm == len(rows_w), desc
        np.testing.assert_array_equal(rws[:mm].cpu().numpy(), rows_w, err_msg=desc)
        np.testing.assert_array_equal(cls[:mm].cpu().numpy(), cols_w, err_msg=desc)


def test_random_group_domains_and_orderings(lq):
    for seed in _seeds(4, 150):
        r = np.random.default_rng(seed)
        rows = int(r.choice([1, 2, 63, 64, 65, 1000, 4099, 300001]))
        nc = int(r.integers(1, 5))
        spans = [int(r.choice([1, 2, 5, 40, 3000, 2 ** 31 - 1])) for _ in range(nc)]
        cols = [r.integers(-s, s, size=rows, dtype=np.int64).astype(np.int32) if s > 1 else np.full(rows, 7, dtype=np.int32)
                for s in spans]
        desc = f"seed={seed} rows={rows} spans={spans}"
        wv, wc = DO.group_domain(cols)
        if len(wv) > 65535:
            with pytest.raises(lq.LQError) as e:
                lq.lq_group_domain([torch.from_numpy(c).cuda() for c in cols])
            assert e.value.status == "LQ_ERR_UNSUPPORTED", desc
        else:
            code, values, card = lq.lq_group_domain([torch.from_numpy(c).cuda() for c in cols])
            torch.cuda.synchronize()
            assert card == len(wv), desc
            np.testing.assert_array_equal(values.cpu().numpy(), wv, err_msg=desc)
            np.testing.assert_array_equal(code.cpu().numpy(), wc, err_msg=desc)
    for seed in _seeds(5, 300):
        r = np.random.default_rng(seed)
        ng = int(r.integers(0, 5))
        card = [int(r.choice([1, 2, 3, 5, 7, 16, 25])) for _ in range(ng)]
        while np.prod(card) > 8192:
            card[int(r.integers(0, ng))] = 1
        G = int(np.prod(card)) if ng else 1
        M = int(r.integers(1, 5))
        counts = r.integers(0, 3, size=G)
        sums = r.integers(-5, 6, size=(M, G))
        if r.random() < 0.3:
            sums = r.integers(-2 ** 63, 2 ** 63 - 1, size=(M, G), dtype=np.int64)
        keys = []
        for _ in range(int(r.integers(0, 5))):
            kd = int(r.integers(0, 3))
            if kd == 0 and ng == 0:
                kd = 2
            keys.append((kd, int(r.integers(0, ng)) if kd == 0 else (int(r.integers(0, M)) if kd == 1 else 0), bool(r.integers(0, 2))))
        desc = f"seed={seed} card={card} M={M} keys={keys}"
        want = DO.order_groups(card, sums, counts, keys)
        order, n_out = lq.lq_order_groups(card, torch.from_numpy(sums.astype(np.int64)).cuda(),
                                          torch.from_numpy(counts.astype(np.int64)).cuda(), keys)
        torch.cuda.synchronize()
        nn = int(n_out.item())
        assert nn == len(want), desc
        np.testing.assert_array_equal(order.cpu().numpy()[:nn], want, err_msg=desc)
