"""GPU parity past 2^31: inputs whose element count (rows x columns) or row count does not fit a
signed 32-bit index.  The oracle checks a deterministic row sample (rows are independent, so the
sample is exact for those rows; it holds the first and the last 4,096 rows, i.e. both ends of the
offset range).  Where the row count itself passes 2^31 the fact columns are one seeded block
repeated many times plus a ragged tail: results that are per row must then repeat with the block,
and sums must be `repetitions x oracle(block) + oracle(tail)` (a filter / join / aggregate over a
disjoint union of row sets is the sum over the parts)."""
import numpy as np
import pytest
import torch

from oracle import lq_oracle as O
from oracle import mmjoin_oracle as MJ
from tests.helpers import TOL_BF16, TOL_F32, assert_close, cpu_list
from workloads import star as WL

pytestmark = pytest.mark.gpu

BLOCK = 1 << 22
N_ROWS = (1 << 31) + 12_345          # row count for the cases that pass 2^31 rows


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _tile(block, n):
    """`block` repeated to n elements (the last repetition cut short)."""
    reps, tail = divmod(n, block.numel())
    return torch.cat([block.repeat(reps), block[:tail]])


def _sample_check(w, Y, tol, what):
    rows = WL.sample_rows(w.n, stride=99_991)
    sub = WL.take_rows(w, rows)
    want = O.join_predict(sub.X, sub.dims, sub.fks, sub.weights, sub.biases, nthreads=16)
    assert_close(Y[rows.to(Y.device)], want, tol, what)


def test_linear_model_with_more_than_2e31_fact_elements(lq):
    n = 300_000_013                      # x 8 fact columns = 2.4e9 elements; Y holds 1.2e9
    w = WL.make_predict("large_linear", n, 8, (1_000, 500), (16, 8), (4,), seed=WL.SEED0 + 900,
                        device="cuda", bias=True)
    assert w.X.numel() > 2**31
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
    torch.cuda.synchronize()
    _sample_check(w, Y, TOL_F32, "large linear model")


def test_mlp_64_to_1_with_more_than_2e31_fact_elements(lq):
    n = 540_000_001                      # x 4 fact columns = 2.16e9 elements
    w = WL.make_predict("large_mlp", n, 4, (1_000, 10_000, 100_000), (8, 8, 8), (64, 1),
                        seed=WL.SEED0 + 901, device="cuda", w_sigma=(0.2, 0.1))
    assert w.X.numel() > 2**31
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
    torch.cuda.synchronize()
    _sample_check(w, Y, TOL_F32, "large 64 -> 1 model")


def test_bf16_256_to_16_with_more_than_2e31_output_elements(lq):
    n = 140_000_003                      # x 16 outputs = 2.24e9 elements
    w = WL.make_predict("large_bf16", n, 0, (10_000,) * 4, (16,) * 4, (256, 16), seed=WL.SEED0 + 902,
                        device="cuda", dtype=torch.bfloat16, w_sigma=(1.0 / 8.0, 1.0 / 16.0))
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=torch.bfloat16)
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
    torch.cuda.synchronize()
    assert Y.numel() > 2**31 and Y.dtype == torch.bfloat16
    _sample_check(w, Y, TOL_BF16, "large bf16 256 -> 16 model")


def test_group_by_over_more_than_2e31_rows(lq):
    base = WL.c3_groupby(device="cuda", n=BLOCK, n_measures=2)
    reps, tail = divmod(N_ROWS, BLOCK)

    def oracle(m):
        return O.groupby_sum([f[:m].cpu() for f in base.fks], base.dim_rows, cpu_list(base.dim_mask),
                             cpu_list(base.dim_code), base.group_card, None,
                             [v[:m].cpu() for v in base.measures], nthreads=16)

    s_block, c_block = oracle(BLOCK)
    s_tail, c_tail = oracle(tail)
    fks = [_tile(f, N_ROWS) for f in base.fks]
    measures = [_tile(v, N_ROWS) for v in base.measures]
    sums, counts = lq.lq_masked_groupby_sum(fks, base.dim_rows, base.dim_mask, base.dim_code, base.group_card,
                                            None, measures)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sums.cpu().numpy(), reps * s_block + s_tail)
    np.testing.assert_array_equal(counts.cpu().numpy(), reps * c_block + c_tail)
    assert int(counts.sum()) > 2**25     # ~2.4 % of 2^31 rows survive the masks


def test_key_mapping_and_compaction_over_more_than_2e31_rows(lq):
    g = np.random.default_rng(WL.SEED0 + 903)
    pool = np.unique(g.integers(-2**31, 2**31 - 1, size=40_000, dtype=np.int64))
    g.shuffle(pool)
    key_S = pool[:30_000].astype(np.int32)
    key_R = g.choice(key_S, size=BLOCK).astype(np.int32)
    miss = g.random(BLOCK) < 0.03
    key_R[miss] = g.choice(pool[30_000:], size=int(miss.sum())).astype(np.int32)
    fk_w, rows_w, cols_w = MJ.key_to_row(key_R, key_S)

    table = lq.lq_keymap_build(torch.from_numpy(key_S).cuda(), flags=lq.LQ_CHECK_KEYS)
    block = torch.from_numpy(key_R).cuda()
    fk = lq.lq_keymap_lookup(table, _tile(block, N_ROWS))
    torch.cuda.synchronize()
    reps, tail = divmod(N_ROWS, BLOCK)
    want = torch.from_numpy(fk_w).cuda()
    assert torch.equal(fk[: reps * BLOCK].view(reps, BLOCK), want.expand(reps, BLOCK))
    assert torch.equal(fk[reps * BLOCK:], want[:tail])

    rows, cols, nnz = lq.lq_compact_matches(fk)
    torch.cuda.synchronize()
    m_block, m_tail = len(rows_w), int((fk_w[:tail] >= 0).sum())
    m = int(nnz.item())
    assert m == reps * m_block + m_tail
    rw, cw = torch.from_numpy(rows_w).cuda(), torch.from_numpy(cols_w).cuda()
    for j in (0, 1, reps // 2, reps - 1):           # whole repetitions: rows shifted by j blocks
        assert torch.equal(rows[j * m_block:(j + 1) * m_block], rw + j * BLOCK)
        assert torch.equal(cols[j * m_block:(j + 1) * m_block], cw)
    assert torch.equal(rows[reps * m_block:m], rw[:m_tail] + reps * BLOCK)
    assert torch.equal(cols[reps * m_block:m], cw[:m_tail])
    assert bool((rows[1:m] > rows[:m - 1]).all())   # matches stay in fact-row order throughout


def test_fused_tree_over_more_than_2e31_rows(lq):
    w = WL.make_predict("large_tree", BLOCK, 0, (800, 160), (12, 12), (1,), seed=WL.SEED0 + 904)
    tree = WL.make_tree(24, 48, WL.SEED0 + 905)
    _, _, leaf_w = O.tree_predict(w.X, w.dims, w.fks, tree.feature, tree.threshold, tree.H)
    f, t, H = tree.feature.cuda(), tree.threshold.cuda(), tree.H.cuda()
    dims = [d.cuda() for d in w.dims]
    tables, target = lq.lq_tree_project_dims(dims, 0, f, t, H)
    fks = [_tile(k.cuda(), N_ROWS) for k in w.fks]
    leaf, _ = lq.lq_fused_join_tree(None, fks, tables, target, f, t, H, want_onehot=False)
    torch.cuda.synchronize()
    reps, tail = divmod(N_ROWS, BLOCK)
    want = torch.from_numpy(np.asarray(leaf_w, dtype=np.int32)).cuda()
    assert torch.equal(leaf[: reps * BLOCK].view(reps, BLOCK), want.expand(reps, BLOCK))
    assert torch.equal(leaf[reps * BLOCK:], want[:tail])
    masks = lq.lq_tree_compress_tables(dims, tables, f, t, H)
    leaf_k, _ = lq.lq_fused_join_tree_masks(fks, masks, f, t, H)
    torch.cuda.synchronize()
    assert torch.equal(leaf_k, leaf)


@pytest.mark.parametrize("shape", [
    # name, dimension rows (the last table's projected rows pass 4 GiB), columns, layers, dtype
    ("mlp_64_1_f32", (1_000, (1 << 24) + 5), (8, 2), (64, 1), torch.float32),          # 256-byte projected rows
    ("mlp_128_4_f32", ((1 << 23) + 5,), (3,), (128, 4), torch.float32),                 # 512-byte projected rows
    ("mlp_64_64_1_f32", (1_000, (1 << 24) + 5), (8, 2), (64, 64, 1), torch.float32),    # matrix-core kernel: 2^28 pieces
    ("mlp_256_2_bf16", ((1 << 23) + 5, 500), (2, 6), (256, 2), torch.bfloat16),         # 512-byte bf16 rows
], ids=lambda s: s[0])
def test_projected_tables_of_4_gib_and_more(lq, shape):
    """A projected table whose byte size passes 2^32: the kernels that keep 32-bit byte offsets into a table
    must stand aside, and whichever kernel runs must address the far end of the table correctly.  Half of the
    fact rows point into the last 1,000 rows of the big table."""
    name, rows, cols, layers, dt = shape
    n = 20_011
    w = WL.make_predict(name, n, 4, rows, cols, layers, seed=WL.SEED0 + 950, device="cuda", dtype=dt,
                        w_sigma=[0.3] + [1.0 / np.sqrt(a) for a in layers[:-1]], bias=True)
    big = int(np.argmax(rows))
    far = torch.arange(n, device="cuda") % 2 == 0
    w.fks[big][far] = (rows[big] - 1 - torch.randint(0, 1_000, (int(far.sum()),), device="cuda")).to(torch.int32)
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=dt)
    assert P[big].numel() * P[big].element_size() >= 2 ** 32
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=torch.float32)
    torch.cuda.synchronize()
    want = O.join_predict(w.X.cpu(), cpu_list(w.dims), cpu_list(w.fks), cpu_list(w.weights), cpu_list(w.biases), nthreads=16)
    assert_close(Y, want, TOL_BF16 if dt == torch.bfloat16 else TOL_F32, f"{name}: projected table of {P[big].numel() * P[big].element_size()} bytes")
