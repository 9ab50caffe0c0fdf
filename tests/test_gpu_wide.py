"""GPU parity for wide linear operators: first-layer widths above 256 (fp32) / 512 (bf16) up to 2^11,
the output shapes of the paper's cardinality setting 2 (Table 5: k = 2^8 .. 2^11, l up to k; Q5 / Q6 of
Section 4.3), against the fp64 oracle.  Dimension tables have setting 2's sizes at sf 4 (Table 4):
part 2,000 * floor(1 + log2 sf) = 6,000 rows, supplier sf * 2,000 = 8,000, date 7 * 365 = 2,555, fact
sf * 3,000 = 12,000 rows; all features live in the dimension tables unless a case says otherwise.

Bar: 1e-4 (fp32) / 2e-2 (bf16) per element as |y - want| <= tol * (|want| + rms(want))."""
import numpy as np
import pytest
import torch

from oracle import lq_oracle as O
from tests.helpers import TOL_BF16, TOL_F32, assert_close, cpu_list, to_dev
from workloads import star as WL

pytestmark = pytest.mark.gpu

S2_ROWS = (6_000, 8_000, 2_555)
S2_FACT = 12_000


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _oracle(w, nthreads=16):
    return O.join_predict(None if w.X is None else w.X.cpu(), cpu_list(w.dims), cpu_list(w.fks),
                          cpu_list(w.weights), cpu_list(w.biases), nthreads=nthreads)


def _cols(k, parts):
    base = k // parts
    return tuple(base + (1 if i < k - base * parts else 0) for i in range(parts))


def _sigmas(k, layers):
    # keeps hidden units and outputs of order one whatever the widths are
    return [1.0 / np.sqrt(k)] + [1.0 / np.sqrt(w) for w in layers[:-1]]


WIDE_F32 = [
    # name, n, c_f, dim_rows, k (joined width), layers, bias
    ("l768_linear", S2_FACT, 0, S2_ROWS, 256, (768,), True),
    ("l1024_linear_cf4", S2_FACT, 4, S2_ROWS, 256, (1024,), False),
    ("l2048_linear", S2_FACT, 0, S2_ROWS, 256, (2048,), True),
    ("l1024_mlp_1", S2_FACT, 0, S2_ROWS, 256, (1024, 1), True),
    ("l2048_mlp_4_cf8", S2_FACT, 8, S2_ROWS, 256, (2048, 4), True),
    ("l768_mlp_16", S2_FACT, 0, S2_ROWS, 256, (768, 16), False),
    # k = l = 2^10 on setting 2 at sf 1 (3,000 fact rows; part 2,000, supplier 2,000)
    ("k1024_l1024_linear_sf1", 3_000, 0, (2_000, 2_000, 2_555), 1024, (1024,), True),
    # widths just above the narrower kernels' limit, not a multiple of a 256-column pass, ragged row counts
    ("l260_linear", 4_099, 4, (300, 200), 64, (260,), True),
    ("l516_mlp_2", 2_049, 3, (300, 200, 100), 96, (516, 2), True),
    ("l1000_mlp_1_one_row", 1, 4, (30, 20), 32, (1000, 1), True),
    ("l1284_linear_63_rows", 63, 0, (30, 20), 32, (1284,), False),
    ("l2048_mlp_3_65_rows", 65, 2, (30,), 16, (2048, 3), True),
    ("l4096_linear", 1_025, 0, (100, 50), 32, (4096,), True),
    ("l512_mlp_9_k4_cf5", 3_001, 5, (50, 60, 70, 80), 64, (512, 9), True),
    # five to eight dimension tables
    ("l768_linear_k5", 2_001, 0, (100, 200, 300, 400, 500), 40, (768,), False),
    ("l1024_mlp_1_k8_cf4", 1_501, 4, (10, 20, 30, 40, 50, 60, 70, 80), 32, (1024, 1), True),
    # shapes that stay on the general kernels: wide first layer followed by a wide or a third layer
    ("l1024_mlp_64_1", 1_033, 4, (100, 200), 32, (1024, 64, 1), True),
    ("l768_mlp_40", 1_111, 0, (100, 200), 32, (768, 40), False),
    ("l768_linear_cf20", 777, 20, (100, 200), 52, (768,), True),
]


@pytest.mark.parametrize("shape", WIDE_F32, ids=[s[0] for s in WIDE_F32])
def test_wide_operators_fp32(lq, shape):
    name, n, c_f, rows, k, layers, bias = shape
    cols = _cols(k - c_f, len(rows))
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 4000 + len(name),
                        w_sigma=_sigmas(k, layers), bias=bias)
    want = _oracle(w)
    w = to_dev(w)
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
    Pw = O.project_dims(cpu_list(w.dims), w.weights[0].cpu(), w.c_f)
    for j in range(len(P)):
        assert_close(P[j], Pw[j], TOL_F32, f"{name}: P[{j}]")
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
    torch.cuda.synchronize()
    assert_close(Y, want, TOL_F32, f"{name}: fused")
    Yg = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, flags=lq.LQ_FORCE_GENERIC)
    torch.cuda.synchronize()
    assert_close(Yg, want, TOL_F32, f"{name}: shape-agnostic kernel")
    Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases, chunk_rows=4096)
    torch.cuda.synchronize()
    assert_close(Ym, want, TOL_F32, f"{name}: non-fused pipeline")


WIDE_BF16 = [
    ("bf16_l1024_linear", S2_FACT, 0, S2_ROWS, 256, (1024,), True),
    ("bf16_l2048_linear_cf4", S2_FACT, 4, S2_ROWS, 256, (2048,), False),
    ("bf16_l1024_mlp_1", S2_FACT, 0, S2_ROWS, 256, (1024, 1), True),
    ("bf16_l2048_mlp_4", S2_FACT, 0, S2_ROWS, 256, (2048, 4), True),
    ("bf16_l520_linear", 4_099, 8, (300, 200), 64, (520,), True),
    ("bf16_l1032_mlp_2_65_rows", 65, 3, (30, 20), 32, (1032, 2), True),
    ("bf16_l4096_linear_k1", 1_025, 0, (100,), 16, (4096,), False),
    ("bf16_l1024_mlp_16", 2_049, 0, (100, 200), 32, (1024, 16), True),
]


@pytest.mark.parametrize("shape", WIDE_BF16, ids=[s[0] for s in WIDE_BF16])
def test_wide_operators_bf16(lq, shape):
    name, n, c_f, rows, k, layers, bias = shape
    cols = _cols(k - c_f, len(rows))
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 4100 + len(name),
                        dtype=torch.bfloat16, w_sigma=_sigmas(k, layers), bias=bias)
    want = _oracle(w)
    w = to_dev(w)
    for p_dtype, y_dtype in ((torch.bfloat16, torch.bfloat16), (torch.bfloat16, torch.float32)):
        P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=p_dtype)
        Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=y_dtype)
        torch.cuda.synchronize()
        assert_close(Y, want, TOL_BF16, f"{name}: fused, Y {y_dtype}")
    Yg = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=torch.float32,
                                  flags=lq.LQ_FORCE_GENERIC)
    torch.cuda.synchronize()
    assert_close(Yg, want, TOL_BF16, f"{name}: shape-agnostic kernel")


def test_wide_operator_on_column_slices(lq):
    """X, the projected tables and Y as column slices of wider buffers (row strides above the widths;
    16-byte alignment kept, then broken): the same results, neighbours untouched."""
    n, c_f, l = 2_049, 4, 1024
    w = WL.make_predict("wide_strided", n, c_f, (300, 200), (16, 16), (l,), seed=WL.SEED0 + 4200,
                        w_sigma=[0.2], bias=True)
    want = _oracle(w)
    w = to_dev(w)
    for pad in (8, 3):
        Xw = torch.zeros((n, c_f + 4), device="cuda"); Xw[:, 4:] = w.X
        P = []
        for d in w.dims:
            buf = torch.zeros((d.shape[0], l + 2 * pad), device="cuda")
            P.append(buf[:, pad:pad + l])
        lq.lq_project_dims(w.dims, w.weights[0], c_f, P=P)
        Yw = torch.full((n, l + 2 * pad), -1.0, device="cuda")
        lq.lq_fused_join_predict(Xw[:, 4:], w.fks, P, w.weights, w.biases, Y=Yw[:, pad:pad + l])
        torch.cuda.synchronize()
        assert_close(Yw[:, pad:pad + l], want, TOL_F32, f"strided wide operator, pad {pad}")
        assert (Yw[:, :pad] == -1).all() and (Yw[:, pad + l:] == -1).all()


def test_wide_operator_fk_indexing_is_bit_exact(lq):
    """Small integers everywhere: every hidden unit and output is an integer below 2^24, so the wide
    kernels must reproduce the oracle bit for bit (a wrong column offset or key would not)."""
    for layers in ((1024,), (768, 4)):
        w = WL.make_predict("wide_exact", 3_003, 4, (97, 1_013, 31), (8, 4, 8), layers, seed=WL.SEED0 + 4300,
                            integer_valued=True, bias=True)
        want = _oracle(w)
        assert np.abs(want).max() < 2 ** 23
        w = to_dev(w)
        P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
        Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(Y.cpu().double().numpy(), want)


LAYERED = [
    # name, n, c_f, dim_rows, k, layers, dtype, bias
    ("l512_64_1", 3_001, 4, S2_ROWS, 256, (512, 64, 1), torch.float32, True),
    ("l1024_1024", 1_025, 0, S2_ROWS, 256, (1024, 1024), torch.float32, False),
    ("l300_64_1", 2_049, 4, (300, 200), 64, (300, 64, 1), torch.float32, True),
    ("l512_17", 4_099, 8, (300, 200, 100), 96, (512, 17), torch.float32, True),
    ("l262_40_3_ragged", 777, 3, (30, 20), 32, (262, 40, 3), torch.float32, True),
    ("l256_300_2_wide_later_layer", 1_111, 4, (100, 200), 32, (256, 300, 2), torch.float32, False),
    ("l2048_256_one_row", 1, 4, (30, 20), 32, (2048, 256), torch.float32, True),
    # more fact columns than the wide kernels take: x W_f + b_1 by a dense product, the gathered rows added to it
    ("l512_1_cf12", 3_001, 12, S2_ROWS, 256, (512, 1), torch.float32, True),
    ("l512_64_1_cf33", 2_049, 33, (300, 200), 97, (512, 64, 1), torch.float32, True),
    ("l262_5_cf20_ragged", 1_025, 20, (30, 20), 52, (262, 5), torch.float32, False),
    ("bf16_l1024_1_cf12", 2_049, 12, (100, 200), 44, (1024, 1), torch.bfloat16, True),
    # more tables than the wide kernels take in one go: passes of up to four tables over the activations
    ("bf16_l2048_8_k5_cf16", 1_025, 16, (30, 40, 50, 60, 70), 76, (2048, 8), torch.bfloat16, True),
    ("bf16_l256_16_k8_cf40", 2_049, 40, (30, 40, 50, 60, 70, 80, 90, 100), 104, (256, 16), torch.bfloat16, False),
    ("l1024_64_1_k7_cf12", 1_025, 12, (30, 40, 50, 60, 70, 80, 90), 68, (1024, 64, 1), torch.float32, True),
    ("bf16_l1024_16", 2_049, 0, (100, 200), 32, (1024, 16), torch.bfloat16, True),
    ("bf16_l1024_64_1", 1_025, 4, (100, 200), 32, (1024, 64, 1), torch.bfloat16, False),
]


@pytest.mark.parametrize("shape", LAYERED, ids=[s[0] for s in LAYERED])
def test_wide_models_that_no_fused_kernel_takes(lq, shape):
    """A wide first layer followed by a wide or a third layer: with a workspace (the binding brings one) the join stage
    runs as a linear operator with the ReLU in its store and the later layers as dense products, in chunks of rows;
    without one, and with a workspace of a single 256-row chunk, the same results from the general kernels / from many
    chunks.  All against the oracle."""
    name, n, c_f, rows, k, layers, dt, bias = shape
    cols = _cols(k - c_f, len(rows))
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 4400 + len(name), dtype=dt,
                        w_sigma=_sigmas(k, layers), bias=bias)
    want = _oracle(w)
    w = to_dev(w)
    tol = TOL_BF16 if dt == torch.bfloat16 else TOL_F32
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=dt)
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(Y, want, tol, f"{name}: default workspace")
    es = 2 if dt == torch.bfloat16 else 4
    one_chunk = 256 + 2 * 256 * ((max(layers[:-1]) * es + 15) // 16 * 16)
    Y1 = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=torch.float32,
                                  ws=torch.empty(one_chunk, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert_close(Y1, want, tol, f"{name}: chunks of 256 rows")
    Y0 = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=torch.float32,
                                  ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert_close(Y0, want, tol, f"{name}: no room for activations, general kernels")
    if dt == torch.bfloat16:
        Yb = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)          # Y in bf16
        torch.cuda.synchronize()
        assert Yb.dtype == torch.bfloat16
        assert_close(Yb, want, tol, f"{name}: bf16 output")


@pytest.mark.parametrize("shape", [
    ("linear_l1024_cf20", 2_049, 20, (300, 200), 84, (1024,), torch.float32, True),
    ("linear_l300_cf64", 1_025, 64, (30, 20), 96, (300,), torch.float32, False),
    ("linear_l130_cf17", 4_099, 17, (300, 200, 100), 65, (130,), torch.float32, True),
    ("bf16_linear_l1024_cf12", 1_025, 12, (100, 200), 44, (1024,), torch.bfloat16, True),
    ("bf16_linear_l1024_k6", 1_025, 0, (30, 40, 50, 60, 70, 80), 48, (1024,), torch.bfloat16, True),
    ("linear_l600_k8_cf20", 777, 20, (30, 40, 50, 60, 70, 80, 90, 100), 84, (600,), torch.float32, False),
], ids=lambda s: s[0])
def test_wide_linear_operators_with_many_fact_columns(lq, shape):
    """A linear operator whose fact table brings more columns of its own than the wide kernels take: x W_f + b goes to Y
    by a dense product and the join stage adds the gathered rows to it (Y of the model's type); with Y of another type
    the general kernels run.  Against the oracle."""
    name, n, c_f, rows, k, layers, dt, bias = shape
    cols = _cols(k - c_f, len(rows))
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 4500 + len(name), dtype=dt,
                        w_sigma=_sigmas(k, layers), bias=bias)
    want = _oracle(w)
    w = to_dev(w)
    tol = TOL_BF16 if dt == torch.bfloat16 else TOL_F32
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=dt)
    for yd in ((dt, torch.float32) if dt == torch.bfloat16 else (dt,)):
        Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=yd)
        torch.cuda.synchronize()
        assert_close(Y, want, tol, f"{name}: Y {yd}")
