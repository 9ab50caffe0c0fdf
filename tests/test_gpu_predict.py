"""GPU parity: pre-fusion, fused join+predict and the materialised pipeline against the fp64 oracle.

Bar: fp32 paths within 1e-4, bf16 paths within 2e-2, per element as
|y - want| <= tol * (|want| + rms(want)); foreign-key indexing bit-exact (integer-valued
features and one-hot / small-integer weights make every result exactly representable)."""
import numpy as np
import pytest
import torch

from oracle import lq_oracle as O
from tests.helpers import TOL_BF16, TOL_F32, assert_close, cpu_list, to_dev
from workloads import star as WL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def _oracle(w, nthreads=8):
    return O.join_predict(None if w.X is None else w.X.cpu(), cpu_list(w.dims), cpu_list(w.fks),
                          cpu_list(w.weights), cpu_list(w.biases), nthreads=nthreads)


def _run_fused(lq, w, p_dtype=None, y_dtype=None, flags=0):
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f, p_dtype=p_dtype or w.dtype)
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=y_dtype, flags=flags)
    torch.cuda.synchronize()
    return P, Y


SHAPES = [
    # name, n, c_f, dim_rows, dim_cols, layers, bias
    ("linear_l1", 10_000, 4, (100, 50), (8, 8), (1,), False),
    ("linear_l4_cf8", 5_003, 8, (300, 200), (16, 12), (4,), True),
    ("linear_l64", 3_001, 4, (64, 1000), (8, 8), (64,), True),
    ("linear_l3_odd", 777, 3, (20, 30, 40), (5, 7, 2), (3,), True),
    ("mlp_64_1", 20_037, 4, (1000, 5000, 200), (32, 32, 32), (64, 1), False),
    ("mlp_64_4_bias", 4_099, 4, (100, 50), (8, 8), (64, 4), True),
    ("mlp_32_16_8_generic", 2_050, 5, (30, 7), (6, 3), (32, 16, 8), True),
    ("mlp_100_10", 1_111, 0, (50, 60), (9, 9), (100, 10), True),
    ("no_fact_cols_K1", 4_000, 0, (17,), (11,), (8,), False),
    ("single_row_dims", 1_000, 2, (1, 1), (4, 4), (16, 2), True),
    ("one_fact_row", 1, 4, (10, 10), (8, 8), (64, 1), True),
    ("k8_dims", 3_000, 4, (10,) * 8, (4,) * 8, (16,), False),
    # widths that do not fill a power-of-two lane group, odd fact-column counts (idle lanes, padded c_f)
    ("linear_l2", 4_001, 1, (50, 60), (5, 5), (2,), True),
    ("linear_l6_cf5", 3_003, 5, (50, 60), (5, 5), (6,), False),
    ("linear_l12", 2_002, 4, (50,), (8,), (12,), True),
    ("linear_l100", 1_501, 11, (70, 80), (6, 6), (100,), True),
    ("linear_l50", 1_777, 16, (70, 80), (6, 6), (50,), False),
    ("linear_l37", 1_234, 2, (70, 80), (6, 6), (37,), True),
    ("mlp_24_2_cf3", 2_345, 3, (33, 44), (7, 7), (24, 2), True),
    ("mlp_10_1", 3_210, 7, (33, 44), (7, 7), (10, 1), True),
    ("linear_l128", 1_999, 4, (100, 200), (16, 16), (128,), False),
    ("linear_l256", 1_001, 4, (100, 200), (16, 16), (256,), True),
    # hidden widths 128 / 256 with 1..4 dimensions, 0 / 4 / 8 fact columns, linear and one-output MLP
    ("mlp_128_1_k3", 20_037, 4, (1000, 5000, 200), (32, 32, 32), (128, 1), True),
    ("mlp_256_1_k3", 8_195, 4, (1000, 5000, 200), (32, 32, 32), (256, 1), False),
    ("mlp_128_1_k1_cf0", 4_099, 0, (300,), (20,), (128, 1), True),
    ("mlp_256_1_k4_cf8", 3_333, 8, (50, 60, 70, 80), (6, 6, 6, 6), (256, 1), True),
    ("linear_l128_k4_cf8", 2_817, 8, (50, 60, 70, 80), (6, 6, 6, 6), (128,), True),
    ("linear_l256_k2_cf0", 257, 0, (50, 60), (6, 6), (256,), False),
    ("mlp_128_1_k2_cf8", 641, 8, (50, 60), (6, 6), (128, 1), False),
    # second layers of up to 16 outputs and hidden width 32 in the same kernel family
    ("mlp_32_1_k3", 6_151, 4, (1000, 5000, 200), (32, 32, 32), (32, 1), True),
    ("linear_l32_k2_cf8", 2_051, 8, (50, 60), (6, 6), (32,), False),
    ("mlp_32_8_k4", 3_079, 0, (50, 60, 70, 80), (6, 6, 6, 6), (32, 8), True),
    ("mlp_64_16_k3", 9_001, 4, (1000, 5000, 200), (32, 32, 32), (64, 16), True),
    ("mlp_64_7_k1", 1_283, 8, (90,), (12,), (64, 7), False),
    ("mlp_128_3_k2", 2_311, 4, (50, 60), (6, 6), (128, 3), True),
    ("mlp_128_9_k4_cf8", 1_931, 8, (50, 60, 70, 80), (6, 6, 6, 6), (128, 9), True),
    ("mlp_256_16_k3", 4_111, 0, (100, 200, 300), (16, 16, 16), (256, 16), True),
    ("mlp_256_5_k2", 769, 4, (100, 200), (16, 16), (256, 5), False),
    # fact-column counts that are not whole 16-byte pieces (read one by one, padded with zeros)
    ("mlp_64_1_cf3", 7_001, 3, (1000, 5000, 200), (32, 32, 32), (64, 1), True),
    ("mlp_128_4_cf5", 2_500, 5, (100, 200), (16, 16), (128, 4), False),
    ("linear_l32_cf7", 1_900, 7, (100, 200), (16, 16), (32,), True),
    ("mlp_256_16_cf1", 1_300, 1, (100, 200, 50), (16, 16, 8), (256, 16), True),
    ("mlp_64_8_cf6_k4", 2_222, 6, (50, 60, 70, 80), (6, 6, 6, 6), (64, 8), True),
    # hidden widths that are not 4 x a power of two (idle lanes) and 9..16 fact columns
    ("mlp_48_1_k3", 5_003, 4, (1000, 5000, 200), (32, 32, 32), (48, 1), True),
    ("mlp_200_6_k2_cf12", 2_111, 12, (100, 200), (16, 16), (200, 6), True),
    ("linear_l72_cf16_k3", 1_501, 16, (70, 80, 90), (6, 6, 6), (72,), False),
    ("mlp_20_3_cf9", 3_333, 9, (33, 44), (7, 7), (20, 3), True),
    # five to eight dimension tables
    ("mlp_64_1_k8_cf4", 6_007, 4, (10, 20, 30, 40, 50, 60, 70, 80), (4,) * 8, (64, 1), True),
    ("linear_l128_k5", 2_001, 0, (100, 200, 300, 400, 500), (8,) * 5, (128,), False),
    ("mlp_24_1_k6_cf3", 3_003, 3, (9, 19, 29, 39, 49, 59), (5,) * 6, (24, 1), True),
    ("mlp_256_1_k7", 1_111, 0, (9, 19, 29, 39, 49, 59, 69), (5,) * 7, (256, 1), False),
    # shapes only the tiled matrix-core MLP kernel covers: wide second layers, three layers
    ("mlp_64_10", 5_555, 4, (100, 2_000, 50), (16, 16, 16), (64, 10), True),
    ("mlp_128_16", 3_001, 4, (100, 200), (16, 16), (128, 16), False),
    ("mlp_64_32_1", 4_321, 4, (100, 200), (16, 16), (64, 32, 1), True),
    ("mlp_256_64_8_3", 1_033, 0, (100, 200), (16, 16), (256, 64, 8, 3), True),
    ("mlp_37_5_odd", 2_047, 3, (60, 70), (5, 9), (37, 5), True),
    # deeper / wider fp32 models whose later layers all run on the matrix cores from registers
    ("deep_64_64_1_k3", 9_001, 4, (1000, 5000, 200), (32, 32, 32), (64, 64, 1), True),
    ("deep_32_24_1_k1_cf0", 2_049, 0, (90,), (12,), (32, 24, 1), False),
    ("deep_128_64_5_k4_cf13", 3_001, 13, (50, 60, 70, 80), (6, 6, 6, 6), (128, 64, 5), True),
    ("deep_64_40_k2", 4_111, 4, (100, 200), (16, 16), (64, 40), True),
    ("deep_64_33_k2_odd", 1_237, 2, (100, 200), (16, 16), (64, 33), False),
    ("deep_32_16_16_3", 2_050, 5, (30, 7), (6, 3), (32, 16, 16, 3), True),
    ("deep_64_48_20_1", 5_013, 4, (100, 2_000, 50), (16, 16, 16), (64, 48, 20, 1), True),
    ("deep_128_32_16_k3_cf16", 2_777, 16, (70, 80, 90), (6, 6, 6), (128, 32, 16), True),
    ("deep_one_row", 1, 4, (10, 10), (8, 8), (64, 64, 1), True),
    ("deep_64_128_1", 3_003, 4, (100, 200), (16, 16), (64, 128, 1), True),
    ("deep_128_100_k2", 1_501, 0, (100, 200), (16, 16), (128, 100), False),
    ("deep_32_96_72_4", 2_222, 3, (60, 70), (5, 9), (32, 96, 72, 4), True),
    # hidden widths that do not fill the padded lane group
    ("deep_48_32_1", 2_345, 4, (100, 200, 50), (16, 16, 8), (48, 32, 1), True),
    ("deep_100_24", 1_999, 0, (100, 200), (16, 16), (100, 24), False),
    ("deep_20_20_20_2", 1_500, 2, (30, 7), (6, 3), (20, 20, 20, 2), True),
    # hidden widths above 128: gathered and fed to the second layer in two column parts
    ("deep_256_64_8_1_k3", 3_001, 4, (1000, 5000, 200), (32, 32, 32), (256, 64, 8, 1), True),
    ("deep_256_16_k4_cf8", 2_049, 8, (50, 60, 70, 80), (6, 6, 6, 6), (256, 16), True),
    ("deep_200_40_3_k1", 1_111, 0, (90,), (12,), (200, 40, 3), False),
    ("deep_132_128_k2", 777, 3, (100, 200), (16, 16), (132, 128), True),
    # five to eight dimension tables (the fifth and later ones are gathered inside the step)
    ("deep_64_64_1_k5", 4_099, 4, (100, 200, 50, 70, 90), (8, 8, 8, 8, 8), (64, 64, 1), True),
    ("deep_128_32_1_k6_cf0", 2_345, 0, (100, 200, 50, 70, 90, 30), (6,) * 6, (128, 32, 1), False),
    ("deep_256_16_k8", 1_501, 3, (10, 20, 30, 40, 50, 60, 70, 80), (4,) * 8, (256, 16), True),
    ("deep_40_24_k7", 1_111, 1, (10, 20, 30, 40, 50, 60, 70), (4,) * 7, (40, 24), True),
    # 17 to 64 fact columns
    ("deep_64_64_1_cf20", 3_003, 20, (100, 200, 50), (8, 8, 8), (64, 64, 1), True),
    ("deep_128_24_cf64_k1", 1_777, 64, (90,), (12,), (128, 24), False),
    ("deep_32_32_3_cf37", 2_222, 37, (60, 70), (5, 9), (32, 32, 3), True),
    # more than 16 outputs after three or four layers
    ("deep_64_32_64", 2_345, 4, (100, 200, 50), (16, 16, 8), (64, 32, 64), True),
    ("deep_128_16_100_k2", 1_501, 0, (100, 200), (16, 16), (128, 16, 100), False),
    ("deep_32_48_24_40", 2_222, 3, (60, 70), (5, 9), (32, 48, 24, 40), True),
    # five to eight layers
    ("deep_six_layers", 2_345, 4, (100, 200, 50), (16, 16, 8), (64, 48, 32, 32, 16, 3), True),
    ("deep_eight_layers_256", 1_501, 0, (100, 200), (16, 16), (256, 24, 20, 16, 12, 10, 8, 1), True),
    # the limits of the interface: 8 layers, 8 dimensions
    ("eight_layers_eight_dims", 1_500, 2, (9,) * 8, (3,) * 8, (24, 20, 16, 12, 10, 8, 6, 2), True),
]


@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_fused_matches_oracle_fp32(lq, shape):
    name, n, c_f, rows, cols, layers, bias = shape
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 1000 + len(name),
                        w_sigma=[0.3] * len(layers), bias=bias)
    want = _oracle(w)
    w = to_dev(w)
    P, Y = _run_fused(lq, w)
    Pw = O.project_dims(cpu_list(w.dims), w.weights[0].cpu(), w.c_f)
    for k in range(len(P)):
        assert_close(P[k], Pw[k], TOL_F32, f"{name}: P[{k}]")
    assert_close(Y, want, TOL_F32, f"{name}: fused")
    # the shape-agnostic kernel must agree with whichever kernel the dispatcher picked
    _, Yg = _run_fused(lq, w, flags=lq.LQ_FORCE_GENERIC)
    assert_close(Yg, want, TOL_F32, f"{name}: generic kernel")
    _, Yt = _run_fused(lq, w, flags=lq.LQ_FORCE_TILE)
    assert_close(Yt, want, TOL_F32, f"{name}: tile kernel")
    # the non-fused pipeline computes the same function
    Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases, chunk_rows=1024)
    torch.cuda.synchronize()
    assert_close(Ym, want, TOL_F32, f"{name}: materialised")


def test_config1_tiny_linear_regression(lq):
    w = WL.c1_tiny_linear()
    want = _oracle(w)
    w = to_dev(w)
    _, Y = _run_fused(lq, w)
    assert_close(Y, want, TOL_F32, "config 1")


def test_fk_indexing_is_bit_exact_fp32(lq):
    """Integer-valued features and weights: every partial sum is an integer far below 2^24,
    so fp32 must reproduce the fp64 oracle exactly, for the fused and the materialised path."""
    for layers in ((4,), (64,), (64, 1), (16, 4)):
        w = WL.make_predict("exact", 6_011, 4, (97, 1_013, 31), (8, 4, 8), layers,
                            seed=WL.SEED0 + 77, integer_valued=True, bias=True)
        want = _oracle(w)
        assert np.abs(want).max() < 2 ** 22
        w = to_dev(w)
        _, Y = _run_fused(lq, w)
        np.testing.assert_array_equal(Y.cpu().double().numpy(), want)
        Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases, chunk_rows=2048)
        np.testing.assert_array_equal(Ym.cpu().double().numpy(), want)


def test_one_hot_weights_make_the_output_a_pure_gather(lq):
    w = WL.make_predict("gather", 5_000, 2, (50, 70), (3, 4), (4,), seed=WL.SEED0 + 78)
    W = torch.zeros((9, 4))
    for o, s in enumerate([8, 0, 3, 6]):
        W[s, o] = 1
    w.weights = [W]
    want = torch.stack([w.dims[1][w.fks[1].long(), 3], w.X[:, 0], w.dims[0][w.fks[0].long(), 1],
                        w.dims[1][w.fks[1].long(), 1]], dim=1)
    w = to_dev(w)
    _, Y = _run_fused(lq, w)
    assert torch.equal(Y.cpu(), want)


def test_all_keys_equal_and_strided_inputs(lq):
    w = WL.make_predict("strided", 2_500, 4, (40, 60), (8, 8), (64, 1), seed=WL.SEED0 + 79,
                        w_sigma=(0.2, 0.2))
    w.fks = [torch.full((2_500,), 7, dtype=torch.int32), torch.full((2_500,), 59, dtype=torch.int32)]
    want = _oracle(w)
    w = to_dev(w)
    # X, a dimension table and Y as column slices of wider buffers (ld > cols, unaligned rows)
    Xw = torch.zeros((2_500, 7), device="cuda"); Xw[:, 1:5] = w.X
    Dw = torch.zeros((40, 11), device="cuda"); Dw[:, 3:11] = w.dims[0]
    Yw = torch.full((2_500, 3), -1.0, device="cuda")
    P = lq.lq_project_dims([Dw[:, 3:11], w.dims[1]], w.weights[0], 4)
    lq.lq_fused_join_predict(Xw[:, 1:5], w.fks, P, w.weights, Y=Yw[:, 1:2])
    torch.cuda.synchronize()
    assert_close(Yw[:, 1:2], want, TOL_F32, "strided fused")
    assert (Yw[:, 0] == -1).all() and (Yw[:, 2] == -1).all()     # neighbours untouched
    Ym = lq.lq_materialized_join_predict(Xw[:, 1:5], [Dw[:, 3:11], w.dims[1]], w.fks, w.weights)
    torch.cuda.synchronize()
    assert_close(Ym, want, TOL_F32, "strided materialised")


@pytest.mark.parametrize("layers,dtype", [((64, 48, 1), torch.float32), ((200, 24), torch.float32),
                                          ((64, 12), torch.float32), ((96, 40, 3), torch.bfloat16)],
                         ids=["f32_64_48_1", "f32_200_24", "f32_64_12", "bf16_96_40_3"])
def test_deeper_models_with_strided_inputs(lq, layers, dtype):
    """The matrix-core kernels for deeper models on operands that are column slices of wider buffers:
    X, the projected tables (row stride > l_1), the weights of the later layers and Y."""
    n, c_f = 3_001, 4
    w = WL.make_predict("deep_strided", n, c_f, (300, 200), (16, 16), layers, seed=WL.SEED0 + 90,
                        dtype=dtype, w_sigma=[0.15] * len(layers), bias=True)
    want = _oracle(w)
    w = to_dev(w)
    tol = TOL_F32 if dtype == torch.float32 else TOL_BF16
    pad = 8                                          # keeps 16-byte alignment of the slices for both dtypes
    Xw = torch.zeros((n, c_f + 3), dtype=dtype, device="cuda"); Xw[:, 2:2 + c_f] = w.X
    P = []
    for d in w.dims:
        buf = torch.zeros((d.shape[0], layers[0] + 2 * pad), dtype=dtype, device="cuda")
        P.append(buf[:, pad:pad + layers[0]])
    lq.lq_project_dims(w.dims, w.weights[0], c_f, P=P)
    weights = [w.weights[0]]
    for W in w.weights[1:]:
        buf = torch.zeros((W.shape[0], W.shape[1] + 5), dtype=dtype, device="cuda")
        buf[:, 2:2 + W.shape[1]] = W
        weights.append(buf[:, 2:2 + W.shape[1]])
    Yw = torch.full((n, layers[-1] + 3), -1.0, dtype=dtype, device="cuda")
    Y = Yw[:, 1:1 + layers[-1]]
    lq.lq_fused_join_predict(Xw[:, 2:2 + c_f], w.fks, P, weights, w.biases, Y=Y)
    torch.cuda.synchronize()
    assert_close(Y, want, tol, "strided deep model")
    assert (Yw[:, 0] == -1).all() and (Yw[:, 1 + layers[-1]:] == -1).all()      # neighbours untouched
    for buf in P:
        assert (buf._base[:, :pad] == 0).all() and (buf._base[:, pad + layers[0]:] == 0).all()


LDS_LINEAR = [
    # name, c_f, dim_rows, dim_cols, outputs, bias; above 2^20 fact rows the small projected tables of
    # such models are kept in LDS, larger ones (here: 100,000 / 40,000 rows) are gathered from memory
    ("l1_c2_star", 4, (1_000, 10_000, 100_000), (32, 32, 32), 1, True),
    ("l1_four_tables_no_fact_columns", 0, (2_556, 30_000, 2_000, 200), (8, 8, 8, 8), 1, False),
    ("l1_one_table_cf3", 3, (5_000,), (6,), 1, True),
    ("l1_cf8", 8, (300, 36_000), (5, 5), 1, True),
    ("l1_six_tables", 4, (100, 2_000, 300, 5_000, 40, 90_000), (3, 4, 5, 6, 7, 8), 1, True),
    ("l1_eight_tables_no_fact_columns", 0, (10, 20, 30, 40, 50, 60, 70, 8_000), (2, 2, 2, 2, 2, 2, 2, 2), 1, False),
    ("l2_two_tables_cf5", 5, (1_000, 17_000), (16, 16), 2, True),
    ("l2_four_tables", 4, (100, 200, 300, 40_000), (4, 4, 4, 4), 2, False),
    ("l4_three_tables", 4, (1_000, 8_000, 100_000), (8, 8, 8), 4, True),
    ("l4_cf7_one_table_fits_exactly", 7, (9_984, 40_000), (6, 6), 4, True),
]


@pytest.mark.parametrize("shape", LDS_LINEAR, ids=[s[0] for s in LDS_LINEAR])
def test_linear_models_with_lds_resident_tables(lq, shape):
    name, c_f, rows, cols, l, bias = shape
    n = (1 << 20) + 2_777                                 # ends inside a workgroup's last step
    w = WL.make_predict(name, n, c_f, rows, cols, (l,), seed=WL.SEED0 + 95, bias=bias)
    want = _oracle(w, nthreads=16)
    w = to_dev(w)
    P, Y = _run_fused(lq, w)
    assert_close(Y, want, TOL_F32, name)
    _, Yg = _run_fused(lq, w, flags=lq.LQ_FORCE_GENERIC)  # the shape-agnostic kernel on the same inputs
    assert_close(Yg, want, TOL_F32, name + " (generic kernel)")
    # operands that are column slices of wider buffers: X and Y keep the kernel (scalar loads / stores),
    # a projected table with a row stride other than l stays in memory
    Yw = torch.full((n, l + 3), -1.0, device="cuda")
    Xs = None
    if c_f:
        Xw = torch.zeros((n, c_f + 1), device="cuda"); Xw[:, 1:] = w.X
        Xs = Xw[:, 1:]
    buf = torch.zeros((rows[0], 2 * l), device="cuda"); buf[:, l:] = P[0]
    Ps = [buf[:, l:]] + list(P[1:])
    lq.lq_fused_join_predict(Xs, w.fks, Ps, w.weights, w.biases, Y=Yw[:, 2:2 + l])
    torch.cuda.synchronize()
    assert_close(Yw[:, 2:2 + l], want, TOL_F32, name + " (strided)")
    assert (Yw[:, :2] == -1).all() and (Yw[:, 2 + l:] == -1).all()


def test_bf16_paths(lq):
    for name, c_f, layers in (("bf16_linear", 8, (8,)), ("bf16_mlp", 0, (64, 4)), ("bf16_mlp16", 4, (256, 16))):
        w = WL.make_predict(name, 6_007, c_f, (300, 1_000), (32, 64), layers, seed=WL.SEED0 + 80,
                            dtype=torch.bfloat16, w_sigma=[0.1] * len(layers), bias=True)
        want = _oracle(w)
        w = to_dev(w)
        for p_dtype, y_dtype in ((torch.bfloat16, torch.bfloat16), (torch.float32, torch.float32),
                                 (torch.bfloat16, torch.float32)):
            P, Y = _run_fused(lq, w, p_dtype=p_dtype, y_dtype=y_dtype)
            assert Y.dtype == y_dtype and P[0].dtype == p_dtype
            assert_close(Y, want, TOL_BF16, f"{name} P {p_dtype} Y {y_dtype}")
        Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases)
        torch.cuda.synchronize()
        assert_close(Ym, want, TOL_BF16, f"{name} materialised")


BF16_MFMA_SHAPES = [
    # name, n, dim_rows, dim_cols, layers, bias[, c_f]   (the matrix-core epilogue kernel)
    ("bf16_256_16", 5_003, (500, 700, 300, 900), (64, 64, 32, 48), (256, 16), False),
    ("bf16_128_10_bias", 3_001, (100, 200), (32, 40), (128, 10), True),
    ("bf16_32_1", 2_047, (50,), (16,), (32, 1), True),
    ("bf16_linear_256", 1_999, (64, 80, 96), (24, 24, 24), (256,), True),
    ("bf16_linear_64", 4_100, (64, 80), (24, 24), (64,), False),
    # with fact columns (a seventh entry): x W_f is added in the same kernel
    ("bf16_64_1_cf4", 6_011, (1000, 5000, 200), (32, 32, 32), (64, 1), True, 4),
    ("bf16_256_16_cf3", 2_111, (300, 200), (32, 32), (256, 16), False, 3),
    ("bf16_linear_128_cf16", 1_777, (64, 80), (24, 24), (128,), True, 16),
    ("bf16_32_8_cf1", 3_001, (70,), (9,), (32, 8), True, 1),
    # one to four outputs or a linear operator: the lane-group form with eight columns per lane
    ("bf16_64_1_k3", 20_037, (1000, 5000, 200), (32, 32, 32), (64, 1), True),
    ("bf16_128_2_cf5", 2_311, (50, 60), (6, 6), (128, 2), True, 5),
    ("bf16_256_4_k4", 3_001, (50, 60, 70, 80), (6, 6, 6, 6), (256, 4), False, 4),
    ("bf16_512_3_k1", 1_025, (90,), (12,), (512, 3), True),
    ("bf16_linear_512_cf8", 777, (64, 80), (24, 24), (512,), True, 8),
    ("bf16_linear_128_k4_cf8", 1_301, (50, 60, 70, 80), (6, 6, 6, 6), (128,), False, 8),
    ("bf16_96_1_k2", 2_049, (100, 200), (16, 16), (96, 1), True, 4),
    ("bf16_linear_40", 1_111, (100, 200), (16, 16), (40,), False),
    # 9 to 16 fact columns on the one-tile kernel (their rows of W_0 staged in LDS); two layers with 5 to 16 outputs and
    # fact columns, or a first layer of another width than 32 / 64 / 128 / 256, on the kernel for deeper models
    ("bf16_linear_256_cf12", 2_003, (64, 80, 96), (24, 24, 24), (256,), True, 12),
    ("bf16_64_3_cf12", 3_001, (100, 200), (16, 16), (64, 3), True, 12),
    ("bf16_128_9_cf12", 1_999, (100, 200), (16, 16), (128, 9), False, 12),
    ("bf16_200_16", 2_311, (100, 200, 50), (16, 16, 8), (200, 16), True),
    ("bf16_72_9_cf5", 1_025, (90, 70), (12, 12), (72, 9), True, 5),
    # deeper / wider bf16 models: later layers chained on the matrix cores
    ("bf16_deep_256_64_16", 3_001, (500, 700, 300, 900), (64, 64, 32, 48), (256, 64, 16), True),
    ("bf16_deep_64_64_1_cf4", 4_099, (1000, 5000, 200), (32, 32, 32), (64, 64, 1), True, 4),
    ("bf16_deep_128_40", 2_049, (100, 200), (32, 40), (128, 40), False),
    ("bf16_deep_32_24_8_3_cf2", 1_777, (64, 80), (24, 24), (32, 24, 8, 3), True, 2),
    ("bf16_deep_256_48_5_k1", 1_025, (90,), (12,), (256, 48, 5), False),
    ("bf16_deep_128_16_16_2", 2_000, (100, 200), (16, 16), (128, 16, 16, 2), True),
    ("bf16_deep_256_256_16", 2_049, (500, 700, 300, 900), (64, 64, 32, 48), (256, 256, 16), True),
    ("bf16_deep_64_100", 1_333, (100, 200), (32, 40), (64, 100), False),
    ("bf16_deep_96_200_130_7_cf3", 1_111, (64, 80), (24, 24), (96, 200, 130, 7), True, 3),
    ("bf16_deep_40_24_1", 1_777, (64, 80), (24, 24), (40, 24, 1), True, 5),
    ("bf16_deep_200_64", 1_025, (90, 70), (12, 12), (200, 64), False),
    ("bf16_deep_8_8_8", 999, (33,), (7,), (8, 8, 8), True),
    ("bf16_deep_five_layers", 2_049, (100, 200, 50), (16, 16, 8), (128, 64, 64, 32, 2), True, 4),
    ("bf16_deep_64_32_1_cf40", 1_501, (100, 200), (16, 16), (64, 32, 1), True, 40),
    ("bf16_deep_64_32_64", 2_049, (100, 200, 50), (16, 16, 8), (64, 32, 64), True, 4),
    ("bf16_deep_256_64_200", 1_025, (90, 70), (12, 12), (256, 64, 200), False),
]


@pytest.mark.parametrize("shape", BF16_MFMA_SHAPES, ids=[s[0] for s in BF16_MFMA_SHAPES])
def test_bf16_wide_models(lq, shape):
    name, n, rows, cols, layers, bias = shape[:6]
    c_f = shape[6] if len(shape) > 6 else 0
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 300 + len(name),
                        dtype=torch.bfloat16, w_sigma=[1.0 / np.sqrt(sum(cols))] + [0.1] * (len(layers) - 1),
                        bias=bias)
    want = _oracle(w)
    w = to_dev(w)
    for y_dtype in (torch.bfloat16, torch.float32):
        P, Y = _run_fused(lq, w, p_dtype=torch.bfloat16, y_dtype=y_dtype)
        assert_close(Y, want, TOL_BF16, f"{name} Y {y_dtype}")
    _, Yg = _run_fused(lq, w, p_dtype=torch.bfloat16, y_dtype=torch.float32, flags=lq.LQ_FORCE_GENERIC)
    assert_close(Yg, want, TOL_BF16, f"{name} generic")
    _, Yt = _run_fused(lq, w, p_dtype=torch.bfloat16, y_dtype=torch.bfloat16, flags=lq.LQ_FORCE_TILE)
    assert_close(Yt, want, TOL_BF16, f"{name} tile")


def test_bf16_matrix_core_epilogue_is_exact_on_small_integers(lq):
    """Integer features/weights small enough that every hidden unit and output is an exactly
    representable bf16 / fp32 integer: the MFMA path must reproduce the oracle bit for bit."""
    w = WL.make_predict("bf16_mfma_exact", 3_333, 0, (40, 50), (4, 4), (32, 16), seed=WL.SEED0 + 82,
                        dtype=torch.bfloat16, integer_valued=True, bias=True)
    want = _oracle(w)                       # |z| <= 8*4*2+2 = 66, |y| <= 32*66*2+2 < 2^13
    w = to_dev(w)
    _, Y = _run_fused(lq, w, p_dtype=torch.bfloat16, y_dtype=torch.float32)
    np.testing.assert_array_equal(Y.cpu().double().numpy(), want)


def test_bf16_fk_indexing_is_bit_exact(lq):
    """Small integers are exact in bf16; with one-hot-like integer weights the bf16 path must
    return exactly the oracle's integers (|values| <= 256 stay representable)."""
    w = WL.make_predict("bf16_exact", 4_001, 0, (50, 60), (8, 8), (8,), seed=WL.SEED0 + 81,
                        dtype=torch.bfloat16, integer_valued=True)
    want = _oracle(w)
    assert np.abs(want).max() <= 256
    w = to_dev(w)
    _, Y = _run_fused(lq, w)
    np.testing.assert_array_equal(Y.float().cpu().double().numpy(), want)


def test_empty_fact_table(lq):
    w = to_dev(WL.make_predict("empty", 0, 4, (10,), (4,), (8, 2), seed=1))
    P, Y = _run_fused(lq, w)
    assert Y.shape == (0, 2)
    Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases)
    assert Ym.shape == (0, 2)


def test_check_fks_flag(lq):
    w = to_dev(WL.make_predict("fkcheck", 5_000, 4, (10, 20), (4, 4), (8,), seed=2))
    P = lq.lq_project_dims(w.dims, w.weights[0], 4)
    Y0 = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, flags=lq.LQ_CHECK_FKS)
    torch.cuda.synchronize()
    bad = [w.fks[0], w.fks[1].clone()]
    bad[1][4_321] = 20
    Y = torch.full_like(Y0, 7.0)
    with pytest.raises(lq.LQError) as e:
        lq.lq_fused_join_predict(w.X, bad, P, w.weights, Y=Y, flags=lq.LQ_CHECK_FKS)
    assert e.value.status == "LQ_ERR_FK_RANGE"
    torch.cuda.synchronize()
    assert (Y == 7.0).all()                                  # outputs untouched on error
    bad[1][4_321] = -1
    with pytest.raises(lq.LQError):
        lq.lq_materialized_join_predict(w.X, w.dims, bad, w.weights, flags=lq.LQ_CHECK_FKS)


def test_materialised_chunking_does_not_change_results(lq):
    w = WL.make_predict("chunks", 10_001, 4, (100, 300), (16, 16), (32, 2), seed=3, w_sigma=(0.2, 0.2))
    want = _oracle(w)
    w = to_dev(w)
    for chunk in (256, 1_024, 16_384):
        Y = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, chunk_rows=chunk)
        torch.cuda.synchronize()
        assert_close(Y, want, TOL_F32, f"chunk {chunk}")


def test_incremental_prefusion_refreshes_only_the_given_rows(lq):
    for layers, rows in (((64, 1), (1_000, 5_003)), ((4,), (300, 2_001))):
        w = WL.make_predict("incr", 100, 4, rows, (32, 24), layers, seed=WL.SEED0 + 90, w_sigma=[0.2] * len(layers))
        w = to_dev(w)
        P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
        before = [p.clone() for p in P]
        lo, cnt = 701, 1_003
        w.dims[1][lo:lo + cnt] += 1.5                      # these dimension rows change
        lq.lq_project_dim_rows(w.dims, w.weights[0], w.c_f, P, 1, lo, cnt)
        full = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
        torch.cuda.synchronize()
        assert torch.equal(P[0], before[0]) and torch.equal(P[1], full[1])
        assert torch.equal(P[1][:lo], before[1][:lo]) and torch.equal(P[1][lo + cnt:], before[1][lo + cnt:])
        assert not torch.equal(P[1][lo:lo + cnt], before[1][lo:lo + cnt])
        Pw = O.project_dims(cpu_list(w.dims), w.weights[0].cpu(), w.c_f)
        assert_close(P[1], Pw[1], TOL_F32, "refreshed table")
        with pytest.raises(lq.LQError):
            lq.lq_project_dim_rows(w.dims, w.weights[0], w.c_f, P, 1, rows[1] - 5, 6)


@pytest.mark.parametrize("shape", [
    # name, fact rows, fact columns, dimension rows, dimension columns, layers, bias
    ("tall_k100_64_1", 300_007, 4, (1_000, 10_000, 500), (32, 32, 32), (64, 1), True),
    ("tall_k37_40", 280_001, 5, (300, 200), (16, 16), (40,), False),          # k and the width not multiples of 4
    ("tall_k255_17_3", 270_013, 0, (400, 300, 200), (85, 85, 85), (17, 3), True),
], ids=lambda s: s[0])
def test_non_fused_first_layer_over_many_rows(lq, shape):
    """The non-fused pipeline with all rows in one chunk (a few hundred thousand rows, at most 64 columns, short k:
    thousands of tiles of the dense first layer in one launch); compared with the oracle on a row sample that holds
    both ends and a stride through the middle."""
    name, n, c_f, rows, cols, layers, bias = shape
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 700 + len(name), device="cuda",
                        w_sigma=[1.0 / np.sqrt(c_f + sum(cols))] + [1.0 / np.sqrt(a) for a in layers[:-1]], bias=bias)
    Ym = lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases, chunk_rows=n)
    torch.cuda.synchronize()
    sample = torch.cat([torch.arange(0, 4_096), torch.arange(4_096, n - 4_096, 257), torch.arange(n - 4_096, n)])
    sub = WL.take_rows(w, sample.to("cuda"))
    want = O.join_predict(None if sub.X is None else sub.X.cpu(), cpu_list(sub.dims), cpu_list(sub.fks), cpu_list(sub.weights),
                          cpu_list(sub.biases), nthreads=16)
    assert_close(Ym[sample.to("cuda")], want, TOL_F32, f"{name}: non-fused, one chunk")


@pytest.mark.parametrize("shape", [
    # name, fact rows, fact columns, dimension rows, dimension columns, layers, bias
    ("w50_1", 20_011, 4, (300, 200, 100), (8, 8, 8), (50, 1), True),
    ("w30_4", 4_099, 3, (300, 200), (8, 8), (30, 4), False),
    ("w102_1_k5", 3_001, 0, (50, 60, 70, 80, 90), (4, 4, 4, 4, 4), (102, 1), True),
    ("w50_linear", 20_011, 4, (300, 200, 100), (8, 8, 8), (50,), True),
    ("w22_linear_one_row_table", 1_025, 0, (1, 40), (8, 8), (22,), False),
    ("w250_13", 2_049, 8, (300, 200), (8, 8), (250, 13), True),
    ("w50_10", 20_011, 4, (300, 200, 100), (8, 8, 8), (50, 10), True),        # matrix-core kernel
    ("w50_30_1", 20_011, 4, (300, 200, 100), (8, 8, 8), (50, 30, 1), True),
    ("w130_64_7_k6", 3_003, 5, (30, 40, 50, 60, 70, 80), (4, 4, 4, 4, 4, 4), (130, 64, 7), False),   # two column parts, six tables
    ("w254_100", 1_111, 0, (100,), (16,), (254, 100), True),
    ("w262_1", 2_049, 4, (300, 200), (8, 8), (262, 1), True),                 # column-tiled kernel
    ("w1001_linear", 1_025, 0, (100, 50), (8, 8), (1_001,), False),
    ("w770_7_k5", 777, 3, (30, 40, 50, 60, 70), (4, 4, 4, 4, 4), (770, 1), True),
    ("w13_1", 20_011, 4, (300, 200, 100), (8, 8, 8), (13, 1), True),          # 12..16 columns: the row-batch kernel too
    ("w16_2", 20_011, 0, (300, 200), (8, 8), (16, 2), False),
], ids=lambda s: s[0])
def test_hidden_widths_that_are_not_multiples_of_four(lq, shape):
    """fp32 first layers of any width: with the row stride of the projected tables padded to four floats (what the
    binding allocates) the row-batch and matrix-core kernels take them, the last 16-byte piece of a row ending in the
    padding, which is filled with NaN here and must not reach the result; with contiguous tables (rows not 16-byte
    aligned) the general kernels run.  Both against the oracle."""
    name, n, c_f, rows, cols, layers, bias = shape
    k = c_f + sum(cols)
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 800 + len(name), device="cuda",
                        w_sigma=[1.0 / np.sqrt(k)] + [1.0 / np.sqrt(a) for a in layers[:-1]], bias=bias)
    want = _oracle(w)
    l1 = layers[0]
    ld = (l1 + 3) // 4 * 4
    padded = []
    for d in w.dims:
        buf = torch.full((d.shape[0], ld), float("nan"), device="cuda")
        padded.append(buf[:, :l1])
    lq.lq_project_dims(w.dims, w.weights[0], w.c_f, P=padded)
    Y = lq.lq_fused_join_predict(w.X, w.fks, padded, w.weights, w.biases)
    torch.cuda.synchronize()
    assert_close(Y, want, TOL_F32, f"{name}: padded row stride")
    for buf in padded:                                   # the padding is untouched
        assert torch.isnan(buf.as_strided((buf.shape[0], ld - l1), (ld, 1), buf.storage_offset() + l1)).all()
    P = [torch.empty((d.shape[0], l1), device="cuda") for d in w.dims]
    lq.lq_project_dims(w.dims, w.weights[0], w.c_f, P=P)
    Yc = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases)
    torch.cuda.synchronize()
    assert_close(Yc, want, TOL_F32, f"{name}: contiguous tables")
    if len(layers) == 1:                                 # a linear model into a column slice of a wider, misaligned buffer
        Yw = torch.full((n, l1 + 3), -7.0, device="cuda")
        lq.lq_fused_join_predict(w.X, w.fks, padded, w.weights, w.biases, Y=Yw[:, 1:1 + l1])
        torch.cuda.synchronize()
        assert_close(Yw[:, 1:1 + l1], want, TOL_F32, f"{name}: misaligned Y")
        assert (Yw[:, 0] == -7).all() and (Yw[:, 1 + l1:] == -7).all()


@pytest.mark.parametrize("shape", [
    ("bf16_w44_1", 4_099, 4, (300, 200, 100), (8, 8, 8), (44, 1), True),
    ("bf16_w100_4", 4_099, 0, (300, 200), (8, 8), (100, 4), False),
    ("bf16_w100_linear", 2_049, 4, (300, 200), (8, 8), (100,), True),
    ("bf16_w500_2", 1_025, 8, (100, 50), (8, 8), (500, 2), True),
    ("bf16_w1001_1", 1_025, 0, (100, 50), (8, 8), (1_001, 1), True),          # column-tiled kernel
], ids=lambda s: s[0])
def test_bf16_hidden_widths_that_are_not_multiples_of_eight(lq, shape):
    """The same for bf16 models (16-byte pieces of eight values): row stride padded to eight values, the padding filled
    with NaN; then contiguous tables (general kernels).  Y in bf16 and in fp32."""
    name, n, c_f, rows, cols, layers, bias = shape
    k = c_f + sum(cols)
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 850 + len(name), device="cuda", dtype=torch.bfloat16,
                        w_sigma=[1.0 / np.sqrt(k)] + [1.0 / np.sqrt(a) for a in layers[:-1]], bias=bias)
    want = _oracle(w)
    l1 = layers[0]
    ld = (l1 + 7) // 8 * 8
    padded = [torch.full((d.shape[0], ld), float("nan"), device="cuda", dtype=torch.bfloat16)[:, :l1] for d in w.dims]
    lq.lq_project_dims(w.dims, w.weights[0], w.c_f, P=padded)
    for yd in (torch.bfloat16, torch.float32):
        Y = lq.lq_fused_join_predict(w.X, w.fks, padded, w.weights, w.biases, y_dtype=yd)
        torch.cuda.synchronize()
        assert_close(Y, want, TOL_BF16, f"{name}: padded row stride, Y {yd}")
    P = [torch.empty((d.shape[0], l1), device="cuda", dtype=torch.bfloat16) for d in w.dims]
    lq.lq_project_dims(w.dims, w.weights[0], w.c_f, P=P)
    Yc = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, y_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(Yc, want, TOL_BF16, f"{name}: contiguous tables")


@pytest.mark.parametrize("shape", [
    ("w64_200", 4_099, 4, (300, 200, 100), (8, 8, 8), (64, 200), True),
    ("w64_256_1", 2_049, 0, (300, 200), (8, 8), (64, 256, 1), False),
    ("w30_130_7_ragged_k6", 1_025, 5, (30, 40, 50, 60, 70, 80), (4, 4, 4, 4, 4, 4), (30, 130, 7), True),
    ("w64_256_256_3", 777, 20, (100,), (16,), (64, 256, 256, 3), True),
    ("w16_129", 63, 1, (10, 20), (3, 3), (16, 129), False),
], ids=lambda s: s[0])
def test_later_layers_of_129_to_256_units_next_to_narrow_first_layers(lq, shape):
    """First layers of up to 64 columns followed by layers of 129 .. 256 units: sixteen 16-unit tiles per later layer
    on the matrix-core kernel.  Against the oracle."""
    name, n, c_f, rows, cols, layers, bias = shape
    k = c_f + sum(cols)
    w = WL.make_predict(name, n, c_f, rows, cols, layers, seed=WL.SEED0 + 900 + len(name), device="cuda",
                        w_sigma=[1.0 / np.sqrt(k)] + [1.0 / np.sqrt(a) for a in layers[:-1]], bias=bias)
    want = _oracle(w)
    P = lq.lq_project_dims(w.dims, w.weights[0], w.c_f)
    Y = lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert_close(Y, want, TOL_F32, name)
