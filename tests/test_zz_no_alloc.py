"""The allocation-free group-by entry point against the workspace-taking one: same results, bit for bit,
on two calls in a row that share the library's static scratch array, the second with a smaller input
(what the first call left in the array must not leak into the second).  Both are also compared with the
oracle.  Collected last so that a failure here hides no other test."""
import ctypes

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


def _both(lq, w):
    """(static sums, counts), (workspace sums, counts), (oracle sums, counts) for one workload."""
    want = O.groupby_sum(cpu_list(w.fks), w.dim_rows, cpu_list(w.dim_mask), cpu_list(w.dim_code),
                         w.group_card, None if w.fact_mask is None else w.fact_mask.cpu(),
                         cpu_list(w.measures), nthreads=8)
    w = to_dev(w)
    G = int(np.prod([c for c, code in zip(w.group_card, w.dim_code) if code is not None] or [1]))
    sums = torch.full((len(w.measures), G), -7, dtype=torch.int64, device="cuda")
    counts = torch.full((G,), -7, dtype=torch.int64, device="cuda")
    lq.lq_masked_groupby_sum_static(w.fks, w.dim_rows, w.dim_mask, w.dim_code, w.group_card, w.fact_mask,
                                    w.measures, sums, counts)
    ref_s, ref_c = lq.lq_masked_groupby_sum(w.fks, w.dim_rows, w.dim_mask, w.dim_code, w.group_card,
                                            w.fact_mask, w.measures)
    torch.cuda.synchronize()
    return (sums.cpu().numpy(), counts.cpu().numpy()), (ref_s.cpu().numpy(), ref_c.cpu().numpy()), want


def test_static_scratch_two_calls_in_a_row(lq):
    assert lq.lq_static_scratch_bytes() == 8 << 20
    # first call: the full-size star-schema aggregate; second: a small, ragged one with other tables
    big = WL.c3_groupby(variant="A")
    r = np.random.default_rng(77)
    n, rows, card = 4_099, (7, 300, 5, 1300), (3, 4, 1, 1)
    small = WL.GroupByWorkload(
        "small", n, [torch.from_numpy(r.integers(0, a, size=n).astype(np.int32)) for a in rows], list(rows),
        [None] + [torch.from_numpy((r.random(a) < 0.6).astype(np.uint8)) for a in rows[1:]],
        [torch.from_numpy(r.integers(0, card[k], size=rows[k]).astype(np.int32)) if card[k] > 1 else None
         for k in range(4)], list(card), torch.from_numpy((r.random(n) < 0.9).astype(np.uint8)),
        [torch.from_numpy(r.integers(-100_000, 100_001, size=n).astype(np.int32)) for _ in range(2)])
    for w in (big, small):
        (s, c), (rs, rc), (ws, wc) = _both(lq, w)
        np.testing.assert_array_equal(s, rs)
        np.testing.assert_array_equal(c, rc)
        np.testing.assert_array_equal(s, ws)
        np.testing.assert_array_equal(c, wc)


def test_static_scratch_refuses_what_does_not_fit(lq):
    # 6 million dimension rows need more side-table room than the static array has: a clear error,
    # nothing enqueued.  Only sizes are read before the refusal, so tiny tensors stand in for the columns.
    fk = torch.zeros(4, dtype=torch.int32, device="cuda")
    meas = torch.ones(4, dtype=torch.int32, device="cuda")
    sums = torch.zeros((1, 1), dtype=torch.int64, device="cuda")
    rows = (ctypes.c_int64 * 1)(6_000_000)
    card = (ctypes.c_int32 * 1)(1)
    from paper_2306_08367_amd import binding as B
    rc = B._lib.lq_masked_groupby_sum_static(4, 1, B._ptr_array([fk]), rows, B._ptr_array([None]),
                                             B._ptr_array([None]), card, None, 1, B._ptr_array([meas]),
                                             sums.data_ptr(), None, 0, None)
    assert rc == 4 and "scratch" in lq.lq_last_error()
    rc = B._lib.lq_masked_groupby_sum_static(4, 1, B._ptr_array([fk]), (ctypes.c_int64 * 1)(10), B._ptr_array([None]),
                                             B._ptr_array([None]), card, None, 1, B._ptr_array([meas]),
                                             sums.data_ptr(), None, 1, None)
    assert rc == 6
