"""The bandwidth yardsticks the benchmarks quote their roofs from: the copy copies, the read and gather
sweeps write nothing, and bad arguments are refused on the host."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lq():
    import paper_2306_08367_amd as lq
    return lq


def test_stream_copy_copies(lq):
    src = torch.randint(0, 255, (3 * 4096 + 16,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    lq.lq_stream_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_read_and_gather_sweeps_touch_nothing(lq):
    buf = torch.randint(0, 255, (1 << 22,), dtype=torch.uint8, device="cuda")
    before = buf.clone()
    sink = torch.full((4,), 7, dtype=torch.int32, device="cuda")
    wbuf = torch.full((1 << 16,), 9, dtype=torch.uint8, device="cuda")
    lq.lq_yardstick_read(buf, 3, sink)
    for row_bytes in (16, 32, 64, 128, 256, 512, 1024):
        lq.lq_yardstick_gather(buf, row_bytes, 100_003, sink, seed=row_bytes)
    keys = torch.randint(0, (1 << 22) // 256, (50_000,), dtype=torch.int32, device="cuda")
    lq.lq_yardstick_gather(buf, 256, 50_000, sink, keys=keys)
    torch.cuda.synchronize()
    assert torch.equal(buf, before) and (sink == 7).all() and (wbuf == 9).all()
    # the stream form overwrites its write buffer with zeros, and only that
    lq.lq_yardstick_stream(buf, 2, wbuf[: (1 << 16) - 4096], sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, before) and (sink == 7).all()
    assert (wbuf[: (1 << 16) - 4096] == 0).all() and (wbuf[(1 << 16) - 4096:] == 9).all()


def test_yardsticks_refuse_bad_arguments(lq):
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(lq.LQError):
        lq.lq_yardstick_gather(buf, 48, 10, sink)                 # row size is not a power of two
    with pytest.raises(lq.LQError):
        lq.lq_yardstick_read(buf[8:4088], 1, sink)                # misaligned
    with pytest.raises(lq.LQError):
        lq.lq_yardstick_read(buf, 0, sink)


def test_matrix_yardstick_runs_and_refuses_bad_arguments(lq):
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(cus * 2 * 256, dtype=torch.float32, device="cuda")
    for nv in (0, 32, 64, 128):
        sink.zero_()
        lq.lq_yardstick_matrix(nv, 2, 3, sink)
        torch.cuda.synchronize()
        assert torch.isfinite(sink).all() and (sink != 0).any()
    with pytest.raises(lq.LQError):
        lq.lq_yardstick_matrix(48, 2, 3, sink)                    # not one of the compiled mixes
    with pytest.raises(lq.LQError):
        lq.lq_yardstick_matrix(0, 3, 3, sink)                     # sink too small for three wavefronts per SIMD
    with pytest.raises(lq.LQError):
        lq.lq_yardstick_matrix(0, 0, 3, sink)
