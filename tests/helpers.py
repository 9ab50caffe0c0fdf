"""Shared helpers for the GPU parity tests."""
import numpy as np
import torch

TOL_F32 = 1e-4     # fp32 path against the fp64 oracle
TOL_BF16 = 2e-2    # bf16 path against the fp64 oracle


def assert_close(y, want, tol, what=""):
    """Per element: |y - want| <= tol * (|want| + rms(want)); also reports the norm-wise error."""
    y = y.detach().float().cpu().double().numpy() if hasattr(y, "detach") else np.asarray(y, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert y.shape == want.shape, f"{what}: shape {y.shape} vs {want.shape}"
    if want.size == 0:
        return
    rms = float(np.sqrt(np.mean(want * want)))
    err = np.abs(y - want)
    bound = tol * (np.abs(want) + rms)
    worst = int(np.argmax(err - bound))
    assert (err <= bound).all(), (
        f"{what}: element {np.unravel_index(worst, want.shape)} got {y.flat[worst]!r} want "
        f"{want.flat[worst]!r} (|err| {err.flat[worst]:.3e} > {bound.flat[worst]:.3e}); "
        f"norm-wise {err.max() / max(np.abs(want).max(), 1e-300):.3e}")


def to_dev(w, device="cuda"):
    """Moves every tensor of a workload dataclass to the device (in place) and returns it."""
    for name in ("X", "fact_mask"):
        if hasattr(w, name) and getattr(w, name) is not None:
            setattr(w, name, getattr(w, name).to(device))
    for name in ("dims", "fks", "weights", "biases", "dim_mask", "dim_code", "measures"):
        if hasattr(w, name):
            setattr(w, name, [None if t is None else t.to(device) for t in getattr(w, name)])
    return w


def cpu_list(ts):
    return [None if t is None else t.cpu() for t in ts]
