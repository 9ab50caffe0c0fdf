"""Every kernel of the library must be reached by the GPU test suite: profiles/pytest_gpu_kernel_trace.txt is
the rocprofv3 kernel trace of `pytest -m gpu`, summed per kernel template; a `__global__` function in csrc/ that
does not occur in it is code no parity test has run.  (CPU only: it reads the committed summary.)"""
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_kernel_occurs_in_the_trace_of_the_gpu_test_suite():
    kernels = {}
    for path in glob.glob(os.path.join(ROOT, "paper_2306_08367_amd", "csrc", "*")):
        with open(path) as f:
            src = f.read()
        for m in re.finditer(r"__global__[^;{]*?void\s+([A-Za-z0-9_]+)\s*\(", src, re.S):
            kernels[m.group(1)] = os.path.basename(path)
    assert len(kernels) > 50
    with open(os.path.join(ROOT, "profiles", "pytest_gpu_kernel_trace.txt")) as f:
        traced = {line.split()[-1]: int(line.split()[0]) for line in f if line.strip() and not line.startswith("#")}
    missing = sorted(f"{k} ({v})" for k, v in kernels.items() if traced.get(k, 0) < 1)
    assert not missing, f"kernels never launched by `pytest -m gpu`: {missing}"
