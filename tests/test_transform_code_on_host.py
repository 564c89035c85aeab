"""The kernels' in-register transform code (pbz_dct.h, pbz_haar.h), compiled for the host and run on the CPU,
against the oracle's transform matrices: forward and inverse images of every unit vector for every supported
length, in FP32 and FP64, and the inverse variant that is told the upper half of its inputs is zero.  This pins
the constants and the even/odd recursion of the GPU code without a GPU; the oracle builds its matrices from the
defining formula (Sec. III-A, Appendix A) and shares no code with the header."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import pbz_oracle as po

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rows(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path_factory.mktemp("host") / "transform_tables")
    src = os.path.join(ROOT, "tests", "host", "transform_tables.hip")
    subprocess.run([hipcc, "--cuda-host-only", "-O1", "-std=c++17", "-I" + os.path.join(ROOT, "paper_2406_11209_amd", "csrc"),
                    "-I" + os.path.join(ROOT, "include"), src, "-o", exe], check=True, capture_output=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    table = {}
    for line in out.splitlines():
        kind, tf, typ, n, k, *vals = line.split()
        table[(kind, tf, typ, int(n), int(k))] = np.array([float(v) for v in vals])
    return table


@pytest.mark.parametrize("tf", ["dct", "haar"])
@pytest.mark.parametrize("typ,tol", [("f64", 4e-15), ("f32", 4e-7)])
@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 32])
def test_transform_code_matches_the_defining_matrices(rows, tf, typ, tol, n):
    H = po.transform_matrix(n, tf)                    # H[m][q]: sample m, coefficient q
    for m in range(n):
        assert np.max(np.abs(rows[("fwd", tf, typ, n, m)] - H[m, :])) <= tol, ("forward", m)
    for q in range(n):
        assert np.max(np.abs(rows[("inv", tf, typ, n, q)] - H[:, q])) <= tol, ("inverse", q)
    for q in range(n // 2):                           # the upper inputs hold 1e30 and must not be read
        assert np.max(np.abs(rows[("half", tf, typ, n, q)] - H[:, q])) <= tol, ("inverse, half the inputs", q)
