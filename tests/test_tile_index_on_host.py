"""The index arithmetic of the general tiled kernels (csrc/pbz_tile_index.h: block and row records, the packed
bounds comparison, the padded LDS addresses of the transform passes, the enumeration of elements and 16-byte pieces),
compiled for the host and checked by exhaustive enumeration against the plain definition (tests/host/
tile_index_check.cpp): every element of the array is reached exactly once, at the right offset, and everything
else is recognised as padding."""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

FIXED = [((8, 8), (37, 53)), ((8, 8, 8), (17, 9, 23)), ((4, 4, 4), (5, 30, 19)), ((2, 4), (3, 5)), ((32,), (100,)),
         ((1, 16, 16), (3, 33, 47)), ((1, 2, 2, 2, 4), (3, 4, 5, 6, 7)), ((2, 1, 2, 1, 2, 4), (2, 3, 2, 5, 6, 7)),
         ((32, 16, 2), (40, 33, 3)), ((32, 32, 1), (33, 40, 2)), ((2, 1, 2, 2, 4, 1, 2, 8), (3, 2, 3, 2, 5, 3, 6, 9)),
         ((2, 2, 2, 2, 2, 2, 2, 4), (3, 2, 2, 2, 2, 2, 3, 38)), ((1,), (7,)), ((1, 1), (5, 3)), ((16, 16, 16), (17, 16, 40)),
         ((32, 32), (64, 96)), ((2, 32), (5, 70)), ((4, 1), (9, 300)), ((1, 32, 4, 32), (2, 33, 5, 40))]


def random_geometries(n, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(n):
        nd = int(g.integers(1, 9))
        while True:
            block = tuple(int(2 ** g.integers(0, 6)) for _ in range(nd))
            if int(np.prod(block)) <= 4096:
                break
        shape = [max(1, int(g.integers(1, 4)) * b + (int(g.integers(0, b)) if g.integers(0, 2) else 0)) for b in block]
        while int(np.prod(shape)) > 60000:
            i = int(np.argmax(shape))
            shape[i] = max(1, shape[i] // 2)
        out.append((block, tuple(shape)))
    return out


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("g++ not found")
    exe = str(tmp_path_factory.mktemp("host") / "tile_index_check")
    subprocess.run([gxx, "-O1", "-std=c++17", "-Wno-unknown-pragmas", "-I" + os.path.join(ROOT, "paper_2406_11209_amd", "csrc"),
                    "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host", "tile_index_check.cpp"),
                    "-o", exe], check=True, capture_output=True)
    return exe


def test_tile_index_arithmetic_matches_the_definition(checker):
    cases = FIXED + random_geometries(120, 20240611)
    text = "".join(f"{len(b)} {' '.join(map(str, b))} {' '.join(map(str, s))}\n" for b, s in cases)
    out = subprocess.run([checker], input=text, check=True, capture_output=True, text=True).stdout.splitlines()
    assert len(out) == len(cases)
    bad = [(cases[i], line) for i, line in enumerate(out) if line != "ok"]
    assert not bad, bad[:5]
