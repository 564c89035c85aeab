"""Build libpbz.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2406_11209_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpbz.so")
EXAMPLE = os.path.join(PKG, "c_abi_roundtrip")
PATTERNS = os.path.join(PKG, "memory_patterns")
SOURCES = ["pbz_api.hip", "pbz_generic.hip", "pbz_ops.hip", "pbz_fast.hip", "pbz_fast_lane.hip", "pbz_fast_quad16.hip",
           "pbz_fast_oct8.hip", "pbz_fast_cube16.hip", "pbz_wasserstein.hip", "pbz_tiled.hip", "pbz_static.hip", "pbz_copy.hip"]

# Packed-FP32 code generation is switched off on purpose (the flag applies to the device pass; the host
# pass prints a harmless "unknown feature" warning).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library; returns its path."""
    cc = hipcc()
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[cc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=6) as pool:
        for out in pool.map(_run, cmds):
            if verbose and out.strip():
                print(out)
    tmp = LIB + ".tmp"
    _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp])
    os.replace(tmp, LIB)
    # the C ABI used from plain C (no Python, no torch): a small round-trip program next to the library
    _run([cc, "-x", "c", os.path.join(PKG, "examples", "c_abi_roundtrip.c"), "-D__HIP_PLATFORM_AMD__",
          "-I" + os.path.join(ROOT, "include"), "-I/opt/rocm/include", "-L" + PKG, "-lpbz", "-L/opt/rocm/lib",
          "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib", "-o", EXAMPLE])
    # the memory-system yardsticks (no library code): what the box gives for the kernels' access patterns
    _run([cc] + FLAGS[:-2] + [os.path.join(PKG, "examples", "memory_patterns.hip"), "-o", PATTERNS])
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))


def build_host_sanitized(outdir: str) -> tuple:
    """The host half of the library (argument validation, layout arithmetic, dispatch) compiled for the CPU only
    with AddressSanitizer and UndefinedBehaviorSanitizer; no device code, so nothing in it can launch.  Returns
    (library path, sanitizer runtime to preload).  Used by a CPU test that runs the host-only checks against it."""
    cc = hipcc()
    os.makedirs(outdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-omit-frame-pointer"]
    objs = [os.path.join(outdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[cc, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC"] + san +
            ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-c", os.path.join(CSRC, s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=6) as pool:
        list(pool.map(_run, cmds))
    # a host-only object still refers to its translation unit's device image: give each an empty stand-in
    undefined = subprocess.run(["nm", "-u"] + objs, stdout=subprocess.PIPE, text=True, check=True).stdout.split()
    images = sorted({w for w in undefined if w.startswith("__hip_fatbin_")})
    stubs = os.path.join(outdir, "device_image_stubs.c")
    with open(stubs, "w") as fh:
        for name in images:
            fh.write("const unsigned char %s[64] __attribute__((aligned(4096))) = {0};\n" % name)
    _run(["gcc", "-c", "-fPIC", stubs, "-o", stubs.replace(".c", ".o")])
    lib = os.path.join(outdir, "libpbz_host_sanitized.so")
    _run([cc, "--cuda-host-only", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] +
         objs + [stubs.replace(".c", ".o"), "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", lib])
    runtime = subprocess.run([cc, "--cuda-host-only", "-print-file-name=libclang_rt.asan-x86_64.so"],
                             stdout=subprocess.PIPE, text=True, check=True).stdout.strip()
    return lib, runtime
