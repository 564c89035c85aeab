"""Compress and decompress one synthetic array a few times: a minimal driver for timing or profiling one setting.

    python3 -m paper_2406_11209_amd.examples.codec_repeat --shape 512 512 1024 --block 16 16 16 --itype i16

prints the kernel the dispatch picked and the average time of each direction (HIP events)."""
import argparse
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from paper_2406_11209_amd.api import PBZ_PATH_GENERIC, Codec  # noqa: E402

TORCH = {"f64": torch.float64, "f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", type=int, nargs="+", required=True)
    ap.add_argument("--block", type=int, nargs="+", required=True)
    ap.add_argument("--dtype", default="f32", choices=list(TORCH), help="element type of the array")
    ap.add_argument("--ftype", default="f32", choices=list(TORCH), help="working float type (storage type of N)")
    ap.add_argument("--itype", default="i8", choices=["i8", "i16", "i32"])
    ap.add_argument("--transform", default="dct", choices=["dct", "haar"])
    ap.add_argument("--keep", type=int, nargs="+", default=None,
                    help="keep only the low-frequency box of this shape of every block (default: keep everything)")
    ap.add_argument("--repeat", type=int, default=5)
    ap.add_argument("--path", default="auto", choices=["auto", "generic"],
                    help="generic: the general kernels, also where a specialised kernel exists")
    args = ap.parse_args()
    shape = tuple(args.shape)
    mask = None
    if args.keep is not None:
        mask = np.zeros(tuple(args.block), dtype=bool)
        mask[tuple(slice(0, k) for k in args.keep)] = True
    codec = Codec(tuple(args.block), args.ftype, args.itype, mask, args.transform)
    if args.path == "generic":
        codec.set_kernel_path(PBZ_PATH_GENERIC)
    gen = torch.Generator(device="cuda").manual_seed(240611209)
    x = torch.randn(shape, dtype=torch.float32, device="cuda", generator=gen).to(TORCH[args.dtype])
    N, F = codec.compress(x)
    y = codec.decompress(N, F, shape, TORCH[args.dtype])
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record()
    for _ in range(args.repeat):
        codec.compress(x, N, F)
    ev[1].record()
    for _ in range(args.repeat):
        codec.decompress(N, F, shape, out=y)
    ev[2].record()
    torch.cuda.synchronize()
    moved = x.numel() * x.element_size() + N.numel() * N.element_size() + F.numel() * F.element_size()
    tc, td = ev[0].elapsed_time(ev[1]) / args.repeat, ev[1].elapsed_time(ev[2]) / args.repeat
    print(f"{codec.kernel_name('compress', shape, args.dtype)}: compress {tc:.3f} ms ({moved / tc / 1e6:.0f} GB/s moved), "
          f"decompress {td:.3f} ms ({moved / td / 1e6:.0f} GB/s moved)")


if __name__ == "__main__":
    main()
