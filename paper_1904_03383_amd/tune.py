"""Tune tile configurations for a list of shapes and write the tune cache.

    python -m paper_1904_03383_amd.tune 4096x4096x4096 1024x1024x1024 512:32x32x64 --out tuned.txt

A shape is ``MxNxK`` or ``BATCH:MxNxK``.  Operands are random, packed and resident in device memory;
a workspace of the size the library asks for is set for the duration.  ``--math pieces`` tunes for the
opt-in math mode that also considers the bf16-piece kernels (entries are kept per mode).  Later processes load
the file with ``tg.load_tune_cache(path)`` (C: ``tg_load_tune_cache``) and never time anything.
"""
from __future__ import annotations

import argparse
import sys


def parse_shape(text: str):
    batch = 1
    if ":" in text:
        b, text = text.split(":", 1)
        batch = int(b)
    m, n, k = (int(x) for x in text.lower().split("x"))
    if min(batch, m, n, k) < 1:
        raise ValueError("sizes must be positive")
    return batch, m, n, k


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("shapes", nargs="+", help="MxNxK or BATCH:MxNxK")
    ap.add_argument("--out", required=True, help="tune cache file to write (merged with --merge)")
    ap.add_argument("--merge", default=None, help="existing tune cache to load first")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--math", choices=["fp32", "pieces"], default="fp32",
                    help="math mode to tune for (pieces: TG_MATH_BF16_PIECES)")
    args = ap.parse_args(argv)
    shapes = [parse_shape(s) for s in args.shapes]

    import torch
    from . import binding as tg
    if not torch.cuda.is_available():
        sys.exit("tune: no GPU visible")
    tg.load_library()
    if args.merge:
        tg.load_tune_cache(args.merge)
    tg.set_math(tg.MATH_BF16_PIECES if args.math == "pieces" else tg.MATH_FP32_MFMA)
    ws_bytes = max(tg.workspace_bytes(*s) for s in shapes)
    ws = torch.empty(max(ws_bytes // 4, 4), dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    try:
        for batch, m, n, k in shapes:
            a = torch.randn((batch, m, k), device="cuda")
            b = torch.randn((batch, k, n), device="cuda")
            tg.tune(a, b, reps=args.reps)
            print(f"{batch}:{m}x{n}x{k}  ->  {tg.last_config()}", flush=True)
            del a, b
        tg.save_tune_cache(args.out)
    finally:
        tg.set_workspace(None)
        tg.set_math(tg.MATH_FP32_MFMA)
    return 0


if __name__ == "__main__":
    sys.exit(main())
