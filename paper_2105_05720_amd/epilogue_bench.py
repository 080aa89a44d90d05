"""Timing of the fused model-parallel epilogue against its unfused pipeline at the sizes of the paper's standalone
model-parallel experiment (Section 6.2.1: GPT-2 8.3B shapes, S = 1024, H = 3072, batch 8 and 16), R = 8 partial
outputs, dropout 0.1: the whole [B, S, H] tensor (the all-reduce-then-pointwise shape) and one rank's 1/8 slice.

    python -m paper_2105_05720_amd.epilogue_bench [--steps 200] [--markdown out.md]
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as cc


def timed(fn, steps: int) -> float:
    """Average microseconds per call over `steps` calls replayed from a HIP graph of 20."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    per = 20
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(per):
            fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(1, steps // per)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * per)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--markdown", type=str, default="")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    cc.load()
    R, S, H, p, seed = args.R, 1024, 3072, 0.1, 2021
    rows = []
    for B in (8, 16):
        full = B * S * H
        for name, n, first in (("whole tensor", full, 0), ("1/8 slice", full // 8, full // 8 * 3)):
            g = torch.Generator(device="cuda")
            g.manual_seed(B)
            partials = [torch.empty(n, device="cuda").normal_(0, 0.3, generator=g).half() for _ in range(R)]
            bias = torch.empty(H, device="cuda").normal_(0, 0.1, generator=g).half()
            residual = torch.empty(n, device="cuda").normal_(0, 1.0, generator=g).half()
            out = torch.empty(n, dtype=torch.float16, device="cuda")
            scratch = torch.empty(n, dtype=torch.float32, device="cuda")
            fused = timed(lambda: cc.cc_fused_epilogue(partials, bias, residual, out, first, H, p, seed), args.steps)
            unfused = timed(lambda: cc.cc_unfused_epilogue(partials, bias, residual, out, scratch, first, H, p, seed), args.steps)
            row = {"B": B, "S": S, "H": H, "R": R, "what": name, "numel": n,
                   "fused_us": round(fused, 2), "fused_GB/s": round((2 * R + 4) * n / fused / 1e3, 1),
                   "unfused_us": round(unfused, 2), "unfused_GB/s": round((2 * R + 12) * n / unfused / 1e3, 1),
                   "speedup": round(unfused / fused, 3)}
            rows.append(row)
            print(json.dumps(row), flush=True)
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write("| B | slice | elements | fused us | GB/s (2R+4 B/elem) | unfused us | GB/s (2R+12 B/elem) | fused speed-up |\n|---|---|---|---|---|---|---|---|\n")
            for r in rows:
                f.write("| %d | %s | %d | %.2f | %.0f | %.2f | %.0f | %.2fx |\n" % (
                    r["B"], r["what"], r["numel"], r["fused_us"], r["fused_GB/s"], r["unfused_us"], r["unfused_GB/s"], r["speedup"]))
    return 0


if __name__ == "__main__":
    sys.exit(main())
