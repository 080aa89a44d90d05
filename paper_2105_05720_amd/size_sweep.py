"""Size sweep of the fused and unfused steps on one flat tensor, 2^10 .. 2^30 elements (the axis of the paper's
standalone experiment, Section 6.1.1 / Fig. 7), with the launch shape tuned per size.

For every size and every path (fused Adam, unfused Adam, fused LAMB, unfused LAMB) the step is timed for each
candidate launch shape (one workgroup per chunk of 1024 / 4096 / 16384 elements, or the ordered persistent
schedule on 4096-element chunks) and the best average is kept, like the paper's autotuner keeps the best
configuration per size.  Steps are replayed from a HIP graph so that small sizes measure the GPU, not the Python caller.

    python -m paper_2105_05720_amd.size_sweep [--min-log2 10] [--max-log2 30] [--R 8] [--markdown out.md]
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as cc
from .shard import Shard

PC, ORD = cc.CC_SCHEDULE_PER_CHUNK, cc.CC_SCHEDULE_ORDERED
SHAPES = ((1024, PC), (4096, PC), (16384, PC), (4096, ORD))       # (chunk elements, schedule)
PATHS = (("fused_adam", cc.cc_fused_adam_step, lambda R: 2 * R + 26),
         ("unfused_adam", cc.cc_unfused_adam_step, lambda R: 2 * R + 38),
         ("fused_lamb", cc.cc_fused_lamb_step, lambda R: 2 * R + 38),
         ("unfused_lamb", cc.cc_unfused_lamb_step, lambda R: 2 * R + 50))


def time_path(shard: Shard, fn, steps: int, per_graph: int) -> float:
    """Average microseconds per step over `steps` steps replayed from a graph of `per_graph` (even) steps."""
    hp = lambda t: cc.Hyper(step=t)
    for t in (1, 2):                                   # warm-up; also allocates the unfused pipeline's buffer
        shard.run(fn, hp(t))
        shard.commit()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(per_graph):
            shard.run(fn, hp(3 + i))
            shard.commit()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(1, steps // per_graph)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    assert int(shard.flag.item()) == 0
    return e0.elapsed_time(e1) * 1e3 / (reps * per_graph)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--min-log2", type=int, default=10)
    ap.add_argument("--max-log2", type=int, default=30)
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--markdown", type=str, default="")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    cc.load()
    R = args.R
    rows = []
    for k in range(args.min_log2, args.max_log2 + 1):
        n = 1 << k
        steps = 1000 if k <= 20 else (200 if k <= 24 else (40 if k <= 27 else 10))
        per_graph = min(20, steps)
        row = {"log2": k, "n": n}
        for name, fn, bpp in PATHS:
            best = None
            for chunk, sched in SHAPES:
                if chunk > 1024 and n < chunk:          # one partial chunk either way
                    continue
                if sched == ORD and n < 2 * chunk:
                    continue
                shard = Shard([n], [0.01], R, chunk_elems=chunk, schedule=sched)
                g = torch.Generator(device="cuda")
                g.manual_seed(k)
                shard.w[0].normal_(0.0, 0.02, generator=g)
                for arena in shard.grads:
                    arena.copy_(torch.empty(arena.numel(), device="cuda").normal_(0.0, 1e-3, generator=g))
                us = time_path(shard, fn, steps, per_graph)
                shard.destroy()
                del shard
                tag = "%d%s" % (chunk, " ordered" if sched == ORD else "")
                if best is None or us < best[0]:
                    best = (us, tag)
                if sched == ORD:
                    row.setdefault("ordered_us", {})[name] = round(us, 3)
            row[name] = {"us": round(best[0], 3), "chunk": best[1], "GB/s": round(bpp(R) * n / best[0] / 1e3, 1)}
        row["adam_fused_over_unfused"] = round(row["unfused_adam"]["us"] / row["fused_adam"]["us"], 3)
        row["lamb_fused_over_unfused"] = round(row["unfused_lamb"]["us"] / row["fused_lamb"]["us"], 3)
        rows.append(row)
        print(json.dumps(row), flush=True)
        torch.cuda.empty_cache()
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write("| log2 N | fused Adam us (chunk) | GB/s | unfused Adam us | fused/unfused speed-up | fused LAMB us (chunk) | GB/s | unfused LAMB us | speed-up |\n")
            f.write("|---|---|---|---|---|---|---|---|---|\n")
            for r in rows:
                f.write("| %d | %.2f (%s) | %.0f | %.2f | %.2fx | %.2f (%s) | %.0f | %.2f | %.2fx |\n" % (
                    r["log2"], r["fused_adam"]["us"], r["fused_adam"]["chunk"], r["fused_adam"]["GB/s"], r["unfused_adam"]["us"],
                    r["adam_fused_over_unfused"], r["fused_lamb"]["us"], r["fused_lamb"]["chunk"], r["fused_lamb"]["GB/s"],
                    r["unfused_lamb"]["us"], r["lamb_fused_over_unfused"]))
    return 0


if __name__ == "__main__":
    sys.exit(main())
