"""Measurement programs behind profiles/*.md, run as `python bench.py --mode <mode> [options]`.

  sweep     size sweep of the fused and unfused steps on one flat tensor, 2^10 .. 2^30 elements (the axis of the paper's
            standalone experiment, Section 6.1.1 / Fig. 7), with the launch shape tuned per size
  rsweep    the same for R in {1, 2, 4, 8, 16} and fp16 / fp32 gradient slices at 2^20, 2^24 and 2^28 elements
  cold      single fused steps with the caches evicted before each one, per cache policy (2^18 .. 2^26 elements)
  sliced    the BERT-Large parameter list with every tensor cut into 8, 64 or 256 slices: one rank's share
  epilogue  the fused model-parallel epilogue against its unfused pipeline at the sizes of the paper's standalone
            model-parallel experiment (Section 6.2.1)
  small     where the time of a launch-bound 2^20-element step goes: the step's memory pattern with parts taken away

Except in `cold`, steps are replayed from a HIP graph so that small sizes measure the GPU, not the Python caller.  Every mode prints one
JSON object per row and can write a markdown table (--markdown FILE).
"""
from __future__ import annotations

import argparse
import json

import torch

from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard

PC, ORD = cc.CC_SCHEDULE_PER_CHUNK, cc.CC_SCHEDULE_ORDERED
STREAM, RESIDENT, THROUGH = cc.CC_CACHE_STREAMING, cc.CC_CACHE_RESIDENT, cc.CC_CACHE_WRITE_THROUGH
# (chunk elements, schedule, cache policy, label): what cc_plan_autotune chooses among
SHAPES = ((1024, PC, RESIDENT, "1024 resident"), (1024, PC, THROUGH, "1024 write-through"), (1024, PC, STREAM, "1024"), (4096, PC, STREAM, "4096"),
          (16384, PC, STREAM, "16384"), (4096, ORD, STREAM, "4096 ordered"))


def paths(R: int, gb: int):
    return (("fused_adam", cc.cc_fused_adam_step, gb * R + 26), ("unfused_adam", cc.cc_unfused_adam_step, gb * R + 38),
            ("fused_lamb", cc.cc_fused_lamb_step, gb * R + 38), ("unfused_lamb", cc.cc_unfused_lamb_step, gb * R + 50))


def replay_us(enqueue, steps: int, per_graph: int = 100) -> float:
    """Average microseconds per call of enqueue(i) over about `steps` calls replayed from a graph of `per_graph` (a replay
    costs the device 4-5 us on top of its nodes: 0.05 us per call at 100 calls per graph)."""
    for i in range(2):
        enqueue(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(per_graph):
            enqueue(i)
    reps = max(1, steps // per_graph)
    for _ in range(max(1, reps // 4)):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * per_graph)


def time_step(shard: Shard, fn, steps: int) -> float:
    def enqueue(i):
        shard.run(fn, cc.Hyper(step=1 + i))
        shard.commit()
    us = replay_us(enqueue, steps, per_graph=min(100, max(2, steps // 2 * 2)))
    assert int(shard.flag.item()) == 0
    return us


def set_shape(shard: Shard, chunk: int, sched: int, policy: int) -> bool:
    """Puts both plans of the shard into one launch shape; False if the shape does not apply to this shard."""
    for p in shard.plans:
        cc.cc_plan_set_schedule(p, cc.CC_SCHEDULE_PER_CHUNK, 0)
        cc.cc_plan_set_chunk_elems(p, chunk)
        if sched == ORD:
            _, chunks, _ = cc.cc_plan_info(p)
            if chunks < 2:
                return False
        cc.cc_plan_set_schedule(p, sched, 0)
        cc.cc_plan_set_cache_policy(p, policy)
    return True


def seeded_flat_shard(n: int, R: int, grad_dtype=torch.float16, seed: int = 0) -> Shard:
    shard = Shard([n], [0.01], R, grad_dtype=grad_dtype, unfused=True)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    shard.w[0].normal_(0.0, 0.02, generator=g)
    for arena in shard.grads:
        arena.copy_(torch.empty(arena.numel(), device="cuda").normal_(0.0, 1e-3, generator=g))
    return shard


def steps_for(log2n: int) -> int:
    return 2000 if log2n <= 20 else (400 if log2n <= 24 else (40 if log2n <= 27 else 10))


def best_shapes(shard: Shard, R: int, gb: int, n: int, steps: int, which=None):
    """{path: {"us", "shape", "GB/s", "all": {shape label: us}}} over the launch shapes that apply."""
    row = {}
    for name, fn, bpp in paths(R, gb):
        if which and name not in which:
            continue
        times = {}
        for chunk, sched, policy, label in SHAPES:
            if chunk > 1024 and n < chunk:               # one partial chunk either way
                continue
            if not set_shape(shard, chunk, sched, policy):
                continue
            times[label] = round(time_step(shard, fn, steps), 3)
        label = min(times, key=times.get)
        set_shape(shard, 0, cc.CC_SCHEDULE_AUTO, cc.CC_CACHE_AUTO)       # what a caller gets without choosing anything
        auto = round(time_step(shard, fn, steps), 3)
        row[name] = {"us": times[label], "shape": label, "GB/s": round(bpp * n / times[label] / 1e3, 1), "all": times, "auto_us": auto}
    return row


def mode_sweep(argv) -> int:
    ap = argparse.ArgumentParser(prog="bench.py --mode sweep")
    ap.add_argument("--min-log2", type=int, default=10)
    ap.add_argument("--max-log2", type=int, default=30)
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--markdown", type=str, default="")
    args = ap.parse_args(argv)
    rows = []
    for k in range(args.min_log2, args.max_log2 + 1):
        n = 1 << k
        shard = seeded_flat_shard(n, args.R, seed=k)
        row = {"log2": k, "n": n}
        row.update(best_shapes(shard, args.R, 2, n, steps_for(k)))
        shard.destroy()
        del shard
        torch.cuda.empty_cache()
        row["adam_fused_over_unfused"] = round(row["unfused_adam"]["us"] / row["fused_adam"]["us"], 3)
        row["lamb_fused_over_unfused"] = round(row["unfused_lamb"]["us"] / row["fused_lamb"]["us"], 3)
        rows.append(row)
        print(json.dumps(row), flush=True)
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write("| log2 N | fused Adam us (shape) | GB/s | % of 8 TB/s | unfused Adam us | fused speed-up | fused LAMB us (shape) | GB/s | % of 8 TB/s | unfused LAMB us | speed-up |\n")
            f.write("|---|---|---|---|---|---|---|---|---|---|---|\n")
            for r in rows:
                f.write("| %d | %.2f (%s) | %.0f | %.1f | %.2f | %.2fx | %.2f (%s) | %.0f | %.1f | %.2f | %.2fx |\n" % (
                    r["log2"], r["fused_adam"]["us"], r["fused_adam"]["shape"], r["fused_adam"]["GB/s"], r["fused_adam"]["GB/s"] / 80.0,
                    r["unfused_adam"]["us"], r["adam_fused_over_unfused"], r["fused_lamb"]["us"], r["fused_lamb"]["shape"],
                    r["fused_lamb"]["GB/s"], r["fused_lamb"]["GB/s"] / 80.0, r["unfused_lamb"]["us"], r["lamb_fused_over_unfused"]))
            labels = [s[3] for s in SHAPES]
            for path, title in (("fused_adam", "Fused Adam"), ("fused_lamb", "Fused LAMB")):
                f.write("\n%s, microseconds per step under every launch shape (chunk elements, schedule, cache policy) and under the "
                        "library's own choice (no cc_plan_set_* call):\n\n" % title)
                f.write("| log2 N | " + " | ".join(labels) + " | automatic | automatic / best |\n|---|" + "---|" * (len(labels) + 2) + "\n")
                for r in rows:
                    f.write("| %d | " % r["log2"] + " | ".join("%.2f" % r[path]["all"][l] if l in r[path]["all"] else "-" for l in labels)
                            + " | %.2f | %.3f |\n" % (r[path]["auto_us"], r[path]["auto_us"] / r[path]["us"]))
    return 0


def mode_rsweep(argv) -> int:
    ap = argparse.ArgumentParser(prog="bench.py --mode rsweep")
    ap.add_argument("--sizes", type=str, default="20,24,28")
    ap.add_argument("--Rs", type=str, default="1,2,4,8,16")
    ap.add_argument("--markdown", type=str, default="")
    args = ap.parse_args(argv)
    rows = []
    for k in [int(x) for x in args.sizes.split(",")]:
        n = 1 << k
        for gname, gdtype, gb in (("f16", torch.float16, 2), ("f32", torch.float32, 4)):
            for R in [int(x) for x in args.Rs.split(",")]:
                shard = seeded_flat_shard(n, R, grad_dtype=gdtype, seed=k)
                row = {"log2": k, "grad": gname, "R": R}
                row.update(best_shapes(shard, R, gb, n, steps_for(k), which=("fused_adam", "unfused_adam")))
                row["adam_fused_over_unfused"] = round(row["unfused_adam"]["us"] / row["fused_adam"]["us"], 3)
                shard.destroy()
                del shard
                torch.cuda.empty_cache()
                rows.append(row)
                print(json.dumps(row), flush=True)
    if args.markdown:
        labels = [s[3] for s in SHAPES]
        with open(args.markdown, "w") as f:
            f.write("| log2 N | slices | R | B/param | best shape | us | GB/s | % of 8 TB/s | " + " | ".join(labels) + " | unfused us (shape) | fused speed-up |\n")
            f.write("|---|---|---|---|---|---|---|---|" + "---|" * len(labels) + "---|---|\n")
            for r in rows:
                fa = r["fused_adam"]
                f.write("| %d | %s | %d | %d | %s | %.2f | %.0f | %.1f | " % (
                    r["log2"], r["grad"], r["R"], (2 if r["grad"] == "f16" else 4) * r["R"] + 26, fa["shape"], fa["us"], fa["GB/s"], fa["GB/s"] / 80.0))
                f.write(" | ".join("%.2f" % fa["all"][l] if l in fa["all"] else "-" for l in labels))
                f.write(" | %.2f (%s) | %.2fx |\n" % (r["unfused_adam"]["us"], r["unfused_adam"]["shape"], r["adam_fused_over_unfused"]))
    return 0


def mode_cold(argv) -> int:
    """One step at a time with the caches evicted first (a 2 GiB copy), as a training loop sees the optimizer step after a
    backward pass: median of `reps` event pairs that bracket the step alone, per cache policy and for the automatic choice."""
    ap = argparse.ArgumentParser(prog="bench.py --mode cold")
    ap.add_argument("--min-log2", type=int, default=18)
    ap.add_argument("--max-log2", type=int, default=26)
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--reps", type=int, default=15)
    ap.add_argument("--markdown", type=str, default="")
    args = ap.parse_args(argv)
    nbytes = 2 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)

    def cold(shard, fn):
        times = []
        for i in range(args.reps):
            cc.cc_copy_probe(dst, src, nbytes)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            shard.run(fn, cc.Hyper(step=1 + i))
            b.record()
            shard.commit()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3)
        times.sort()
        return round(times[len(times) // 2], 2)

    shapes = ((1024, PC, STREAM, "non-temporal"), (1024, PC, THROUGH, "write-through"), (1024, PC, RESIDENT, "resident"),
              (0, cc.CC_SCHEDULE_AUTO, cc.CC_CACHE_AUTO, "automatic"))
    rows = []
    for k in range(args.min_log2, args.max_log2 + 1):
        shard = seeded_flat_shard(1 << k, args.R, seed=k)
        row = {"log2": k}
        for name, fn in (("adam", cc.cc_fused_adam_step), ("lamb", cc.cc_fused_lamb_step)):
            for chunk, sched, policy, label in shapes:
                set_shape(shard, chunk, sched, policy)
                row[name + " " + label] = cold(shard, fn)
        assert int(shard.flag.item()) == 0
        shard.destroy()
        del shard
        torch.cuda.empty_cache()
        rows.append(row)
        print(json.dumps(row), flush=True)
    if args.markdown:
        cols = [name + " " + s[3] for name in ("adam", "lamb") for s in shapes]
        with open(args.markdown, "w") as f:
            f.write("| log2 N | " + " | ".join(cols) + " |\n|---|" + "---|" * len(cols) + "\n")
            for r in rows:
                f.write("| %d | " % r["log2"] + " | ".join("%.2f" % r[c] for c in cols) + " |\n")
    return 0


def mode_sliced(argv) -> int:
    """Every tensor of the BERT-Large list cut into `ranks` slices, one rank's share (Section 5.2, "Sliced Tensor": what a
    rank updates after the fused schedule's reduce-scatter): 398 tensors per rank, most of them a handful of elements."""
    from paper_2105_05720_amd import workloads as W
    ap = argparse.ArgumentParser(prog="bench.py --mode sliced")
    ap.add_argument("--ranks", type=str, default="8,64,256")
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--markdown", type=str, default="")
    args = ap.parse_args(argv)
    specs = W.bert_large_list()
    rows = []
    for ranks in (int(x) for x in args.ranks.split(",")):
        numels = [(s.numel + ranks - 1) // ranks for s in specs]
        shard = Shard(numels, [0.01 if s.decays else 0.0 for s in specs], args.R, align_elems=1024, unfused=True)
        g = torch.Generator(device="cuda")
        g.manual_seed(ranks)
        shard.w[0].normal_(0.0, 0.02, generator=g)
        for arena in shard.grads:
            arena.copy_(torch.empty(arena.numel(), device="cuda").normal_(0.0, 1e-3, generator=g))
        n = sum(numels)
        chunk, block, policy = cc.cc_plan_layout(shard.plans[0])
        row = {"ranks": ranks, "numel": n, "tensors": len(numels), "chunks": cc.cc_plan_info(shard.plans[0])[1],
               "chunk_elems": chunk, "cache_policy": policy}
        for name, fn, bpp in paths(args.R, 2):
            us = time_step(shard, fn, 2000 if n < (1 << 23) else 400)
            row[name] = {"us": round(us, 2), "GB/s": round(bpp * n / us / 1e3, 1)}
        shard.destroy()
        del shard
        torch.cuda.empty_cache()
        rows.append(row)
        print(json.dumps(row), flush=True)
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write("| ranks | elements per rank | tensors | chunks | fused Adam us | GB/s | % of 8 TB/s | unfused Adam us | speed-up | fused LAMB us | GB/s | unfused LAMB us | speed-up |\n"
                    "|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")
            for r in rows:
                a, ua, l, ul = r["fused_adam"], r["unfused_adam"], r["fused_lamb"], r["unfused_lamb"]
                f.write("| %d | %d | %d | %d | %.2f | %.0f | %.1f | %.2f | %.2fx | %.2f | %.0f | %.2f | %.2fx |\n" % (
                    r["ranks"], r["numel"], r["tensors"], r["chunks"], a["us"], a["GB/s"], a["GB/s"] / 80.0, ua["us"], ua["us"] / a["us"],
                    l["us"], l["GB/s"], ul["us"], ul["us"] / l["us"]))
    return 0


def mode_epilogue(argv) -> int:
    ap = argparse.ArgumentParser(prog="bench.py --mode epilogue")
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--markdown", type=str, default="")
    ap.add_argument("--once", action="store_true", help="3 plain launches of each variant on the whole [8, 1024, 3072] tensor (for counter runs)")
    args = ap.parse_args(argv)
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
            grid = lambda i: cc.cc_fused_epilogue(partials, bias, residual, out, first, H, p, seed)
            unfused_fn = lambda i: cc.cc_unfused_epilogue(partials, bias, residual, out, scratch, first, H, p, seed)
            if args.once:
                if B == 8 and name == "whole tensor":
                    for fn in (grid, unfused_fn):
                        for i in range(3):
                            fn(i)
                    torch.cuda.synchronize()
                continue
            fused, t_unf = replay_us(grid, args.steps), replay_us(unfused_fn, args.steps)
            row = {"B": B, "S": S, "H": H, "R": R, "what": name, "numel": n, "step_bytes": (2 * R + 4) * n,
                   "fused_us": round(fused, 2),
                   "fused_GB/s": round((2 * R + 4) * n / fused / 1e3, 1),
                   "unfused_us": round(t_unf, 2), "unfused_GB/s": round((2 * R + 12) * n / t_unf / 1e3, 1),
                   "speedup": round(t_unf / fused, 3)}
            rows.append(row)
            print(json.dumps(row), flush=True)
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write("| B | slice | elements | step bytes (MB) | fused us | GB/s (2R+4 B/elem) | % of 8 TB/s | unfused us | GB/s (2R+12 B/elem) | fused speed-up |\n|---|---|---|---|---|---|---|---|---|---|\n")
            for r in rows:
                f.write("| %d | %s | %d | %.0f | %.2f | %.0f | %.1f | %.2f | %.0f | %.2fx |\n" % (
                    r["B"], r["what"], r["numel"], r["step_bytes"] / 1e6, r["fused_us"], r["fused_GB/s"],
                    r["fused_GB/s"] / 80.0, r["unfused_us"], r["unfused_GB/s"], r["speedup"]))
    return 0


POLICIES = ((STREAM, "non-temporal loads and stores"), (RESIDENT, "plain loads, write-through stores"),
            (THROUGH, "non-temporal loads, write-through stores"))


def mode_small(argv) -> int:
    ap = argparse.ArgumentParser(prog="bench.py --mode small")
    ap.add_argument("--log2", type=int, default=20)
    ap.add_argument("--R", type=int, default=4)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--markdown", type=str, default="")
    ap.add_argument("--once", action="store_true", help="40 plain launches of every variant instead of timed graph replays (for a kernel trace)")
    args = ap.parse_args(argv)
    n, R = 1 << args.log2, args.R
    shard = seeded_flat_shard(n, R, seed=1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    tensors = []
    for src in (0, 1):
        dst = 1 - src
        tensors.append(cc.Tensor(numel=n, w_in=shard.w[src], m_in=shard.m[src], v_in=shard.v[src], w_out=shard.w[dst], m_out=shard.m[dst],
                                 v_out=shard.v[dst], w16_out=shard.w16[dst], grad=list(shard.grads), weight_decay=0.01))
    rows = []
    names = {0: "empty workgroups", 1: "loads only", 2: "stores only", 3: "loads + stores, no arithmetic, no flag"}
    variants = [(names[what], pname, (lambda i, what=what, policy=policy: cc.cc_pattern_probe(tensors[i & 1], R, what, policy, sink)))
                for what in (0, 1, 2, 3) for policy, pname in POLICIES
                if policy == STREAM or what == 3 or (what, policy) in ((1, RESIDENT), (2, THROUGH))]
    for policy, pname in POLICIES:
        def full(i, policy=policy):
            shard.run(cc.cc_fused_adam_step, cc.Hyper(step=1 + i))
            shard.commit()
        variants.append(("the fused Adam step", pname, full, policy))
    for v in variants:
        name, pname, fn = v[0], v[1], v[2]
        if len(v) == 4:
            set_shape(shard, 1024, PC, v[3])
        if args.once:
            for i in range(40):
                fn(i)
            torch.cuda.synchronize()
            continue
        us = replay_us(fn, args.steps)
        row = {"variant": name, "accesses": pname, "us": round(us, 3)}
        rows.append(row)
        print(json.dumps(row), flush=True)
    assert int(shard.flag.item()) == 0
    if args.markdown and rows:
        bytes_step = (2 * R + 26) * n
        with open(args.markdown, "w") as f:
            f.write("| variant (one 128-thread workgroup per 1024 elements, N = 2^%d, R = %d) | accesses | us per launch | GB/s of the step's %.2f MB |\n|---|---|---|---|\n" % (
                args.log2, R, bytes_step / 1e6))
            for r in rows:
                f.write("| %s | %s | %.2f | %s |\n" % (r["variant"], r["accesses"], r["us"],
                                                     "%.0f" % (bytes_step / r["us"] / 1e3) if r["variant"] == "the fused Adam step" else ""))
    shard.destroy()
    return 0


def main(mode: str, argv) -> int:
    return {"sweep": mode_sweep, "rsweep": mode_rsweep, "cold": mode_cold, "sliced": mode_sliced, "epilogue": mode_epilogue, "small": mode_small}[mode](argv)
