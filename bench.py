#!/usr/bin/env python3
"""Benchmark: batch-1 fp32 inference latency of ResNet-50 v1.5 (headline) and
BERT-base seq 128 on one MI355X, run as a sequence of fused-operator kernels
under the placement the library's own measurer + dynamic programme choose.

    python bench.py --gpus 1 --steps 200 --warmup 20

A step is one pass of the compiled kernel sequence over one synthetic input
that is already resident in HBM.  The set-up part of the path (registration,
match enumeration, per-subgraph cost profiling, placement search, compile) runs
once before the timed region; its wall time is reported under "optimise".
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_HBM_GBPS = 8000.0            # MI355X HBM3E
# the MFMA kernel variants registered as separate backends; the search picks one per fused subgraph
VARIANTS = ("igemm", "igemm_s", "igemm_s8", "igemm_s16", "igemm_m", "igemm_l", "igemm_s_nk", "igemm_s8_nk",
            "igemm_s16_nk", "igemm_r32", "igemm_r16", "igemm_r32_w4", "igemm_r32_w8", "igemm_r16_w4", "igemm_r16_w8",
            "igemm_r16x2_w4", "igemm_r16x2_w8", "igemm_r16_sk", "igemm_r16_sk_w4", "igemm_r32_sk")


# HBM-side traffic of the fp32 MFMA kernels of one step, from two rocprofv3 --pmc runs of this file with
# --passes-only (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch, summed over the MFMA-kernel dispatches and divided
# by the warm-up + steps passes of the run: ResNet-50 54 such dispatches per pass - 51 convolution launches, two of
# them regions of two, and 3 split-K reductions; BERT-base 60).  Scale factors from the 256 MiB plain device
# copy of --calib-copy in the same runs: WRITE_SIZE read 262144.0 KiB for it (factor 1.000), FETCH_SIZE
# 131083.5 KiB (factor 2.000).  profiles/*_pmc_summary.txt hold the runs.  The figures hold for the kernel sources
# they were taken with; after any change to them `traffic` is reported as null.
TRAFFIC = {"resnet50": {"sources": "95fd1455c2556476", "fetch_bytes": 290.96e6, "write_bytes": 45.06e6},
           "bert_base": {"sources": "95fd1455c2556476", "fetch_bytes": 689.36e6, "write_bytes": 47.19e6}}


def kernel_sources_fingerprint():
    import glob
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2111_00655_amd", "csrc")
    files = glob.glob(os.path.join(d, "gemm_*.hip")) + glob.glob(os.path.join(d, "gemm_*.h"))
    files += [os.path.join(d, n) for n in ("kernels_gemm.hip", "device_common.h", "kernels.h")]
    for f in sorted(files):                     # the convolution / GEMM kernels, their headers and argument blocks
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def optimise(desc, reg, opts, cost_log="", rules=()):
    """register -> match -> profile -> search -> compile; returns pieces + timings.
    With a cost log file, measured costs are reused from / added to it."""
    import paper_2111_00655_amd as clg
    from paper_2111_00655_amd import binding as B
    t0 = time.perf_counter()
    s = clg.Session(desc, reg, device=0, rules=rules)
    if cost_log and os.path.exists(cost_log):
        B.clg_cost_log_load(s.ctx, cost_log)
    t1 = time.perf_counter()
    ms = s.match()
    t2 = time.perf_counter()
    costs = s.profile(opts)
    t3 = time.perf_counter()
    if cost_log:
        B.clg_cost_log_save(s.ctx, cost_log)
    total, ids = s.search(costs, 0)
    t4 = time.perf_counter()
    plan = s.compile(ids).bind()
    t5 = time.perf_counter()
    timing = dict(build_graph_s=t1 - t0, match_s=t2 - t1, profile_s=t3 - t2, search_s=t4 - t3,
                  compile_s=t5 - t4, n_matches=len(ms), n_kernels=plan.n_kernels,
                  predicted_ms=total / 1e6)
    return s, plan, costs, ids, timing


def graph_level(plan, steps, warmup, seed=0):
    """Graph-level placement (paper Sec. 4.3) on a compiled op-level plan: evolutionary search over the
    digit strings of the region backend (lanes = 1), every string priced by timing the whole sequence.
    Leaves the plan set to the best string; op-level and graph-level step times are re-measured the way
    the headline figure is (time_steps)."""
    import numpy as np
    from paper_2111_00655_amd import binding as B
    plan.bind()
    n = plan.n_kernels
    plan.set_handover([0] * n, lanes=1)
    launches_before = plan.n_launches
    op_ms = time_steps(plan, steps, warmup)
    rand = np.random.default_rng(seed).integers(0, 2 ** 32, 1 << 20, dtype=np.uint64).tolist()
    t0 = time.perf_counter()
    best, best_ns, seed_ns, evals, hist = plan.search_graph_level(
        B.make_es_opts(population=12, generations=12, tournament=3, patience=5, p_init=0.5, p_mutate=0.5, p_flip=0.1, p_cross=0.5,
                       seed_ones=True),
        rand, lanes=1, warmup=3, batches=3, reps=20)
    search_s = time.perf_counter() - t0
    gl_ms = time_steps(plan, steps, warmup)
    rg = plan.regions()
    return dict(op_level_ms=round(op_ms, 4), graph_level_ms=round(gl_ms, 4), launches_before=launches_before,
                launches_after=plan.n_launches, regions=max(rg) + 1 if rg else 0, kernels=n, handed_over=int(sum(best)),
                digits=[int(b) for b in best],
                search_seed_ns=int(seed_ns), search_best_ns=int(best_ns), strings_priced=evals,
                history_ms=[round(h / 1e6, 4) for h in hist], search_s=round(search_s, 2))


def weight_memory(plan):
    """Device memory of the weights: the plan's packed copies, and the caller's copies that no execution of the
    plan reads any more (clg_plan_reads_constant): capacity that could be released, not traffic."""
    import numpy as np
    nr = plan.constants_not_read()
    d = plan.s.desc
    return dict(packed_mb=round(sum(nr.values()) / 1e6, 1),
                caller_copies_not_read_mb=round(sum(4.0 * float(np.prod(d.nodes[n]["shape"])) for n in nr) / 1e6, 1),
                caller_constants_read_mb=round(sum(4.0 * float(np.prod(nd["shape"])) for n, nd in enumerate(d.nodes)
                                                   if nd["kind"] == "const" and n not in nr) / 1e6, 1))


def large_shapes(path):
    """Single operators large enough to be bound by the matrix cores, priced under every MFMA variant backend by the
    library's measurer (launch-inclusive time of back-to-back launches).  Returns {case: {backend: TFLOP/s}}."""
    import numpy as np
    import workloads as wl
    import paper_2111_00655_amd as clg
    from paper_2111_00655_amd import binding as B
    reg = wl.default_registry(VARIANTS)
    opts = B.ProfileOpts(warmup=5, batches=5, min_batch_us=200, max_launches=200)
    r = np.random.default_rng(0)
    cases = []
    for (m, n, k) in ((4096, 4096, 4096), (2048, 2048, 2048), (8192, 1024, 1024)):
        d = wl.GraphDesc("large_dense")
        x = d.input(r.standard_normal((m, k), dtype=np.float32))
        w = d.const(r.standard_normal((n, k), dtype=np.float32))
        d.mark_output(d.op("dense", [x, w]))
        cases.append((f"dense {m}x{k} . {n}x{k}^T", d, 2.0 * m * n * k))
    for (b, c, co, h) in ((32, 256, 256, 56), (32, 512, 512, 28)):
        d = wl.GraphDesc("large_conv")
        x = d.input(r.standard_normal((b, c, h, h), dtype=np.float32))
        w = d.const(r.standard_normal((co, c, 3, 3), dtype=np.float32))
        d.mark_output(d.op("conv2d", [x, w], stride=(1, 1), pad=(1, 1), groups=1))
        cases.append((f"conv2d 3x3 batch {b} {c}->{co} {h}x{h}", d, 2.0 * b * co * h * h * c * 9))
    out = {}
    lines = ["Compute-bound single operators, fp32, one MI355X: launch-inclusive time per launch from the library's measurer",
             f"and the operator's own flops over it; fp32 MFMA peak {PEAK_MFMA_F32_TFLOPS} TFLOP/s.", "",
             f"{'operator':40s} {'backend':14s} {'us':>9s} {'TFLOP/s':>8s} {'of peak':>8s}"]
    for label, d, flops in cases:
        s = clg.Session(d, reg, device=0)
        ms = s.match()
        costs = s.profile(opts)
        out[label] = {}
        for i, m in enumerate(ms):
            backend = reg[m.pattern][0]
            if backend == "direct" or costs[i] >= B.COST_INF:
                continue
            tf = flops / costs[i] / 1e3
            out[label][backend] = round(tf, 1)
            lines.append(f"{label:40s} {backend:14s} {costs[i] / 1e3:9.1f} {tf:8.1f} {tf / PEAK_MFMA_F32_TFLOPS:8.3f}")
        s.close()
    os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    return out


def time_steps(plan, steps, warmup):
    import torch
    for _ in range(warmup):
        plan.execute()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        plan.execute()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def graph_replay_ms(plan, steps, warmup):
    """The same kernel sequence captured once into a HIP graph and replayed.
    The replayed outputs are checked against the eager ones (bitwise) before timing."""
    import torch
    plan.execute()
    torch.cuda.synchronize()
    ref = [t.clone() for t in plan._out]
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        plan.execute()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            plan.execute()
    torch.cuda.synchronize()
    for rep in range(3):                       # several replays with eager work between them
        for t in plan._out:
            t.zero_()
        g.replay()
        torch.cuda.synchronize()
        if not all(torch.equal(a, b) for a, b in zip(ref, plan._out)):
            return None
    for _ in range(warmup):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def cold_cache_ms(plan, steps=20):
    """One pass at a time with the caches scrubbed in between (a 512 MB buffer is
    rewritten before each pass), timed with an event pair around the pass."""
    import torch
    scrub = torch.empty(512 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tot = 0.0
    for i in range(steps):
        scrub.fill_(float(i))
        e0.record()
        plan.execute()
        e1.record()
        torch.cuda.synchronize()
        tot += e0.elapsed_time(e1)
    return tot / steps


def ablation(desc, variants, opts, cost_log, steps, warmup):
    """Latency of the placement found when the MFMA kernels are restricted to a
    single variant, next to the search over all of them (paper Sec. 5.5 studies
    the same question for its backends)."""
    import workloads as wl
    from workloads import patterns as wp
    out = {}
    for v in variants:
        if v in wp.DENSE_ONLY_BACKENDS:        # a variant for dense layers only covers no network by itself
            continue
        reg = wl.default_registry((v,))
        try:
            s, plan, _, _, t = optimise(desc, reg, opts, cost_log)
        except Exception as e:                 # a variant alone may not cover the graph (grouped conv)
            out[v] = None
            continue
        out[v] = round(time_steps(plan, steps, warmup), 4)
        plan.destroy()
        s.close()
    return out


def kernel_table(plan, reps=20):
    """Per-kernel durations (HIP events around every launch, on the launch
    stream), averaged over `reps` passes."""
    import numpy as np
    plan.execute_timed()
    acc = np.zeros(plan.n_kernels)
    for _ in range(reps):
        acc += plan.execute_timed()
    ns = acc / reps
    rows = []
    for k, t in zip(plan.kernels(), ns):
        r = dict(k)
        r["ns"] = float(t)
        r["tflops"] = k["flops"] / t / 1e3 if t > 0 else 0.0
        r["gbps"] = k["bytes"] / t if t > 0 else 0.0
        rows.append(r)
    return rows


def roofline_of(rows, step_ns=None):
    """Dominant kernel family = the fp32 MFMA kernels (convolutions / GEMMs):
    algorithmic flops of all their launches in one step over the summed launch
    durations.  An event pair around every kernel serialises the stream and
    lengthens each launch (their sum exceeds the step time measured without
    them), so with `step_ns` given the per-kernel event durations are scaled to
    add up to that undisturbed step time; the rocprofv3 kernel trace of the
    same command gives the same per-kernel averages."""
    total = sum(r["ns"] for r in rows)
    scale = step_ns / total if step_ns and total > 0 else 1.0
    mf = [r for r in rows if r["bound"] == "mfma"]
    t = sum(r["ns"] for r in mf) * scale
    fl = sum(r["flops"] for r in mf)
    achieved = fl / t / 1e3 if t > 0 else 0.0
    n_launch = sum(1 for r in mf if r["ns"] > 0)       # the members of a fused region count once (the first carries the time)
    return dict(bound="mfma", achieved=round(achieved, 3), peak=PEAK_MFMA_F32_TFLOPS, unit="TFLOP/s",
                frac=round(achieved / PEAK_MFMA_F32_TFLOPS, 5), traffic=None,
                kernel="fp32 MFMA convolution / GEMM kernels (all their launches of one step)", launches=n_launch,
                avg_launch_us=round(t / max(n_launch, 1) / 1e3, 3),
                share_of_kernel_time=round(t / max(total * scale, 1), 4))


def measurer_spread(s, plan, repeats=5):
    """Run-to-run spread of the measurer: every distinct kernel of the plan priced `repeats` times with the
    cost log off; per kernel (max - min) / median, then the median and the largest of those figures."""
    import numpy as np
    from paper_2111_00655_amd import binding as B
    nocache = B.ProfileOpts(warmup=10, batches=5, min_batch_us=200, max_launches=500, no_cache=1)
    seen, rel = set(), []
    for k in plan.kernels():
        if k["name"].endswith("_alias"):
            continue
        key = B.clg_match_key(s.ctx, s.graph, k["match"])
        if key in seen:
            continue
        seen.add(key)
        c = [B.clg_profile_match(s.ctx, s.graph, k["match"], nocache) for _ in range(repeats)]
        rel.append(((max(c) - min(c)) / float(np.median(c)), k["name"], [int(x) for x in c]))
    vals = [r[0] for r in rel]
    worst = sorted(rel, reverse=True)[:3]
    return dict(kernels=len(rel), repeats=repeats, median_rel_spread=round(float(np.median(vals)), 4),
                p90_rel_spread=round(float(np.quantile(vals, 0.9)), 4), max_rel_spread=round(float(max(vals)), 4),
                widest=[dict(kernel=w[1], ns=w[2]) for w in worst])


def cpu_baseline(desc):
    """The oracle as it stands, one full forward pass on the host cores (and one on a single thread)."""
    from oracle.graph import Graph
    from oracle import ops
    g = Graph(desc)
    g.run()                                   # page in weights / warm the library
    t0 = time.perf_counter()
    g.run()
    dt = time.perf_counter() - t0
    n = ops.max_threads()
    ops.set_threads(1)
    t0 = time.perf_counter()
    g.run()
    dt1 = time.perf_counter() - t0
    ops.set_threads(n)
    return dict(value=round(dt * 1e3, 2), unit="ms", cores=n, kind="oracle",
                sample="one full batch-1 forward pass of the same graph (all layers), second of two runs",
                single_thread_ms=round(dt1 * 1e3, 2))


def oracle_us_per_group(desc, groups):
    """The oracle's time for each fused group (all host cores): every operator timed while the oracle evaluates the
    graph once (after one untimed pass), summed over the operators of the group."""
    from oracle.graph import Graph
    g = Graph(desc)
    g.run()
    _, secs = g.run_timed()
    return [sum(secs[v] for v in grp) * 1e6 for grp in groups]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--model", default="resnet50", help="headline workload (resnet50 | bert_base | ...)")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--dump", default="", help="write the per-kernel table to this JSON file")
    ap.add_argument("--table", default="", metavar="FILE",
                    help="write a text table of every fused kernel of a step: time, achieved TFLOP/s or GB/s, fraction of "
                         "the fp32 MFMA peak or of the HBM bandwidth")
    ap.add_argument("--cost-log", default="", help="cost-log file: reuse measured subgraph costs from it, add new ones")
    ap.add_argument("--ablation", action="store_true", help="also time the placement under each single MFMA kernel variant")
    ap.add_argument("--batch-sweep", default="", metavar="B1,B2,...",
                    help="also time ResNeXt-50 at these batch sizes (the paper's Fig. 8 varies the batch for this model)")
    ap.add_argument("--graph-level", default="", metavar="MODEL,...",
                    help="also run the graph-level evolutionary search (paper Sec. 4.3) on these workloads' op-level plans")
    ap.add_argument("--rules", action="store_true",
                    help="build the registry with the pattern generator from pattern rules instead of the listed patterns")
    ap.add_argument("--large-shapes", default="", metavar="FILE",
                    help="also price a few compute-bound single operators (large dense, batch-32 3x3 convolutions) under every "
                         "MFMA kernel variant with the library's measurer and write TFLOP/s per variant to FILE: what the "
                         "kernels reach where launch and memory latency do not bound them")
    ap.add_argument("--digits", default="", metavar="FILE",
                    help="graph-level digits: written to FILE after the search; with --passes-only read from it instead of searching")
    ap.add_argument("--passes-only", action="store_true",
                    help="for hardware-counter runs: op-level placement from the cost log, graph-level digits from --digits, then "
                         "nothing but warm-up + steps passes of the final plan (no per-kernel timing, graph replay, cold-cache "
                         "leg or other workloads), so that every dispatch of the run belongs to one of warmup + steps equal passes")
    ap.add_argument("--variants", default="", metavar="NAME,...",
                    help="register only these MFMA kernel-variant backends instead of all of them")
    ap.add_argument("--summary", default="", metavar="FILE",
                    help="write a short text summary of the run (headline figure, and whichever of --ablation, --batch-sweep, "
                         "--graph-level were asked for, and the measurer's run-to-run spread) with the command that made it")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MIB",
                    help="also run three plain device copies of MIB MiB (read MIB, write MIB): the known-size kernel "
                         "against which hardware byte counters of a profiled run are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: batch-1 inference of one graph is a dependency chain and "
              "nothing here shards across GPUs; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (torch.cuda.is_available() is False)", file=sys.stderr)
        sys.exit(2)
    import workloads as wl
    from paper_2111_00655_amd import binding as B

    variants = tuple(args.variants.split(",")) if args.variants else VARIANTS
    reg = wl.default_registry(variants, sepconv=True, attention=True)
    opts = B.ProfileOpts(warmup=10, batches=5, min_batch_us=200, max_launches=500)

    rules = ()
    if args.rules:
        from workloads import patterns as wp
        reg, rules = wp.rule_registry(VARIANTS)
    desc = wl.MODEL_BUILDERS[args.model](0)
    s, plan, costs, ids, timing = optimise(desc, reg, opts, args.cost_log, rules)
    timing["n_patterns"] = B.clg_num_patterns(s.ctx)
    if args.passes_only:
        digits = [int(c) for c in open(args.digits).read().strip()] if args.digits else [0] * plan.n_kernels
        plan.bind()
        plan.set_handover(digits, lanes=1)
        ms = time_steps(plan, args.steps, args.warmup)
        if args.calib_copy:
            n = args.calib_copy * 1024 * 1024 // 4
            src = torch.ones(n, dtype=torch.float32, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            torch.cuda.synchronize()
        print(json.dumps({"metric": f"batch-1 fp32 latency (ms) {args.model}", "value": round(ms, 4), "unit": "ms", "passes":
                          args.steps + args.warmup, "launches_per_pass": plan.n_launches,
                          "kernels": [k["name"] for k in plan.kernels()]}))
        return
    # op-level placement done; the graph-level search (Sec. 4.3) then decides which sibling kernels share a launch
    gl_main = graph_level(plan, max(50, args.steps // 2), args.warmup)
    if args.digits:
        with open(args.digits, "w") as f:
            f.write("".join(str(int(b)) for b in gl_main["digits"]) + "\n")
    timing["graph_level_s"] = gl_main["search_s"]
    ms_per_step = time_steps(plan, args.steps, args.warmup)
    rows = kernel_table(plan)
    roof = roofline_of(rows, ms_per_step * 1e6)
    roof["algorithmic_bytes"] = int(sum(r["bytes"] for r in rows if r["bound"] == "mfma"))
    roof["algorithmic_flops"] = int(sum(r["flops"] for r in rows if r["bound"] == "mfma"))
    tr = TRAFFIC.get(args.model)
    if tr and tr["sources"] == kernel_sources_fingerprint():
        roof["traffic"] = int(tr["fetch_bytes"] + tr["write_bytes"])      # bytes per step, same launches as `achieved`
    kernel_only_ms = sum(r["ns"] for r in rows) / 1e6
    empty_ns = B.clg_profile_empty(s.ctx)
    spread = measurer_spread(s, plan)
    graph_ms = graph_replay_ms(plan, args.steps, args.warmup)
    cold_ms = cold_cache_ms(plan)
    abl = ablation(desc, VARIANTS, opts, args.cost_log, max(20, args.steps // 2), args.warmup) if args.ablation else None

    extra = {}
    if not args.no_extra:
        for name in ("bert_base", "resnext50", "dcgan_b1", "dcgan_b64", "tiny_cnn", "nasnet_a", "resnet3d_50", "resnet50"):
            if name == args.model:
                continue
            d2 = wl.MODEL_BUILDERS[name](0)
            s2, p2, _, _, t2 = optimise(d2, reg, opts, "", rules)
            gl2 = graph_level(p2, max(20, args.steps // 2), args.warmup)
            ms2 = time_steps(p2, max(20, args.steps // 2), args.warmup)
            r2 = kernel_table(p2, reps=5)
            roof2 = roofline_of(r2, ms2 * 1e6)
            roof2["algorithmic_bytes"] = int(sum(r["bytes"] for r in r2 if r["bound"] == "mfma"))
            roof2["algorithmic_flops"] = int(sum(r["flops"] for r in r2 if r["bound"] == "mfma"))
            tr2 = TRAFFIC.get(name)
            if tr2 and tr2["sources"] == kernel_sources_fingerprint():
                roof2["traffic"] = int(tr2["fetch_bytes"] + tr2["write_bytes"])
            extra[name] = dict(ms_per_step=round(ms2, 4), cold_cache_ms=round(cold_cache_ms(p2, steps=10), 4), kernels=p2.n_launches,
                               kernel_only_ms=round(sum(r["ns"] for r in r2) / 1e6, 4),
                               mfma_tflops=roof2["achieved"], roofline=roof2, graph_level=gl2, weights=weight_memory(p2),
                               optimise_s=round(sum(
                                   v for k, v in t2.items() if k.endswith("_s")) + gl2["search_s"], 2))
            p2.destroy()
            s2.close()

    sweep = None
    if args.batch_sweep:
        sweep = {}
        for b in [int(x) for x in args.batch_sweep.split(",")]:
            d2 = wl.resnext50(0, batch=b)
            s2, p2, _, _, t2 = optimise(d2, reg, opts, "", rules)
            ms2 = time_steps(p2, max(20, args.steps // 4), args.warmup)
            sweep[str(b)] = dict(ms_per_step=round(ms2, 4), images_per_s=round(b / ms2 * 1e3, 1), kernels=p2.n_kernels)
            p2.destroy()
            s2.close()

    large = None
    if args.large_shapes:
        large = large_shapes(args.large_shapes)

    graph_level_rows = None
    if args.graph_level:
        graph_level_rows = {}
        for name in args.graph_level.split(","):
            if name == args.model:
                graph_level_rows[name] = gl_main
                continue
            d2 = wl.MODEL_BUILDERS[name](0)
            s2, p2, _, _, _ = optimise(d2, reg, opts, "", rules)
            graph_level_rows[name] = graph_level(p2, max(50, args.steps // 2), args.warmup)
            p2.destroy()
            s2.close()

    cpu = None if args.no_cpu else cpu_baseline(desc)

    if args.calib_copy:
        n = args.calib_copy * 1024 * 1024 // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.table:
        scale = ms_per_step * 1e6 / sum(r["ns"] for r in rows)
        cpu_us = None
        if not args.no_cpu:
            cpu_us = oracle_us_per_group(desc, [list(s.matches[r["match"]].nodes[:s.matches[r["match"]].n_nodes]) for r in rows])
        lines = [f"{args.model} batch 1 fp32, one MI355X: the {len(rows)} fused kernels of one step in execution order.",
                 f"Durations: HIP event pair around every launch, scaled by {scale:.3f} so that they add up to the step time "
                 f"measured without the events ({ms_per_step * 1e3:.1f} us).",
                 f"Peaks: fp32 MFMA {PEAK_MFMA_F32_TFLOPS} TFLOP/s, HBM {PEAK_HBM_GBPS} GB/s.  flops / bytes are the operator's own "
                 "(no padding or tile waste; every operand and the output once).",
                 ] + (["oracle us: the CPU oracle's time for the same fused group (sum over its operators, all host cores)."]
                      if cpu_us else []) + [
                 "",
                 f"{'#':>3s} {'kernel':34s} {'bound':5s} {'us':>7s} {'MFLOP':>9s} {'KB':>9s} {'TFLOP/s':>8s} {'GB/s':>8s} {'of peak':>8s}"
                 + (f" {'oracle us':>10s}" if cpu_us else "")]
        if len(rows) > 150:
            # a long kernel list (NasNet-A): one line per kernel name instead, most expensive first
            agg = {}
            for i, r in enumerate(rows):
                a = agg.setdefault(r["name"], dict(bound=r["bound"], n=0, ns=0.0, flops=0.0, bytes=0.0, cpu=0.0))
                a["n"] += 1
                a["ns"] += r["ns"] * scale
                a["flops"] += r["flops"]
                a["bytes"] += r["bytes"]
                a["cpu"] += cpu_us[i] if cpu_us else 0.0
            lines = lines[:-1]
            lines[0] = f"{args.model} batch 1 fp32, one MI355X: the {len(rows)} fused kernels of one step summed by kernel name."
            lines.append(f"{'kernel':34s} {'bound':5s} {'count':>5s} {'sum us':>8s} {'avg us':>7s} {'MFLOP':>9s} {'KB':>10s} "
                         f"{'TFLOP/s':>8s} {'GB/s':>8s}" + (f" {'oracle us':>10s}" if cpu_us else ""))
            for name, a in sorted(agg.items(), key=lambda kv: -kv[1]["ns"]):
                t = max(a["ns"], 1.0)
                lines.append(f"{name[:34]:34s} {a['bound']:5s} {a['n']:5d} {a['ns'] / 1e3:8.1f} {a['ns'] / a['n'] / 1e3:7.2f} "
                             f"{a['flops'] / 1e6:9.1f} {a['bytes'] / 1e3:10.1f} {a['flops'] / t / 1e3:8.3f} {a['bytes'] / t:8.1f}"
                             + (f" {a['cpu']:10.0f}" if cpu_us else ""))
        else:
            for i, r in enumerate(rows):
                t = r["ns"] * scale
                tf, gb = (r["flops"] / t / 1e3, r["bytes"] / t) if t > 0 else (0.0, 0.0)
                frac = tf / PEAK_MFMA_F32_TFLOPS if r["bound"] == "mfma" else gb / PEAK_HBM_GBPS
                lines.append(f"{i:3d} {r['name'][:34]:34s} {r['bound']:5s} {t / 1e3:7.2f} {r['flops'] / 1e6:9.1f} "
                             f"{r['bytes'] / 1e3:9.1f} {tf:8.2f} {gb:8.1f} {frac:8.4f}"
                             + (f" {cpu_us[i]:10.0f}" if cpu_us else ""))
        if cpu_us and len(rows) > 150:
            lines.append(f"{'sum':34s} {'':5s} {len(rows):5d} {sum(r['ns'] for r in rows) * scale / 1e3:8.1f} {'':7s} {'':9s} {'':10s} {'':8s} {'':8s} "
                         f"{sum(cpu_us):10.0f}")
        elif cpu_us:
            lines.append(f"{'':3s} {'sum':34s} {'':5s} {sum(r['ns'] for r in rows) * scale / 1e3:7.2f} {'':9s} {'':9s} {'':8s} {'':8s} {'':8s} "
                         f"{sum(cpu_us):10.0f}")
        os.makedirs(os.path.dirname(os.path.abspath(args.table)), exist_ok=True)
        with open(args.table, "w") as f:
            f.write("\n".join(lines) + "\n")

    if args.dump:
        os.makedirs(os.path.dirname(os.path.abspath(args.dump)), exist_ok=True)
        with open(args.dump, "w") as f:
            json.dump(dict(model=args.model, kernels=rows, timing=timing), f, indent=1)

    out = {
        "metric": f"batch-1 fp32 latency (ms) {args.model}",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.model} batch 1 fp32, seeded random weights, placement from the "
                               "library's measurer + DP over the igemm tile variants and the direct, rowwise, eltwise, "
                               "separable-convolution and attention kernel families",
                   "placement": "op-level dynamic programme, then graph-level evolutionary search over regions",
                   "kernels_per_step": plan.n_launches},
        "roofline": roof,
        "cpu_baseline": cpu,
        "kernel_only_ms": round(kernel_only_ms, 4),
        "graph_replay_ms": None if graph_ms is None else round(graph_ms, 4),
        "cold_cache_ms": round(cold_ms, 4),
        "ablation_ms": abl,
        "resnext50_batch_sweep": sweep,
        "large_shapes_tflops": large,
        "graph_level": gl_main,
        "graph_level_search": graph_level_rows,
        "weights": weight_memory(plan),
        "empty_launch_ns": int(empty_ns),
        "measurer_spread": spread,
        "optimise": {k: (round(v, 4) if isinstance(v, float) else v) for k, v in timing.items()},
        "other_workloads": extra,
    }
    print(json.dumps(out))
    if args.summary:
        lines = [f"{args.model} batch 1 fp32 on one MI355X, placement searched over all kernel-variant backends: "
                 f"{ms_per_step:.4f} ms per step, {plan.n_launches} launches (op-level placement alone: "
                 f"{gl_main['op_level_ms']:.4f} ms, {gl_main['launches_before']} launches; its cost table predicted "
                 f"{timing['predicted_ms']:.4f} ms).",
                 "command: python3 bench.py " + " ".join(sys.argv[1:]), ""]
        if abl is not None:
            lines += ["Placement under a single MFMA kernel variant (every fused-operator kind on that one backend; glue on",
                      "the direct / rowwise / eltwise families as always), ms per step; '-' = the variant alone cannot cover the graph:",
                      f"  {'search over all variants':28s} {gl_main['op_level_ms']:8.4f}   (op-level placement; {ms_per_step:.4f} after the graph-level search)"]
            lines += [f"  {v:28s} {(f'{t:8.4f}' if t is not None else '       -')}" for v, t in abl.items()]
            best = min((t for t in abl.values() if t is not None), default=None)
            if best is not None:
                lines += [f"  best single variant / searched mix (both op-level) = {best / gl_main['op_level_ms']:.3f}", ""]
        if sweep is not None:
            lines += ["ResNeXt-50 32x4d at growing batch (placement searched anew per batch size):",
                      f"  {'batch':>5s} {'ms/step':>9s} {'images/s':>9s} {'launches':>8s}"]
            lines += [f"  {b:>5s} {v['ms_per_step']:9.4f} {v['images_per_s']:9.1f} {v['kernels']:8d}" for b, v in sweep.items()]
            lines += [""]
        if graph_level_rows is not None:
            lines += ["Graph-level search (evolutionary, seeded with the op-level placement; region backend: the handed-over",
                      "members of a region of independent kernels of one kind share one launch), ms per step before / after:",
                      f"  {'workload':12s} {'op-level ms':>11s} {'graph-level ms':>14s} {'gain':>6s} {'launches':>9s} {'digits=1':>8s} {'strings':>7s} {'search s':>8s}"]
            for n, v in graph_level_rows.items():
                lines.append(f"  {n:12s} {v['op_level_ms']:11.4f} {v['graph_level_ms']:14.4f} {v['op_level_ms'] / v['graph_level_ms']:6.3f} "
                             f"{str(v.get('launches_before', '')) + '->' + str(v.get('launches_after', '')):>9s} {v['handed_over']:8d} "
                             f"{v['strings_priced']:7d} {v['search_s']:8.2f}")
            lines += [""]
        lines += [f"Measurer: {spread['kernels']} distinct kernels priced {spread['repeats']} times each with the cost log off; "
                  f"(max - min) / median per kernel: median {spread['median_rel_spread']:.4f}, 90th percentile "
                  f"{spread['p90_rel_spread']:.4f}, largest {spread['max_rel_spread']:.4f}."]
        os.makedirs(os.path.dirname(os.path.abspath(args.summary)), exist_ok=True)
        with open(args.summary, "w") as f:
            f.write("\n".join(lines) + "\n")
    plan.destroy()
    s.close()


if __name__ == "__main__":
    main()
