#!/usr/bin/env python3
"""Benchmark of the reversible backward pass on one MI355X.

One "step" is one whole backward pass of the stack (every recompute and every
gradient kernel of all N blocks) over one synthetic batch already resident in
HBM.  The headline value is the PaReprop schedule's samples/s on the Rev-ViT-B
shaped workload (batch 64); the sequential Reprop schedule, the two chains on
their own, the per-family kernel times and the CPU oracle are reported beside
it on the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vit_b]
    python bench.py --sweep-batch 1,2,4,8,16,32,64,128,256     # throughput and memory against batch size
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak
PEAK_FP32_TFLOPS = 157.3      # vector/matrix fp32
PEAK_HBM_GBS = 8000.0



def profiled_traffic(workload, family):
    """Fabric-side bytes per launch of a kernel family (rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by what
    the same counter reads for a plain 256 MiB device copy), read from the tracked counter summary of this
    workload: profiles/<workload>_backward_reprop_hbm_traffic_pmc.txt, whose header holds the two profiler
    commands.  It is an offline measurement, so the source file travels with the value; (None, None) when no
    summary of this workload and family is tracked."""
    import re
    path = os.path.join(ROOT, "profiles", f"{workload}_backward_reprop_hbm_traffic_pmc.txt")
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m = re.search(rf"^{re.escape(family)} family:.*=\s*([0-9.eE+-]+)\s*bytes", text, flags=re.M)
    return (float(m.group(1)), os.path.relpath(path, ROOT)) if m else (None, None)



def algorithmic_flops(cfg):
    """Backward-path flops: per block one forward unit of recomputation and two of
    gradient work (the paper's cost model, Sec. 3.3), a forward unit being the four
    linear maps plus the two attention contractions."""
    M = cfg["batch"] * cfg["seq_len"]
    D, Dm, T = cfg["d_model"], cfg["d_mlp"], cfg["seq_len"]
    fwd_unit = 2 * M * D * (3 * D + D + 2 * Dm) + 4 * M * T * D
    return 3 * cfg["n_blocks"] * fwd_unit


def memory_model(B, c, cfg):
    """Workspace bytes of the two reversible schedules as the library sizes them, and what
    backpropagation with stored activations would need with the same kernels: every block keeps its
    activation slot and its two output streams instead of one (or two) slots and two (or three)
    residual levels being reused."""
    M = cfg["batch"] * cfg["seq_len"]
    slot = B.rev_stack_slot_bytes(c)
    level = 2 * M * cfg["d_model"] * 4
    reprop = B.rev_stack_workspace_bytes_reprop(c)
    pareprop = B.rev_stack_workspace_bytes(c)
    N = cfg["n_blocks"]
    stored = reprop + (N - 1) * slot + max(N - 2, 0) * level
    return {"reprop_bytes": reprop, "pareprop_bytes": pareprop, "stored_activation_bytes": stored,
            "slot_bytes": slot, "pareprop_over_reprop": pareprop / reprop, "stored_over_reprop": stored / reprop}


def sweep_batch(args, cfg, B, synth, torch, np):
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    batches = [int(b) for b in args.sweep_batch.split(",") if b]
    flat = synth.make_params(cfg, seed=0)
    rows = []
    main_s = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    for b in batches:
        cb = dict(cfg, batch=b)
        c = B.make_cfg(**cb)
        params = torch.from_numpy(flat).cuda().to(B.param_dtype(c))
        x, dy1, dy2 = synth.make_inputs(cb, seed=0, batch=b)
        X, dY1, dY2 = (torch.from_numpy(a).cuda() for a in (x, dy1, dy2))
        ws = B.alloc_workspace(c)
        Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws)
        out = {}
        out.update(B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws))
        torch.cuda.synchronize()
        res = {}
        for name, fn in (("pareprop", lambda: B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side,
                                                                             workspace=ws, out=out)),
                         ("reprop", lambda: B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2,
                                                                         workspace=ws, out=out))):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            ev = []
            for _ in range(args.steps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(main_s)
                fn()
                e1.record(main_s)
                ev.append((e0, e1))
            torch.cuda.synchronize()
            ms = np.array([a.elapsed_time(z) for a, z in ev])
            res[name] = {"ms_median": float(np.median(ms)), "ms_mean": float(ms.mean()), "ms_std": float(ms.std()),
                         "samples_per_s": b / (float(np.median(ms)) * 1e-3)}
        row = {"batch": b, **res, "pareprop_over_reprop": res["pareprop"]["samples_per_s"] / res["reprop"]["samples_per_s"],
               "memory": memory_model(B, c, cb)}
        rows.append(row)
        print(f"# batch {b}: pareprop {res['pareprop']['samples_per_s']:.1f}/s reprop {res['reprop']['samples_per_s']:.1f}/s "
              f"x{row['pareprop_over_reprop']:.3f}  ws {row['memory']['pareprop_bytes'] / 2**20:.0f} / "
              f"{row['memory']['reprop_bytes'] / 2**20:.0f} MiB, stored {row['memory']['stored_activation_bytes'] / 2**20:.0f} MiB",
              file=sys.stderr, flush=True)
        del ws, X, dY1, dY2, Y1, Y2, out, params
        torch.cuda.empty_cache()
    best = max(rows, key=lambda r: r["pareprop"]["samples_per_s"])
    print(json.dumps({"metric": f"reversible backward samples/s against batch size, {args.workload}",
                      "value": best["pareprop"]["samples_per_s"], "unit": "samples/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": best["pareprop"]["ms_median"],
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg["mode"],
                      "data": "synthetic",
                      "config": {"workload": f"{args.workload}, batch sweep", "best_batch": best["batch"]},
                      "sweep": rows}))


def bench_hierarchy(args, hier, B, synth, torch, np):
    """Hierarchical (window-attention shaped) workload.  One step is the backward pass of the whole
    hierarchy, last stage first: the reversible backward of a stage's stack over its attention windows,
    then the backward of the stage transition below it (stream averaging + patch merging), whose input
    cotangents are the output cotangents of the next stack.  The stage outputs the transitions need are
    kept from one untimed forward pass, as a training step would have them."""
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    main_s = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    stages = []
    merges = []
    mcfgs = synth.merge_cfgs(hier, fusion=args.fusion)
    X1 = X2 = None
    for si, cfg in enumerate(hier["stages"]):
        c = B.make_cfg(**cfg)
        params = torch.from_numpy(synth.make_params(cfg, seed=si)).cuda().to(B.param_dtype(c))
        shape = (cfg["batch"], cfg["seq_len"], cfg["d_model"])
        if si == 0:
            x, _, _ = synth.make_inputs(cfg, seed=si)
            X1 = X2 = torch.from_numpy(x).cuda()
        ws = B.alloc_workspace(c)
        Y1, Y2 = B.rev_stack_forward(c, params, X1.view(shape), X2.view(shape), workspace=ws)
        out = {}
        st = dict(cfg=cfg, c=c, params=params, Y1=Y1, Y2=Y2, ws=ws, out=out)
        stages.append(st)
        if si + 1 < len(hier["stages"]):
            mc = B.make_merge_cfg(**mcfgs[si])
            mp = torch.from_numpy(synth.make_merge_params(mcfgs[si], seed=si)).cuda().to(B.param_dtype(mc))
            mws = torch.empty(B.rev_merge_workspace_bytes(mc), dtype=torch.uint8, device="cuda")
            rows = cfg["batch"] * cfg["seq_len"]
            merged = B.rev_merge_forward(mc, mp, Y1.view(rows, -1), Y2.view(rows, -1), workspace=mws)
            merges.append(dict(c=mc, params=mp, ws=mws, out={}, rows=rows))
            X1 = X2 = merged
    # cotangents of the last stage's outputs
    _, dy1, dy2 = synth.make_inputs(hier["stages"][-1], seed=len(stages) - 1)
    top = (torch.from_numpy(dy1).cuda(), torch.from_numpy(dy2).cuda())
    torch.cuda.synchronize()

    def stage_backward(si, schedule, dY1, dY2):
        st = stages[si]
        if schedule == "pareprop":
            return B.rev_stack_backward_pareprop(st["c"], st["params"], st["Y1"], st["Y2"], dY1, dY2, side,
                                                 workspace=st["ws"], out=st["out"])
        return B.rev_stack_backward_reprop(st["c"], st["params"], st["Y1"], st["Y2"], dY1, dY2,
                                           workspace=st["ws"], out=st["out"])

    def merge_backward(mi, dA, dB):
        m, below = merges[mi], stages[mi]
        rows = m["rows"]
        return B.rev_merge_backward(m["c"], m["params"], below["Y1"].view(rows, -1), below["Y2"].view(rows, -1),
                                    dA.view(rows // 4, -1), dB.view(rows // 4, -1), workspace=m["ws"], out=m["out"])

    def run(schedule):
        dY1, dY2 = top
        for si in reversed(range(len(stages))):
            res = stage_backward(si, schedule, dY1, dY2)
            stages[si]["out"].update(res)
            if si > 0:
                mres = merge_backward(si - 1, res["dX1"], res["dX2"])
                merges[si - 1]["out"].update(mres)
                shape = stages[si - 1]["Y1"].shape
                dY1, dY2 = mres["dX1"].view(shape), mres["dX2"].view(shape)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = []
        t0 = time.perf_counter()
        for _ in range(steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main_s)
            fn()
            e1.record(main_s)
            ev.append((e0, e1))
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, np.array([a.elapsed_time(z) for a, z in ev])

    wall_p, ms_p = timed(lambda: run("pareprop"), args.steps, args.warmup)
    wall_r, ms_r = timed(lambda: run("reprop"), args.steps, args.warmup)
    finite = all(bool(torch.isfinite(st["out"]["dparams"]).all()) for st in stages) and \
        all(bool(torch.isfinite(m["out"]["dparams"]).all()) for m in merges)
    # per-stage and per-transition times, each run alone with the cotangents the full pass left behind
    grads_in = []
    for si in range(len(stages)):
        if si + 1 == len(stages):
            grads_in.append(top)
        else:
            shape = stages[si]["Y1"].shape
            grads_in.append((merges[si]["out"]["dX1"].clone().view(shape), merges[si]["out"]["dX2"].clone().view(shape)))
    per_stage = []
    few = max(5, args.steps // 3)
    for si, st in enumerate(stages):
        d1, d2 = grads_in[si]
        _, a = timed(lambda: stage_backward(si, "pareprop", d1, d2), few, 2)
        _, b = timed(lambda: stage_backward(si, "reprop", d1, d2), few, 2)
        cfg = st["cfg"]
        B.rev_profile_begin()
        for _ in range(3):
            stage_backward(si, "reprop", d1, d2)
        fam = {k: round(ms / 3, 4) for k, (ms, n, work, is_flops) in B.rev_profile_end().items() if n}
        entry = {"stage": si + 1, "family_ms": fam, "blocks": cfg["n_blocks"], "d_model": cfg["d_model"], "windows": cfg["batch"],
                 "tokens": cfg["seq_len"], "pareprop_ms": float(np.median(a)), "reprop_ms": float(np.median(b)),
                 "algorithmic_tflop": algorithmic_flops(cfg) / 1e12}
        if si > 0:
            dA, dB = st["out"]["dX1"].clone(), st["out"]["dX2"].clone()
            _, t = timed(lambda: merge_backward(si - 1, dA, dB), few, 2)
            entry["transition_below_ms"] = float(np.median(t))
        per_stage.append(entry)
    images = hier["images"]
    flops = sum(algorithmic_flops(st["cfg"]) for st in stages)
    value = images * args.steps / wall_p
    print(json.dumps({
        "metric": f"reversible backward images/s (PaReprop schedule), {args.workload}-shaped hierarchy",
        "value": value, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_p / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {len(stages)} stages of window-attention shaped reversible stacks joined by "
                               f"{len(merges)} stage transitions (stream fusion by {'a small MLP' if args.fusion == 'mlp' else 'averaging'} "
                               f"+ patch merging), {images} images of 224x224",
                   "schedule": "pareprop (2 HIP streams)"},
        "pareprop": {"images_per_s": value, "ms_median": float(np.median(ms_p)), "ms_std": float(ms_p.std())},
        "reprop": {"images_per_s": images * args.steps / wall_r, "ms_median": float(np.median(ms_r)),
                   "ms_std": float(ms_r.std())},
        "pareprop_over_reprop": float(np.median(ms_r)) / float(np.median(ms_p)),
        "algorithmic_tflop_per_step": flops / 1e12,
        "mfma_fraction_whole_path": flops / (float(np.median(ms_p)) * 1e-3) / (PEAK_BF16_TFLOPS * 1e12),
        "finite_gradients": finite,
        "stages": per_stage}))


def both_schedules(name, B, synth, torch, np, steps, warmup):
    """PaReprop and Reprop backward passes of one workload: samples/s of each, their ratio and the share of the
    bf16 (fp32 for the tiny workload) peak over the whole pass."""
    cfg = dict(synth.CONFIGS[name])
    c = B.make_cfg(**cfg)
    params = torch.from_numpy(synth.make_params(cfg, seed=0)).cuda().to(B.param_dtype(c))
    x, dy1, dy2 = synth.make_inputs(cfg, seed=0)
    X, dY1, dY2 = (torch.from_numpy(a).cuda() for a in (x, dy1, dy2))
    ws = B.alloc_workspace(c)
    Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws)
    main_s = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    out = {}
    out.update(B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws))
    torch.cuda.synchronize()
    med = {}
    for sched, fn in (("pareprop", lambda: B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side,
                                                                          workspace=ws, out=out)),
                      ("reprop", lambda: B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws, out=out))):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = []
        for _ in range(steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main_s)
            fn()
            e1.record(main_s)
            ev.append((e0, e1))
        torch.cuda.synchronize()
        med[sched] = float(np.median([a.elapsed_time(z) for a, z in ev]))
    peak = PEAK_BF16_TFLOPS if cfg["mode"] == "bf16" else PEAK_FP32_TFLOPS
    flops = algorithmic_flops(cfg)
    res = {"workload": f"{cfg['n_blocks']} blocks, D={cfg['d_model']}, H={cfg['n_heads']}, Dm={cfg['d_mlp']}, "
                       f"T={cfg['seq_len']}, batch={cfg['batch']}, {cfg['mode']}",
           "pareprop": cfg["batch"] / (med["pareprop"] * 1e-3), "reprop": cfg["batch"] / (med["reprop"] * 1e-3),
           "pareprop_ms": med["pareprop"], "reprop_ms": med["reprop"], "ratio": med["reprop"] / med["pareprop"],
           "mfma_fraction_whole_path": flops / (med["pareprop"] * 1e-3) / (peak * 1e12),
           "finite": bool(torch.isfinite(out["dparams"]).all().item())}
    del ws, X, dY1, dY2, Y1, Y2, out, params
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vit_b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", choices=["all", "reprop", "pareprop"], default="all",
                    help="restrict the run to one schedule (for profiler runs); the JSON line then lacks the other")
    ap.add_argument("--fusion", choices=["average", "mlp"], default="average",
                    help="hierarchical workloads: how a stage transition fuses the two streams (Sec. 3.4)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short both-schedules runs on the other workloads")
    ap.add_argument("--cpu-samples", type=int, default=0, help="samples the oracle is timed on (0 = auto)")
    ap.add_argument("--sweep-batch", default="",
                    help="comma-separated batch sizes: time both schedules and report workspace bytes at each "
                         "(the paper's throughput-vs-batch and memory-vs-batch comparisons); replaces the default run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2306_09342_amd import binding as B
    from paper_2306_09342_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload in synth.HIERARCHIES:
        bench_hierarchy(args, synth.HIERARCHIES[args.workload], B, synth, torch, np)
        return
    cfg = dict(synth.CONFIGS[args.workload])
    if args.sweep_batch:
        sweep_batch(args, cfg, B, synth, torch, np)
        return
    c = B.make_cfg(**cfg)
    Bsz = cfg["batch"]

    flat = synth.make_params(cfg, seed=0)
    x, dy1, dy2 = synth.make_inputs(cfg, seed=0)
    params = torch.from_numpy(flat).cuda().to(B.param_dtype(c))
    X = torch.from_numpy(x).cuda()
    dY1 = torch.from_numpy(dy1).cuda()
    dY2 = torch.from_numpy(dy2).cuda()
    ws = B.alloc_workspace(c)
    Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws)      # untimed
    torch.cuda.synchronize()

    main_s = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    out = {}

    def reprop():
        return B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws, out=out)

    def pareprop():
        return B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws, out=out)

    def chain(which):
        return lambda: B.rev_stack_backward_chain(c, params, Y1, Y2, dY1, dY2, which, workspace=ws, out=out)

    out.update(reprop())
    torch.cuda.synchronize()

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        per = []
        t0 = time.perf_counter()
        for _ in range(steps):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(main_s)
            fn()
            e1.record(main_s)
            per.append((e0, e1))
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = np.array([a.elapsed_time(b) for a, b in per])
        return wall, ms

    def calibration_copy():
        # one plain device copy of known size (256 MiB read + 256 MiB written): the yardstick the HBM
        # byte counters of a profiler run are scaled by
        cal_src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()

    if args.only != "all":
        fn = reprop if args.only == "reprop" else pareprop
        wall, ms = timed(fn, args.steps, args.warmup)
        calibration_copy()
        print(json.dumps({"metric": f"reversible backward samples/s ({args.only} only), {args.workload}",
                          "value": Bsz * args.steps / wall, "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": cfg["mode"], "data": "synthetic",
                          "config": {"workload": args.workload, "schedule": args.only},
                          "ms_median": float(np.median(ms))}))
        return

    wall_p, ms_p = timed(pareprop, args.steps, args.warmup)
    wall_r, ms_r = timed(reprop, args.steps, args.warmup)
    _, ms_rc = timed(chain(0), max(3, args.steps // 3), 2)
    _, ms_vc = timed(chain(1), max(3, args.steps // 3), 2)

    # per-family kernel times: HIP events around every launch, on the launching stream (Reprop order)
    B.rev_profile_begin()
    prof_steps = max(2, min(5, args.steps))
    for _ in range(prof_steps):
        reprop()
    fam = B.rev_profile_end()

    calibration_copy()

    def measured_peaks():
        # what this machine reaches on the two textbook yardsticks, so that fractions can be read against
        # achievable as well as nominal peaks: a streaming device copy and a long square bf16 GEMM
        # from the vendor library (torch.matmul); neither is part of the path
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        a = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
        b = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
        res = {}
        for name, fn, work in (("copy_GBs", lambda: dst.copy_(src), 2 * src.numel() * 4 / 1e9),
                               ("library_gemm_bf16_8192_TFLOPs", lambda: torch.matmul(a, b.t()), 2 * 8192 ** 3 / 1e12)):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                fn()
            e1.record()
            torch.cuda.synchronize()
            res[name] = work / (e0.elapsed_time(e1) / 10 * 1e-3)
        del src, dst, a, b
        # the same library on the GEMM shapes of this workload (plain products: no bias, GELU, residual or
        # column sums, which the path's kernels fuse), aggregated like the kernel families above:
        # total flops / total time of one block's launches
        M, D, Dm = cfg["batch"] * cfg["seq_len"], cfg["d_model"], cfg["d_mlp"]
        bf = dict(device="cuda", dtype=torch.bfloat16)

        def lib_family(shapes, make):
            t_us, fl = 0.0, 0.0
            for N, K in shapes:
                fn = make(N, K)
                for _ in range(3):
                    fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                t_us += e0.elapsed_time(e1) / 10 * 1e3
                fl += 2.0 * M * N * K
            return fl / t_us * 1e-6

        def nt(N, K):          # activations [M, K] x weights [N, K]^T
            x, w = torch.randn(M, K, **bf), torch.randn(N, K, **bf)
            return lambda: torch.matmul(x, w.t())

        def nn(N, K):          # output cotangents [M, K] x weights [K, N]
            x, w = torch.randn(M, K, **bf), torch.randn(K, N, **bf)
            return lambda: torch.matmul(x, w)

        def tn(N, K):          # weight gradient [N, K] = cotangents [M, N]^T x activations [M, K]
            g, x = torch.randn(M, N, **bf), torch.randn(M, K, **bf)
            return lambda: torch.matmul(g.t(), x)

        fwd = [(3 * D, D), (D, D), (Dm, D), (D, Dm)]                 # qkv, proj, fc1, fc2
        bwd = [(D, 3 * D), (D, D), (D, Dm), (Dm, D)]                 # their input gradients
        t_nt, t_nn = lib_family(fwd, nt), lib_family(bwd, nn)
        res["library_gemm_workload_shapes_TFLOPs"] = {
            "activation_products": t_nt, "input_gradients": t_nn, "weight_gradients": lib_family(fwd, tn),
            "note": "torch.matmul (vendor library) on this workload's own GEMM shapes, plain products without the "
                    "epilogues the path's kernels fuse; compare with kernel_families gemm_nt (both of the first two) "
                    "and gemm_wgrad"}
        return res

    peaks = measured_peaks()

    flops = algorithmic_flops(cfg)
    ms_step = wall_p / args.steps * 1e3
    value = Bsz * args.steps / wall_p
    reprop_value = Bsz * args.steps / wall_r
    peak = PEAK_BF16_TFLOPS if cfg["mode"] == "bf16" else PEAK_FP32_TFLOPS

    families = {}
    for name, (ms, n, work, is_flops) in fam.items():
        if n == 0:
            continue
        rate = work / (ms * 1e-3) if ms > 0 else 0.0
        families[name] = {"ms_per_step": ms / prof_steps, "launches_per_step": n / prof_steps,
                          ("tflops" if is_flops else "gbs"): rate / (1e12 if is_flops else 1e9)}
    # dominant kernel family = the one with most time
    dom = max((k for k in families), key=lambda k: families[k]["ms_per_step"])
    ms_d, n_d, work_d, is_flops_d = fam[dom]
    achieved = work_d / (ms_d * 1e-3) / (1e12 if is_flops_d else 1e9)
    traffic, traffic_src = profiled_traffic(args.workload, dom)
    roofline = {
        "kernel": dom,
        "bound": "mfma" if is_flops_d else "hbm",
        "achieved": achieved,
        "peak": peak if is_flops_d else PEAK_HBM_GBS,
        "unit": "TFLOP/s" if is_flops_d else "GB/s",
        "frac": achieved / (peak if is_flops_d else PEAK_HBM_GBS),
        "avg_launch_ms": ms_d / n_d,
        "work_per_launch": work_d / n_d,
        "traffic": traffic,
        "traffic_source": traffic_src,
        "launches_per_step": n_d / prof_steps,
        "note": "family average over all launches of the dominant kernel family in a Reprop pass, each "
                "bracketed by HIP events on its own stream",
    }

    hidden = (float(np.median(ms_r)) - float(np.median(ms_p))) / float(np.median(ms_rc))
    line = {
        # the headline metric as named for this path: `value` is the PaReprop schedule's samples/s, the Reprop
        # figure and the matrix-core fractions are on the same line ("reprop", "mfma_fraction_whole_path", "roofline")
        "metric": "reversible backward samples/s (PaReprop vs Reprop), Rev-ViT-B bs=64; MFMA util"
                  if args.workload == "vit_b" else f"reversible backward samples/s (PaReprop vs Reprop), {args.workload}; MFMA util",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["mode"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg['n_blocks']} blocks, D={cfg['d_model']}, H={cfg['n_heads']}, "
                               f"Dm={cfg['d_mlp']}, T={cfg['seq_len']}, batch={Bsz}",
                   "schedule": "pareprop (2 HIP streams)", "seed": 0},
        "pareprop": {"samples_per_s": value, "ms_mean": float(ms_p.mean()), "ms_std": float(ms_p.std()),
                     "ms_median": float(np.median(ms_p))},
        "reprop": {"samples_per_s": reprop_value, "ms_mean": float(ms_r.mean()), "ms_std": float(ms_r.std()),
                   "ms_median": float(np.median(ms_r))},
        "pareprop_over_reprop": value / reprop_value,
        "recompute_chain_ms": float(np.median(ms_rc)), "gradient_chain_ms": float(np.median(ms_vc)),
        "hidden_recompute_fraction": hidden,
        # the longer chain alone bounds the parallel schedule from below; what the pass takes beyond it is the
        # part of the shorter chain that is still exposed
        "exposed_beyond_longer_chain_ms": float(np.median(ms_p)) - max(float(np.median(ms_rc)), float(np.median(ms_vc))),
        "algorithmic_tflop_per_step": flops / 1e12,
        "mfma_fraction_whole_path": {"pareprop": flops / (float(np.median(ms_p)) * 1e-3) / (peak * 1e12),
                                     "reprop": flops / (float(np.median(ms_r)) * 1e-3) / (peak * 1e12)},
        "kernel_families": families,
        "roofline": roofline,
        "measured_peaks": peaks,
        "memory": memory_model(B, c, cfg),
        "workspace_bytes": int(ws.numel()),
        "paper_context": "paper reports whole-training-step gains only (A100 80GB, precision unstated): ViT ~0%, "
                         "up to +20% on Swin; no backward-only number",
    }

    # ---- both schedules on the other workloads of the comparison (shorter runs; the headline stays the
    # workload named above)
    if args.workload == "vit_b" and not args.no_other_configs:
        line["other_configs"] = {}
        for name in ("tiny", "vit_s", "roberta_base", "vit_h"):
            line["other_configs"][name] = both_schedules(name, B, synth, torch, np, steps=20, warmup=5)

    # ---- whole training step (the quantity the paper's throughput figures are about): forward of
    # the stack, reversible backward, AdamW update of every parameter; dY stays the fixed synthetic
    # cotangent (no head / loss), the weights really change from step to step
    master = params.float().clone()
    mom1, mom2 = torch.zeros_like(master), torch.zeros_like(master)
    Yt1, Yt2 = torch.empty_like(Y1), torch.empty_like(Y2)
    tstep = [0]

    def train_step(schedule):
        def fn():
            tstep[0] += 1
            B.rev_stack_forward(c, params, X, X, workspace=ws, Y1=Yt1, Y2=Yt2)
            if schedule == "pareprop":
                B.rev_stack_backward_pareprop(c, params, Yt1, Yt2, dY1, dY2, side, workspace=ws, out=out)
            else:
                B.rev_stack_backward_reprop(c, params, Yt1, Yt2, dY1, dY2, workspace=ws, out=out)
            B.rev_adamw_step(master, out["dparams"], mom1, mom2, tstep[0], lr=1e-5,
                             params_bf16=params if cfg["mode"] == "bf16" else None)
            if cfg["mode"] != "bf16":
                params.copy_(master)
        return fn

    tsteps = max(5, args.steps // 2)
    _, ms_tp = timed(train_step("pareprop"), tsteps, 3)
    _, ms_tr = timed(train_step("reprop"), tsteps, 3)
    _, ms_fwd = timed(lambda: B.rev_stack_forward(c, params, X, X, workspace=ws, Y1=Yt1, Y2=Yt2), tsteps, 2)

    def adam_only():
        tstep[0] += 1
        B.rev_adamw_step(master, out["dparams"], mom1, mom2, tstep[0], lr=1e-5,
                         params_bf16=params if cfg["mode"] == "bf16" else None)
    _, ms_opt = timed(adam_only, tsteps, 2)
    nparam = int(params.numel())
    opt_bytes = nparam * (30 if cfg["mode"] == "bf16" else 28)
    line["training_step"] = {
        "what": "rev_stack_forward + reversible backward + rev_adamw_step, no head/loss, synthetic cotangents",
        "pareprop": {"samples_per_s": Bsz / (float(np.median(ms_tp)) * 1e-3), "ms_median": float(np.median(ms_tp))},
        "reprop": {"samples_per_s": Bsz / (float(np.median(ms_tr)) * 1e-3), "ms_median": float(np.median(ms_tr))},
        "pareprop_over_reprop": float(np.median(ms_tr)) / float(np.median(ms_tp)),
        "forward_ms": float(np.median(ms_fwd)),
        "adamw_ms": float(np.median(ms_opt)),
        "adamw_GBs": opt_bytes / (float(np.median(ms_opt)) * 1e-3) / 1e9,
        "adamw_hbm_fraction": opt_bytes / (float(np.median(ms_opt)) * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "parameters": nparam,
        "finite_after_steps": bool(torch.isfinite(master).all().item()),
    }

    # ---- padded text batches (text workloads only): the same backward pass with a key-padding mask,
    # lengths drawn once from a seeded uniform law on [T/8, T] as a stand-in for variable-length text
    if args.workload.startswith("roberta"):
        lens = synth.make_key_lengths(cfg, seed=0)
        klen = torch.from_numpy(lens).cuda()
        Ym1, Ym2 = B.rev_stack_forward_masked(c, params, X, X, klen, workspace=ws)
        B.rev_stack_backward_reprop_masked(c, params, Ym1, Ym2, klen, dY1, dY2, workspace=ws, out=out)
        torch.cuda.synchronize()
        few = max(5, args.steps // 2)
        _, ms_mp = timed(lambda: B.rev_stack_backward_pareprop_masked(c, params, Ym1, Ym2, klen, dY1, dY2, side,
                                                                      workspace=ws, out=out), few, 3)
        _, ms_mr = timed(lambda: B.rev_stack_backward_reprop_masked(c, params, Ym1, Ym2, klen, dY1, dY2,
                                                                    workspace=ws, out=out), few, 3)
        line["key_padding_mask"] = {
            "what": "same pass through the *_masked entry points, key lengths ~ U[T/8, T] (seed 0)",
            "mean_length": float(lens.mean()), "min_length": int(lens.min()),
            "pareprop": {"samples_per_s": Bsz / (float(np.median(ms_mp)) * 1e-3), "ms_median": float(np.median(ms_mp))},
            "reprop": {"samples_per_s": Bsz / (float(np.median(ms_mr)) * 1e-3), "ms_median": float(np.median(ms_mr))},
            "finite": bool(torch.isfinite(out["dparams"]).all().item()),
        }

    if not args.no_cpu_baseline:
        from oracle import rev_oracle as O
        blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
        y1 = Y1.cpu().numpy()
        y2 = Y2.cpu().numpy()
        H = cfg["n_heads"]
        nb = args.cpu_samples
        if nb <= 0:
            t0 = time.perf_counter()
            O.stack_backward_reversible(y1[:1].astype(np.float64), y2[:1].astype(np.float64), blocks, H,
                                        dy1[:1].astype(np.float64), dy2[:1].astype(np.float64))
            t1 = time.perf_counter() - t0
            nb = int(max(1, min(Bsz, 15.0 / max(t1, 1e-3))))
        t0 = time.perf_counter()
        O.stack_backward_reversible_chunked(y1[:nb], y2[:nb], blocks, H, dy1[:nb], dy2[:nb], chunk=8)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        line["cpu_baseline"] = {"value": nb / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
                                "sample": f"fp64 numpy oracle, reversible backward of the first {nb} of {Bsz} samples "
                                          f"(all {cfg['n_blocks']} blocks), {dt:.1f} s"}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
