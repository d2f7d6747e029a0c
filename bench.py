#!/usr/bin/env python3
"""Benchmark of the AR-Topk compressor step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c4|c2|c1|c3] [--rho R]

A "step" is one artopk_step() call: EF add + leader choice + exact Top-k on the
leader + gather + ordered sum + residual rewrite + dense update, for all W
simulated workers, with every input already resident in HBM.  Prints ONE JSON
line.  `value` is W*N / t_step in G elements/s.  `roofline` describes the
dominant kernel (the fused pass over all workers, 12*W*N algorithmic bytes per
launch; or, with a leader known up front, the fused pass over the other W-1
workers), timed with HIP events on the library's stream.  `cpu_baseline` is the
NumPy oracle timed on a bounded sample of the same workload on the host (single
thread).  With the default workload (c5, the 1e9 x 8 configuration) the line
also carries the three keep fractions of the 138 M x 4 configuration under
`other` (--no-c4 leaves them out).

Inputs: two gradient sets (steps 1 and 2 of the workload's seeded recipe) are
generated and uploaded before the timed region and alternate from step to step,
with the residual carried, so leader, threshold and guess outcome change between
steps as they do with a fresh gradient per step.
"""

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profile_traffic(tag, rho, kernel, suffix=""):
    """HBM bytes per launch of `kernel` as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, each
    scaled by what the counter reads for a plain copy): read from the committed summary of the same
    workload, profiles/artopk_step_<tag>_rho<rho><suffix>.md (suffix: _bf16 for gradients stored so).  (None, None) if there is no such summary or
    it does not list the kernel: the figure is never carried in this file."""
    rel = os.path.join("profiles", f"artopk_step_{tag}_rho{rho}{suffix}.md")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    in_table = False
    for line in open(path):
        if line.startswith("## HBM traffic per launch"):
            in_table = True
            continue
        if in_table and line.startswith("|"):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and re.match(rf"{re.escape(kernel)}(<|$)", cells[0]):
                try:
                    return float(cells[4]) * 1e6, rel
                except ValueError:
                    return None, None
    return None, None


def algorithmic_bytes(w, n, k, with_vals, g_bytes=4, reread=True, dense_update=True):
    """Bytes one step must move (fp32, 4-byte granularity for the k-sized terms).  reread: the
    selection reads the leader's vector once more after the fused pass (it does not when the
    survivor list is written from the fused pass' bit mask).  dense_update False: the model update
    in its sparse form (idx and sum read, k weights read and written) instead of N floats written."""
    pass_a = (8 + g_bytes) * w * n      # read g, read residual, write acc
    select = 4 * n if reread else 0
    update = 4 * n if dense_update else 16 * k
    ksized = k * (8 * w + (4 * w if with_vals else 0) + 20)
    return pass_a, pass_a + select + update + ksized


class Inputs:
    """Two gradient sets of one workload resident on the GPU (generated once, shared by all its keep
    fractions) and the residuals."""

    def __init__(self, args, cfg, torch, inp):
        import numpy as np

        self.wl = wl = inp.workload(cfg)
        dev = torch.device("cuda:0")
        t0 = time.perf_counter()
        host = np.empty(wl.n, dtype=np.float32)
        self.g_sets = []
        for step in (1, 2):
            g = []
            for r in range(wl.w):
                wl.gen_into(host, step, r, threads=args.gen_threads)
                t = torch.from_numpy(host).to(dev)
                if args.g16:  # 16-bit gradient storage: rounded once here, outside the timed region
                    t = t.to(torch.bfloat16 if args.g16 == "bf16" else torch.float16)
                g.append(t)
            self.g_sets.append(g)
            log(f"[bench]   {wl.name}: gradient set {step} generated and uploaded ({time.perf_counter() - t0:.1f} s)")
        self.res = [torch.zeros(wl.n, dtype=torch.float32, device=dev) for _ in range(wl.w)]

    def reset(self):
        for r in self.res:
            r.zero_()


def run_workload(args, data, rho, steps, warmup, torch, pkg, inp):
    wl = data.wl
    k = wl.k(rho)
    seg_off = None if wl.seg_off is None else [int(v) for v in wl.seg_off]
    seg_k = None if wl.seg_off is None else [int(v) for v in wl.seg_k(rho)]
    if args.bucket_elems:   # the flat vector cut into buckets, every bucket its own Top-k of the same keep fraction
        seg_off = list(range(0, wl.n, args.bucket_elems)) + [wl.n]
        seg_k = [max(1, math.ceil(rho * (seg_off[i + 1] - seg_off[i]))) for i in range(len(seg_off) - 1)]
        k = sum(seg_k)
    dev = torch.device("cuda:0")
    mode = pkg.ARTOPK_STAR if wl.mode == inp.MODE_STAR else pkg.ARTOPK_VAR
    log(f"[bench] workload {wl.name}: N={wl.n} W={wl.w} rho={rho} k={k} mode={'STAR' if mode == 0 else 'VAR'}")
    data.reset()
    res = data.res
    ctx = pkg.Context(wl.w, wl.n, k, 1 if seg_k is None else len(seg_k))
    for name, value in args.options.items():   # route switches (results are the same on every route)
        ctx.set_option(getattr(pkg, "ARTOPK_OPT_" + name.upper()), value)
    update = None if args.sparse_update else torch.empty(wl.n, dtype=torch.float32, device=dev)
    weights = torch.zeros(wl.n, dtype=torch.float32, device=dev) if args.sparse_update else None
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    summed = torch.empty(k, dtype=torch.float32, device=dev)
    leader = torch.zeros(1, dtype=torch.int32, device=dev)
    var = torch.zeros(wl.w, dtype=torch.float64, device=dev)

    g_bytes = 2 if args.g16 else 4
    g_type = {None: pkg.ARTOPK_G_F32, "bf16": pkg.ARTOPK_G_BF16, "f16": pkg.ARTOPK_G_F16}[args.g16]

    def one(step_no):
        g = data.g_sets[(step_no - 1) % 2]
        if args.g16:
            ctx.artopk_step_g16(g, g_type, res, k, mode, step_no, idx, summed, update, leader_out=leader,
                                var_out=var, seg_off=seg_off, seg_k=seg_k)
        else:
            ctx.artopk_step(g, res, k, mode, step_no, idx, summed, update, leader_out=leader, var_out=var,
                            seg_off=seg_off, seg_k=seg_k)
        if args.sparse_update:   # `update` is the model here: w[idx] -= eta * sum instead of N floats written
            ctx.artopk_apply_update(weights, idx, summed, k, 1e-3)

    step_no = 1
    for _ in range(warmup):
        one(step_no)
        step_no += 1
    torch.cuda.synchronize()
    ctx.status()

    # timed region: K steps, the dominant kernel bracketed by HIP events on the library's stream
    ctx.set_profile(1)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(steps):
        one(step_no)
        step_no += 1
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start
    # level-1 events bracket the dominant kernel: the fused pass over all workers (VAR) or,
    # when the leader is known up front, the fused pass over the W-1 other workers
    # (the library says which of the two it ran: an option can turn the second off)
    info = ctx.select_info()
    star = info["dominant_workers"] == wl.w - 1 and wl.w > 1
    # the fused pass of the guess route (also, without a bound, of a long segmented step) / of the histogram route
    striding = info["guessed"] or (seg_off is not None and wl.n >= ctx.get_option(pkg.ARTOPK_OPT_GUESS_MIN_N))
    fused = "k_pass_mark" if striding else "k_pass_a"
    dom_name, dom_stage, dom_workers = ("k_pass_rest", "gather", wl.w - 1) if star else (fused, "pass_a", wl.w)
    dom_ms = ctx.get_profile()[dom_stage]  # averaged over the timed steps
    # stage breakdown from a few extra, untimed steps (an event at every stage boundary)
    ctx.set_profile(2)
    for _ in range(min(4, steps)):
        one(step_no)
        step_no += 1
    stage_ms = ctx.get_profile()
    ctx.set_profile(0)
    ctx.status()
    ms_per_step = 1e3 * t_total / steps
    _, b_step = algorithmic_bytes(wl.w, wl.n, k, False, g_bytes, reread=not info["from_mask"],
                                  dense_update=not args.sparse_update)
    _, b_scope = algorithmic_bytes(wl.w, wl.n, k, False, g_bytes, reread=True, dense_update=not args.sparse_update)
    b_dom = (8 + g_bytes) * dom_workers * wl.n
    out = {
        "wl": wl, "k": k, "rho": rho, "ms_per_step": ms_per_step,
        "gelem_per_s": wl.w * wl.n / (ms_per_step * 1e-3) / 1e9,
        "dom_ms": dom_ms, "dom_gbps": b_dom / (dom_ms * 1e-3) / 1e9,
        "step_alg_gbps": b_step / (ms_per_step * 1e-3) / 1e9,
        "stages": stage_ms, "b_dom": b_dom, "b_step": b_step, "leader": int(leader.item()), "dom_name": dom_name,
        "from_mask": bool(info["from_mask"]), "b_scope": b_scope,
    }
    log(f"[bench]   {ms_per_step:.3f} ms/step, {out['gelem_per_s']:.1f} G elem/s, {dom_name} {dom_ms:.3f} ms = "
        f"{out['dom_gbps']:.0f} GB/s, whole step {out['step_alg_gbps']:.0f} GB/s algorithmic; stages {out['stages']}")
    del ctx
    return out


def run_entry_points(args, data, rho, reps, torch, pkg):
    """Times the stand-alone calls of the boundary on one workload: every call `reps` times back to
    back on vectors resident in HBM (gradient set 1 stands for the error-fed vectors, worker 0 is
    the selected one).  ms per call and the algorithmic bytes it moves."""
    wl = data.wl
    n, w = wl.n, wl.w
    k = wl.k(rho)
    dev = torch.device("cuda:0")
    acc = data.g_sets[0]
    ctx = pkg.Context(w, n, k, 1)
    for name, value in args.options.items():
        ctx.set_option(getattr(pkg, "ARTOPK_OPT_" + name.upper()), value)
    var = torch.zeros(w, dtype=torch.float64, device=dev)
    arg = torch.zeros(1, dtype=torch.int32, device=dev)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    idx_rows = torch.empty(w * k, dtype=torch.int32, device=dev)
    vals = torch.empty(w * k, dtype=torch.float32, device=dev)
    summed = torch.empty(k, dtype=torch.float32, device=dev)
    sq = torch.zeros(w, dtype=torch.float64, device=dev)
    gain = torch.zeros(w, dtype=torch.float64, device=dev)
    update = torch.empty(n, dtype=torch.float32, device=dev)
    calls = [
        ("artopk_variance", lambda: ctx.artopk_variance(acc, var, arg), 4 * w * n),
        ("artopk_select_topk", lambda: ctx.artopk_select_topk(acc[0], k, idx), 8 * n + 4 * k),
        ("artopk_gather_sum", lambda: ctx.artopk_gather_sum(acc, idx, k, vals, summed), k * (4 + 8 * w + 4)),
        ("artopk_scatter_residual", lambda: ctx.artopk_scatter_residual(data.res, idx, k, summed, update),
         4 * n + k * (8 + 4 * w)),
        ("artopk_topk_workers", lambda: ctx.artopk_topk_workers(acc, k, idx_rows, vals, sq, arg), w * (8 * n + 8 * k)),
        ("artopk_compression_gain", lambda: ctx.artopk_compression_gain(data.res, vals, k, gain), 4 * w * n + 4 * w * k),
        ("artopk_apply_update", lambda: ctx.artopk_apply_update(update, idx, summed, k, 1e-3), 16 * k),
    ]
    out = {}
    for name, call, nbytes in calls:
        call()
        torch.cuda.synchronize()
        ctx.status()
        t0 = time.perf_counter()
        for _ in range(reps):
            call()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / reps
        out[name] = {"ms": round(ms, 4), "algorithmic_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
        log(f"[bench]   {name}: {ms:.3f} ms, {out[name]['GBps']:.0f} GB/s algorithmic")
    ctx.status()
    del ctx
    return {"workload": wl.name, "N": n, "W": w, "rho": rho, "k": k, "calls": out}


def roofline_of(r, tag, g16):
    traffic, source = profile_traffic(tag, r["rho"], r["dom_name"], f"_{g16}" if g16 else "")
    return {"bound": "hbm", "kernel": r["dom_name"], "achieved": round(r["dom_gbps"], 1),
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(r["dom_gbps"] / HBM_PEAK_GBPS, 4),
            "traffic": traffic, "traffic_source": source, "algorithmic_bytes_per_launch": r["b_dom"],
            "avg_launch_ms": round(r["dom_ms"], 4)}


def step_of(r):
    return {"bytes": r["b_step"], "GBps": round(r["step_alg_gbps"], 1),
            "frac_of_hbm_peak": round(r["step_alg_gbps"] / HBM_PEAK_GBPS, 4),
            "leader_reread_counted": not r["from_mask"],
            # the scope table's formula always counts one re-read of the leader (4 N): for comparison
            "bytes_with_leader_reread": r["b_scope"],
            "frac_of_hbm_peak_with_leader_reread": round(r["b_scope"] / (r["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "stage_ms": {k_: round(v, 4) for k_, v in r["stages"].items()}}


def cpu_baseline(cfg, rho, inp, n_cap=1 << 24, budget_s=15.0, max_steps=12):
    """The oracle, as it stands, on a bounded sample of the workload (one thread)."""
    import numpy as np
    from oracle import artopk_oracle as orc

    full = inp.workload(cfg)
    n = min(full.n, n_cap)
    wl = inp.workload(cfg, n=n)
    k = wl.k(rho)
    seg_off = None if wl.seg_off is None else [int(v) for v in wl.seg_off]
    seg_k = None if wl.seg_off is None else [int(v) for v in wl.seg_k(rho)]
    mode = orc.MODE_STAR if wl.mode == inp.MODE_STAR else orc.MODE_VAR
    res = [np.zeros(n, np.float32) for _ in range(wl.w)]
    steps, spent = 0, 0.0
    while spent < budget_s and steps < max_steps:
        g = [wl.gen(steps + 1, r, threads=8) for r in range(wl.w)]
        t0 = time.perf_counter()
        out = orc.step(g, res, k, mode, step_no=steps + 1, seg_off=seg_off, seg_k=seg_k)
        spent += time.perf_counter() - t0
        res = out.residual
        steps += 1
    size = "at its full size" if n == full.n else f"shrunk to N={n}"
    return {
        "value": wl.w * n * steps / spent / 1e9, "unit": "G elements/s", "cores": 1, "kind": "oracle",
        "sample": f"{steps} step(s) of workload {wl.name} {size} (W={wl.w}, rho={rho}), "
                  f"{spent:.1f} s of single-thread NumPy",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--rho", type=float, default=None)
    ap.add_argument("--gen-threads", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--g16", choices=["bf16", "f16"], default=None,
                    help="store the gradients in 16 bits (artopk_step_g16); not the headline configuration")
    ap.add_argument("--no-c4", action="store_true",
                    help="with the default workload: leave out the 138 M x 4 configuration's rows under 'other'")
    ap.add_argument("--sparse-update", action="store_true",
                    help="leave out the dense update (update_out = NULL) and apply w[idx] -= eta * sum instead "
                         "(artopk_apply_update); not the headline configuration")
    ap.add_argument("--bucket-elems", type=int, default=0, metavar="E",
                    help="run the step bucketed: segments of E elements (16777216 = 64 MB of float32), each with "
                         "its own Top-k; not the headline configuration")
    ap.add_argument("--entry-points", action="store_true",
                    help="instead of the step, time the stand-alone calls of the boundary (variance, selection, "
                         "gather + sum, scatter + residual, and the neighbours of the step) on the workload")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="set a library route switch before measuring, e.g. guess_min_n=4096 or stage_tiles=2 "
                         "(artopk_set_option; recorded under config.options)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy five times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    args.options = {o.split("=", 1)[0]: int(o.split("=", 1)[1]) for o in args.option}
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import artopk_inputs as inp
    import paper_2312_02493_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        sys.exit(2)
    pkg.load_library()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4}))
        return

    cfg = int(args.workload[1])
    wl0 = inp.workload(cfg)
    rho = args.rho if args.rho is not None else {1: 0.01, 2: 0.01, 3: 0.01, 4: 0.01, 5: 0.001}[cfg]
    data = Inputs(args, cfg, torch, inp)
    if args.entry_points:
        if args.g16:
            print("--entry-points takes float32 vectors", file=sys.stderr)
            sys.exit(2)
        print(json.dumps({"entry_points": run_entry_points(args, data, rho, args.steps, torch, pkg)}), flush=True)
        return
    r = run_workload(args, data, rho, args.steps, args.warmup, torch, pkg, inp)
    del data
    torch.cuda.empty_cache()

    # the second target configuration (138 M x 4, round-robin leader) at its three keep fractions
    other = {}
    if cfg == 5 and args.rho is None and not args.no_c4:
        data4 = Inputs(args, 4, torch, inp)
        for rh in (0.1, 0.01, 0.001):
            o = run_workload(args, data4, rh, max(args.steps, 20), max(args.warmup, 3), torch, pkg, inp)
            other[f"c4_rho{rh}"] = {
                "config": {"workload": data4.wl.name, "N": data4.wl.n, "W": data4.wl.w, "rho": rh, "k": o["k"],
                           "leader_rule": "STAR"},
                "ms_per_step": round(o["ms_per_step"], 4), "value": round(o["gelem_per_s"], 2),
                "unit": "G elements/s", "roofline": roofline_of(o, "c4", args.g16), "step_algorithmic": step_of(o)}
        del data4
        torch.cuda.empty_cache()
        if not args.no_cpu_baseline:   # the oracle at this configuration's own size: one step, a full sort of 138 M keys
            other["c4_rho0.01"]["cpu_baseline"] = cpu_baseline(4, 0.01, inp, n_cap=1 << 31, budget_s=1.0, max_steps=1)

    base = None if args.no_cpu_baseline else cpu_baseline(cfg, rho, inp)

    line = {
        "metric": "compressed gradient elements/s per AR-Topk step (1 GPU)",
        "value": round(r["gelem_per_s"], 3),
        "unit": "G elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if not args.g16 else f"f32 (gradients stored as {args.g16})",
        "data": "synthetic (seeded recipe of the workload; two pre-generated gradient sets, steps 1 and 2 of "
                "the recipe, alternate from step to step; residual carried)",
        "config": {"workload": wl0.name, "N": wl0.n, "W": wl0.w, "rho": rho, "k": r["k"],
                   "leader_rule": "STAR" if wl0.mode == inp.MODE_STAR else "VAR",
                   **({"gradient_storage": args.g16} if args.g16 else {}),
                   **({"update": "sparse (artopk_apply_update)"} if args.sparse_update else {}),
                   **({"bucket_elems": args.bucket_elems} if args.bucket_elems else {}),
                   **({"options": args.options} if args.options else {})},
        "roofline": roofline_of(r, args.workload, args.g16),
        "step_algorithmic": step_of(r),
        "cpu_baseline": base,
    }
    if other:
        line["other"] = other
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
