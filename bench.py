#!/usr/bin/env python3
"""Benchmark of the AR-Topk compressor step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c4|c2|c1|c3] [--rho R]

A "step" is one artopk_step() call: EF add + leader choice + exact Top-k on the
leader + gather + ordered sum + residual rewrite + dense update, for all W
simulated workers, with every input already resident in HBM.  Prints ONE JSON
line.  `value` is W*N / t_step in G elements/s.  `roofline` describes the
dominant kernel (the fused EF-add / variance / histogram pass, 12*W*N
algorithmic bytes per launch), timed with HIP events on the library's stream.
`cpu_baseline` is the NumPy oracle timed on a bounded sample of the same
workload on the host (single thread).
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of the dominant kernel, measured with two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for a plain 1 GiB
# device copy (profiles/artopk_step_<workload>_rho<rho>.md); None where it was not measured.
MEASURED_TRAFFIC_BYTES = {
    ("c5", 0.001): 97127.0e6,   # k_pass_mark, all 8 workers: 64.0 GB fetched + 33.1 GB written (1 GB of it bit masks)
    ("c4", 0.01): 5006.4e6,     # k_pass_rest, 3 workers: 3.33 GB fetched + 1.68 GB written
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(w, n, k, with_vals, g_bytes=4):
    """Bytes one step must move (fp32, 4-byte granularity for the k-sized terms)."""
    pass_a = (8 + g_bytes) * w * n      # read g, read residual, write acc
    select = 4 * n                      # one re-read of the leader after the threshold digit is known
    update = 4 * n                      # dense update written once
    ksized = k * (8 * w + (4 * w if with_vals else 0) + 20)
    return pass_a, pass_a + select + update + ksized


def run_workload(args, cfg, rho, steps, warmup, torch, pkg, inp):
    wl = inp.workload(cfg)
    k = wl.k(rho)
    seg_off = None if wl.seg_off is None else [int(v) for v in wl.seg_off]
    seg_k = None if wl.seg_off is None else [int(v) for v in wl.seg_k(rho)]
    dev = torch.device("cuda:0")
    mode = pkg.ARTOPK_STAR if wl.mode == inp.MODE_STAR else pkg.ARTOPK_VAR
    log(f"[bench] workload {wl.name}: N={wl.n} W={wl.w} rho={rho} k={k} mode={'STAR' if mode == 0 else 'VAR'}")

    t0 = time.perf_counter()
    g, res = [], []
    import numpy as np
    host = np.empty(wl.n, dtype=np.float32)
    for r in range(wl.w):
        wl.gen_into(host, 1, r, threads=args.gen_threads)
        t = torch.from_numpy(host).to(dev)
        if args.g16:  # 16-bit gradient storage: rounded once here, outside the timed region
            t = t.to(torch.bfloat16 if args.g16 == "bf16" else torch.float16)
        g.append(t)
        res.append(torch.zeros(wl.n, dtype=torch.float32, device=dev))
        log(f"[bench]   worker {r} generated and uploaded ({time.perf_counter() - t0:.1f} s)")
    del host
    ctx = pkg.Context(wl.w, wl.n, k, 1 if seg_k is None else len(seg_k))
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    summed = torch.empty(k, dtype=torch.float32, device=dev)
    update = torch.empty(wl.n, dtype=torch.float32, device=dev)
    leader = torch.zeros(1, dtype=torch.int32, device=dev)
    var = torch.zeros(wl.w, dtype=torch.float64, device=dev)

    g_bytes = 2 if args.g16 else 4
    g_type = {None: pkg.ARTOPK_G_F32, "bf16": pkg.ARTOPK_G_BF16, "f16": pkg.ARTOPK_G_F16}[args.g16]

    def one(step_no):
        if args.g16:
            ctx.artopk_step_g16(g, g_type, res, k, mode, step_no, idx, summed, update, leader_out=leader,
                                var_out=var, seg_off=seg_off, seg_k=seg_k)
        else:
            ctx.artopk_step(g, res, k, mode, step_no, idx, summed, update, leader_out=leader, var_out=var,
                            seg_off=seg_off, seg_k=seg_k)

    step_no = 1
    for _ in range(warmup):
        one(step_no)
        step_no += 1
    torch.cuda.synchronize()
    ctx.status()

    # timed region: K steps, pass A bracketed by HIP events on the library's stream
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
    # (the library says which of the two it ran: an environment switch can turn the second off)
    info = ctx.select_info()
    star = info["dominant_workers"] == wl.w - 1 and wl.w > 1
    fused = "k_pass_mark" if info["guessed"] else "k_pass_a"   # the fused pass of the guess / histogram route
    dom_name, dom_stage, dom_workers = ("k_pass_rest", "gather", wl.w - 1) if star else (fused, "pass_a", wl.w)
    pass_a_ms = [ctx.get_profile()[dom_stage]]  # averaged over the timed steps
    # stage breakdown from a few extra, untimed steps (an event at every stage boundary)
    ctx.set_profile(2)
    for _ in range(min(3, steps)):
        one(step_no)
        step_no += 1
    stage_ms = [ctx.get_profile()]
    ctx.set_profile(0)
    ctx.status()
    ms_per_step = 1e3 * t_total / steps
    pa = sum(pass_a_ms) / len(pass_a_ms)
    _, b_step = algorithmic_bytes(wl.w, wl.n, k, False, g_bytes)
    b_pass_a = (8 + g_bytes) * dom_workers * wl.n
    out = {
        "wl": wl, "k": k, "rho": rho, "ms_per_step": ms_per_step,
        "gelem_per_s": wl.w * wl.n / (ms_per_step * 1e-3) / 1e9,
        "pass_a_ms": pa, "pass_a_gbps": b_pass_a / (pa * 1e-3) / 1e9,
        "step_alg_gbps": b_step / (ms_per_step * 1e-3) / 1e9,
        "stages": {name: sum(s[name] for s in stage_ms) / len(stage_ms) for name in stage_ms[0]},
        "b_pass_a": b_pass_a, "b_step": b_step, "leader": int(leader.item()), "dom_name": dom_name,
    }
    log(f"[bench]   {ms_per_step:.3f} ms/step, {out['gelem_per_s']:.1f} G elem/s, {dom_name} {pa:.3f} ms = "
        f"{out['pass_a_gbps']:.0f} GB/s, whole step {out['step_alg_gbps']:.0f} GB/s algorithmic; stages {out['stages']}")
    del g, res, update, ctx
    torch.cuda.empty_cache()
    return out


def cpu_baseline(cfg, rho, inp, budget_s=15.0):
    """The oracle, as it stands, on a bounded sample of the workload (one thread)."""
    import numpy as np
    from oracle import artopk_oracle as orc

    full = inp.workload(cfg)
    n = min(full.n, 1 << 24)
    wl = inp.workload(cfg, n=n)
    k = wl.k(rho)
    seg_off = None if wl.seg_off is None else [int(v) for v in wl.seg_off]
    seg_k = None if wl.seg_off is None else [int(v) for v in wl.seg_k(rho)]
    mode = orc.MODE_STAR if wl.mode == inp.MODE_STAR else orc.MODE_VAR
    res = [np.zeros(n, np.float32) for _ in range(wl.w)]
    steps, spent = 0, 0.0
    while spent < budget_s and steps < 12:
        g = [wl.gen(steps + 1, r) for r in range(wl.w)]
        t0 = time.perf_counter()
        out = orc.step(g, res, k, mode, step_no=steps + 1, seg_off=seg_off, seg_k=seg_k)
        spent += time.perf_counter() - t0
        res = out.residual
        steps += 1
    return {
        "value": wl.w * n * steps / spent / 1e9, "unit": "G elements/s", "cores": 1, "kind": "oracle",
        "sample": f"{steps} steps of workload {wl.name} shrunk to N={n} (W={wl.w}, rho={rho}), "
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
    ap.add_argument("--also-c4", action="store_true", help="append the 138M workload's numbers under 'other'")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy five times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
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
    r = run_workload(args, cfg, rho, args.steps, args.warmup, torch, pkg, inp)

    other = {}
    if args.also_c4 and cfg != 4:
        for rh in (0.1, 0.01, 0.001):
            o = run_workload(args, 4, rh, args.steps, args.warmup, torch, pkg, inp)
            other[f"c4_rho{rh}"] = {"ms_per_step": round(o["ms_per_step"], 4),
                                    "G_elements_per_s": round(o["gelem_per_s"], 2),
                                    "step_alg_GBps": round(o["step_alg_gbps"], 1),
                                    "pass_a_GBps": round(o["pass_a_gbps"], 1)}

    base = None if args.no_cpu_baseline else cpu_baseline(cfg, rho, inp)

    traffic = None if args.g16 else MEASURED_TRAFFIC_BYTES.get((args.workload, rho))
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
        "data": "synthetic (seeded recipe of the workload; step-1 gradients reused every step, residual carried)",
        "config": {"workload": wl0.name, "N": wl0.n, "W": wl0.w, "rho": rho, "k": r["k"],
                   "leader_rule": "STAR" if wl0.mode == inp.MODE_STAR else "VAR",
                   **({"gradient_storage": args.g16} if args.g16 else {})},
        "roofline": {"bound": "hbm", "kernel": r["dom_name"], "achieved": round(r["pass_a_gbps"], 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(r["pass_a_gbps"] / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "algorithmic_bytes_per_launch": r["b_pass_a"],
                     "avg_launch_ms": round(r["pass_a_ms"], 4)},
        "step_algorithmic": {"bytes": r["b_step"], "GBps": round(r["step_alg_gbps"], 1),
                             "frac_of_hbm_peak": round(r["step_alg_gbps"] / HBM_PEAK_GBPS, 4),
                             "stage_ms": {k_: round(v, 4) for k_, v in r["stages"].items()}},
        "cpu_baseline": base,
    }
    if other:
        line["other"] = other
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
