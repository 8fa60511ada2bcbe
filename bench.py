#!/usr/bin/env python3
"""Benchmark of the FSD candidate-verification step on one MI355X.

A step is one complete fsd_verify_chain call (counter reset, vocabulary reduction, acceptance
scan and Gumbel-max token) on one batch of synthetic logits already resident in HBM.  The
workload is configuration C2 (B=64 sequences, K=8 candidates, V=128256, bfloat16, JS divergence,
T=0.1); several distinct input sets are rotated so that the working set exceeds the on-die caches.

Order of a run: an untimed settle phase (calls until the device has been busy for --settle-ms, so
that the timed steps do not fall into the clock ramp of an idle GPU; its length is reported in
`config`), the W warm-up steps, the K timed steps between two synchronisations, and then a
separate pass of the same K steps with a start and a stop event on the vocabulary-reduction kernel's launch (the
events stay out of the timed region).

Prints one JSON line: verified candidate positions per second, plus the roofline of the
vocabulary-reduction kernel (algorithmic bytes / its event-timed duration against the 8 TB/s HBM
peak) and the CPU oracle's rate on the host cores as a reported baseline.
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

HBM_PEAK_GBS = 8000.0          # MI355X published peak


def traffic_from_profile(workload: str):
    """HBM bytes per launch of the reduction kernel, from the committed counter summary (or None).
    A cross-check measured in its own rocprofv3 run (counters cannot be read inside this process); the
    summary names the kernel and workload it was taken on."""
    path = os.path.join(ROOT, "profiles", f"pair_kernel_{workload}_pmc.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C2", choices=["C2", "C3", "C4", "C5"])
    ap.add_argument("--div", default="js", choices=["kl", "js", "tv"])
    ap.add_argument("--method", default="fsd", choices=["fsd", "sd", "rfsd"],
                    help="fsd: the paper's rule (default); sd: the strict baseline (chain or tree); rfsd: reducible FSD (chain)")
    ap.add_argument("--sets", type=int, default=0, help="distinct input sets to rotate (0 = enough for > 1 GB)")
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="untimed calls before the warm-up until the device has been busy this long (0 = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--phase-split", action="store_true",
                    help="load the development library built with `python -m paper_2502_20704_amd.build "
                         "--phase-timing` and also print the reduction kernel's cycles per phase (its counters "
                         "cost time: the rates of such a run are not the headline)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference kernel for scaling rocprofv3's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2502_20704_amd as fsd
    from paper_2502_20704_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if args.phase_split:
        from paper_2502_20704_amd import binding, build as fsd_build

        if not os.path.exists(fsd_build.LIB_PHASE_TIMING):
            print(f"{fsd_build.LIB_PHASE_TIMING} is missing: python -m paper_2502_20704_amd.build --phase-timing",
                  file=sys.stderr)
            return 2
        binding.LIB_PATH = fsd_build.LIB_PHASE_TIMING
    fsd.library()
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    div = {"kl": fsd.DIV_KL, "js": fsd.DIV_JS, "tv": fsd.DIV_TV}[args.div]
    T = cfg["T"][0]
    tree = cfg["shape"] == "tree"
    rows = cfg["N"] if tree else cfg["K"]
    B, V = cfg["B"], cfg["V"]
    es = 2 if cfg["dtype"] == "bf16" else 4
    set_bytes = B * (2 * rows + 1) * V * es
    nsets = args.sets or max(2, -(-(1200 << 20) // set_bytes))
    if set_bytes * nsets > (24 << 30):
        nsets = max(1, (24 << 30) // set_bytes)

    sets, host_sets = [], []
    target_rows_read = []   # per input set: distinct target rows the pairs refer to
    for s in range(nsets):
        inp = synth.config_inputs(args.config, seed=100 + s)
        if tree:   # the children of a node share its target row: it counts once
            par = inp["parent"].reshape(B, rows)
            target_rows_read.append(sum(len(set(par[b].tolist())) for b in range(B)))
        else:
            target_rows_read.append(B * rows)
        if s < 4:
            host_sets.append(inp)
        if tree:
            dev = {k: synth.as_torch(inp[k]) for k in ("target", "draft", "node_tokens", "parent")}
            dev["max_depth"] = int(inp["max_depth"])
        else:
            dev = {k: synth.as_torch(inp[k]) for k in ("target", "draft", "cand")}
        sets.append(dev)
    dt_code = fsd.BF16 if cfg["dtype"] == "bf16" else fsd.F32
    ws = torch.empty(fsd.fsd_workspace_bytes(B, rows, V, dt_code) + 256, dtype=torch.uint8, device="cuda")
    outs = [None] * nsets

    if args.method == "rfsd" and tree:
        print("reducible FSD is built for chains only", file=sys.stderr)
        return 2

    def step(i):
        d = sets[i % nsets]
        if args.method == "sd" and tree:
            outs[i % nsets] = fsd.sd_verify_tree(d["target"], d["draft"], d["node_tokens"], d["parent"],
                                                 d["max_depth"], fsd.SAMPLE, seed=1, offset=i,
                                                 out=outs[i % nsets], workspace=ws)
        elif args.method == "sd":
            outs[i % nsets] = fsd.sd_verify_chain(d["target"], d["draft"], d["cand"], fsd.SAMPLE, seed=1, offset=i,
                                                  out=outs[i % nsets], workspace=ws)
        elif args.method == "rfsd":
            outs[i % nsets] = fsd.rfsd_verify_chain(d["target"], d["draft"], d["cand"], T, div, fsd.SAMPLE, seed=1,
                                                    offset=i, out=outs[i % nsets], workspace=ws)
        elif tree:
            outs[i % nsets] = fsd.fsd_verify_tree(d["target"], d["draft"], d["node_tokens"], d["parent"],
                                                  d["max_depth"], T, div, fsd.SAMPLE, seed=1, offset=i,
                                                  out=outs[i % nsets], workspace=ws)
        else:
            outs[i % nsets] = fsd.fsd_verify_chain(d["target"], d["draft"], d["cand"], T, div, fsd.SAMPLE, seed=1,
                                                   offset=i, out=outs[i % nsets], workspace=ws)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- settle: the same calls, untimed, until the device has been busy for a while
    settle_calls = 0
    t_s = time.perf_counter()
    while (time.perf_counter() - t_s) * 1e3 < args.settle_ms:
        for _ in range(16):
            step(settle_calls)
            settle_calls += 1
        torch.cuda.synchronize()
    settle_ms = (time.perf_counter() - t_s) * 1e3

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # ---- the same steps once more with events around the reduction kernel (outside the timed region)
    fsd.profile_enable(True)
    fsd.profile_collect()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    n_ev, k1_mean_ms, k1_min_ms = fsd.profile_collect()
    fsd.profile_enable(False)

    phase_split = None
    if args.phase_split:
        # one more call with a buffer the kernel's wavefronts write their cycle counts to: per wavefront,
        # cycles between the marks in the step (summed over its steps), its start time and its lifetime
        import ctypes

        lib = fsd.library()
        lib.fsd_debug_set_dbg.argtypes = [ctypes.c_void_p]
        lib.fsd_debug_set_dbg.restype = None
        dbg = torch.zeros(16384 * 10, dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        lib.fsd_debug_set_dbg(ctypes.c_void_p(dbg.data_ptr()))
        step(0)
        torch.cuda.synchronize()
        lib.fsd_debug_set_dbg(None)
        a = dbg.cpu().numpy().reshape(-1, 10)
        a = a[a[:, 9] > 0]
        names = ["wait for the logits + maximum pass", "exponential pass", "team merge (waiting for the team's words included)",
                 "wave sums, request of the next pair, post", "phase 2", "finishing duty", "drain", "second evaluations"]
        phase_split = {"wavefronts": int(len(a)), "lifetime_cycles_median": float(np.median(a[:, 9])),
                       "mean_cycles_per_wavefront": {n: float(v) for n, v in zip(names, a[:, :8].mean(0))}}
        print(f"reduction kernel, {len(a)} wavefronts, median lifetime {np.median(a[:, 9]):.0f} cycles "
              f"(p10 {np.percentile(a[:, 9], 10):.0f}, p90 {np.percentile(a[:, 9], 90):.0f}); mean cycles per "
              "wavefront between the marks of a step, summed over its steps (the compiler moves arithmetic "
              "across the marks: neighbouring phases are only roughly apart):", file=sys.stderr)
        for n, v in zip(names, a[:, :8].mean(0)):
            print(f"  {n:<55} {v:>10.0f}", file=sys.stderr)

    positions = B * rows
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = positions * args.steps / (t1 - t0)
    # one draft row per position and every distinct target row, each read once (mean over the sets)
    alg_bytes = int(V * es * (positions + sum(target_rows_read) / len(target_rows_read)))
    achieved = alg_bytes / (k1_mean_ms * 1e-3) / 1e9 if n_ev else None
    rule = {"fsd": f"{args.div.upper()} T={T}", "sd": "strict SD", "rfsd": f"reducible {args.div.upper()} T={T}"}[args.method]
    workload = (f"{args.config}: {'tree' if tree else 'chain'} verify B={B} {'N' if tree else 'K'}={rows} V={V} "
                f"{cfg['dtype']} {rule}")
    whole_call = (alg_bytes + B * V * es) / (ms_per_step * 1e-3) / 1e9

    result = {
        "metric": "verified candidate positions/sec and achieved HBM GB/s (% peak) at V=128256",
        "value": value,
        "unit": "positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload, "input_sets_rotated": nsets, "input_bytes_per_set": set_bytes,
                   "logits_dtype": cfg["dtype"], "settle_calls_untimed": settle_calls, "settle_ms": settle_ms,
                   "whole_call_GBps": whole_call, "whole_call_frac_of_peak": whole_call / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                     "traffic": traffic_from_profile(args.config), "kernel": "pair_kernel",
                     "kernel_ms_mean": k1_mean_ms, "kernel_ms_min": k1_min_ms, "launches_timed": n_ev,
                     "algorithmic_bytes_per_launch": alg_bytes},
    }
    if phase_split:
        result["phase_split"] = phase_split

    if not args.no_cpu_baseline:
        import oracle

        def oracle_pass(inp, nb):
            if args.method == "sd" and tree:
                oracle.sd_verify_tree(inp["target"][:nb], inp["draft"][:nb], inp["node_tokens"][:nb],
                                      inp["parent"][:nb], int(inp["max_depth"]), seed=1)
            elif args.method == "sd":
                oracle.sd_verify_chain(inp["target"][:nb], inp["draft"][:nb], inp["cand"][:nb], seed=1)
            elif args.method == "rfsd":
                oracle.rfsd_verify_chain(inp["target"][:nb], inp["draft"][:nb], inp["cand"][:nb], T, div, seed=1)
            elif tree:
                oracle.verify_tree(inp["target"][:nb], inp["draft"][:nb], inp["node_tokens"][:nb], inp["parent"][:nb],
                                   int(inp["max_depth"]), T, div, seed=1)
            else:
                oracle.verify_chain(inp["target"][:nb], inp["draft"][:nb], inp["cand"][:nb], T, div, seed=1)

        all_threads = oracle.num_threads()
        nb_all = min(B, 8 if tree else 64)
        t0 = time.perf_counter()
        npos = 0
        for inp in host_sets * 3:
            oracle_pass(inp, nb_all)
            npos += nb_all * rows
        dt = time.perf_counter() - t0
        # the same oracle on one core, on a smaller sample of the same workload
        oracle.set_num_threads(1)
        nb_one = min(B, 1 if tree else 8)
        t0 = time.perf_counter()
        npos1 = 0
        for inp in host_sets[:2]:
            oracle_pass(inp, nb_one)
            npos1 += nb_one * rows
        dt1 = time.perf_counter() - t0
        oracle.set_num_threads(all_threads)
        result["cpu_baseline"] = {"value": npos / dt, "unit": "positions/s", "cores": all_threads,
                                  "kind": "oracle",
                                  "sample": f"{npos} positions of the same workload ({len(host_sets)} input sets, 3 passes), "
                                            f"{dt:.2f} s wall on {all_threads} threads "
                                            f"(about {dt * all_threads:.0f} core-seconds)",
                                  "single_core": {"value": npos1 / dt1, "unit": "positions/s", "cores": 1,
                                                  "sample": f"{npos1} positions (2 input sets), {dt1:.2f} s on one thread"}}
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
