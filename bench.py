#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" = one hmm_smooth call + one hmm_viterbi call (element construction, forward and
reversed scans, marginal combine, max-plus scan, back-pointer scan, path write) on the
D=4, T=2^20 burst-channel workload, inputs resident in HBM.  Steps rotate over several distinct
input/output buffer sets so that consecutive steps do not find their data in the 256 MB
Infinity Cache.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
SMOOTH_KERNELS = ("sd_reduce_sp", "sd_carry_sp", "sd_smooth_apply", "sd_finalize", "sd_clear_sp", "sd_smooth_fused")
VITERBI_KERNELS = ("sd_reduce_mp", "sd_carry_mp", "sd_viterbi_forward", "sd_viterbi_suffix", "sd_viterbi_path",
                   "sd_clear_mp", "sd_viterbi_fused")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--sets", type=int, default=24, help="distinct buffer sets rotated over (cold-cache timing)")
    ap.add_argument("--T", type=int, default=1 << 20, help="sequence length (default: the headline 2^20)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 32 MiB per step (a kernel of known traffic, for scaling "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2102_05743_amd as hmm
    from paper_2102_05743_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    hmm.load_library()            # fails loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    p = wl.config2(T=args.T)
    T, D, B = p.T, p.D, p.batch
    nsets = max(1, args.sets)
    prior = torch.from_numpy(p.prior).to(dev)
    A = torch.from_numpy(p.A).to(dev)
    ll0 = torch.from_numpy(p.loglik).to(dev)
    lls = [ll0] + [ll0.clone() for _ in range(nsets - 1)]
    margs = [torch.empty((B, T, D), dtype=torch.float32, device=dev) for _ in range(nsets)]
    paths = [torch.empty((B, T), dtype=torch.int32, device=dev) for _ in range(nsets)]
    logliks = torch.empty((nsets, B), dtype=torch.float64, device=dev)
    logprobs = torch.empty((nsets, B), dtype=torch.float64, device=dev)
    ws_s, ws_v = hmm.hmm_workspace_bytes(T, D, B)
    ws_smooth = torch.empty((max(ws_s, 256),), dtype=torch.uint8, device=dev)
    ws_viterbi = torch.empty((max(ws_v, 256),), dtype=torch.uint8, device=dev)

    cal_src = cal_dst = None
    if args.copy_calibration:
        cal_src = torch.ones((8 << 20,), dtype=torch.float32, device=dev)     # 32 MiB
        cal_dst = torch.empty_like(cal_src)

    def step(i: int) -> None:
        s = i % nsets
        if cal_src is not None:
            cal_dst.copy_(cal_src)
        hmm.hmm_smooth(prior, A, lls[s], marginals=margs[s], loglik_out=logliks[s], workspace=ws_smooth)
        hmm.hmm_viterbi(prior, A, lls[s], path=paths[s], logprob_out=logprobs[s], workspace=ws_viterbi)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- the same K steps again with a HIP start/stop event pair attached to every kernel dispatch
    # (hipExtLaunchKernel, same stream): per-kernel durations for the roofline.  Kept out of the
    # region above because the instrumented launch path costs host time per launch.
    hmm.hmm_kernel_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ktimes = hmm.hmm_kernel_timing_get()
    hmm.hmm_kernel_timing_enable(False)
    ms_per_step_events = (t1 - t0) * 1e3 / args.steps

    # ---- warm-cache variant (one buffer set) for reference
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(0)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step_warm = (t1 - t0) * 1e3 / args.steps

    state_steps = B * T * D
    value = state_steps / (ms_per_step * 1e-3)

    per_kernel = {k: {"avg_us": 1e3 * ms / max(n, 1), "launches": n} for k, (ms, n) in ktimes.items()}
    smooth_us = sum(v["avg_us"] * v["launches"] for k, v in per_kernel.items() if k in SMOOTH_KERNELS) / args.steps
    viterbi_us = sum(v["avg_us"] * v["launches"] for k, v in per_kernel.items() if k in VITERBI_KERNELS) / args.steps
    dom = max(per_kernel.items(), key=lambda kv: kv[1]["avg_us"] * kv[1]["launches"])
    dom_name, dom_us = dom[0], dom[1]["avg_us"]
    # algorithmic bytes per step of the sequence: smoother 8*D (read log-likelihoods, write marginals),
    # Viterbi 4*D + 4 (read log-likelihoods, write the int32 path); one launch covers all B*T steps
    alg_bytes = B * T * (8 * D if dom_name in SMOOTH_KERNELS else 4 * D + 4)
    achieved = alg_bytes / (dom_us * 1e-6) / 1e9
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "traffic_" + dom_name + "_C2.json")
    if os.path.exists(tfile):
        try:
            traffic = json.load(open(tfile)).get("traffic_bytes_per_launch")
        except Exception:
            traffic = None
    roofline = {"bound": "hbm", "kernel": dom_name, "avg_us": dom_us, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "algorithmic_bytes_per_launch": alg_bytes,
                "smooth_call": {"kernel_us": smooth_us, "frac": (B * T * 8 * D) / (smooth_us * 1e-6) / 1e9 / HBM_PEAK_GBS
                                if smooth_us > 0 else None},
                "viterbi_call": {"kernel_us": viterbi_us,
                                 "frac": (B * T * (4 * D + 4)) / (viterbi_us * 1e-6) / 1e9 / HBM_PEAK_GBS
                                 if viterbi_us > 0 else None}}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        best_s, best_v = float("inf"), float("inf")
        reps = 3
        for _ in range(reps):
            c0 = time.perf_counter()
            oracle.smooth(p.prior[0], p.A[0], p.loglik[0], want_filtered=False)
            c1 = time.perf_counter()
            oracle.viterbi(p.prior[0], p.A[0], p.loglik[0])
            c2 = time.perf_counter()
            best_s, best_v = min(best_s, c1 - c0), min(best_v, c2 - c1)
        cpu_baseline = {"value": state_steps / (best_s + best_v), "unit": "state-steps/s", "cores": 1,
                        "kind": "oracle", "sample": f"the full workload (one sequence, T={T}, D={D}), smoother + "
                        f"Viterbi, best of {reps}; the recursion is sequential in T so one thread is all it can use",
                        "smooth_s": best_s, "viterbi_s": best_v}

    out = {
        "metric": "state-steps/sec (T*D/s), smoother + Viterbi, D=4, T=2^20",
        "value": value, "unit": "state-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"C2: single HMM, D={D}, T={T}, burst-channel-style model, binary observations",
                   "batch": B, "buffer_sets": nsets, "step": "hmm_smooth + hmm_viterbi"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "extra": {"ms_per_step_with_kernel_events": ms_per_step_events, "ms_per_step_warm_cache": ms_per_step_warm,
                  "smooth_state_steps_per_s": state_steps / (smooth_us * 1e-6) if smooth_us > 0 else None,
                  "viterbi_state_steps_per_s": state_steps / (viterbi_us * 1e-6) if viterbi_us > 0 else None,
                  "per_kernel": per_kernel,
                  "loglik": float(logliks[0, 0]), "logprob": float(logprobs[0, 0])},
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
