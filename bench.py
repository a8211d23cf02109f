#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" = one hmm_smooth call + one hmm_viterbi call (element construction, forward and
reversed scans, marginal combine, max-plus scan, back-pointer scan, path write) on the
D=4, T=2^20 burst-channel workload, inputs resident in HBM.  Steps rotate over several distinct
input/output buffer sets so that consecutive steps do not find their data in the 256 MB
Infinity Cache.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2|C3|C4|C5]
    python bench.py --ge-sweep      (the paper's Gilbert-Elliott model over a range of T, Sec. VI)
    python bench.py --machine-peaks (what library copy / GEMM kernels sustain on this GPU, beside the published peaks)

--workload selects one of the other synthetic configurations (D=32 long sequence, 256 x D=16
batch, D=128 compute-bound) for the same measurement; the headline line is the default, C2.
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
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X published dense FP32 matrix-core rate
# Max-plus is one add and one max per term and the two do not fuse into one instruction: the vector
# units issue 256 CUs x 128 lanes x 2.4 GHz = 78.6e12 such instructions per second (half the FMA-based
# 157.3 TFLOP/s figure, which counts two operations per lane and clock).
VALU_F32_PEAK_TOPS = 78.6
SMOOTH_KERNELS = ("sd_reduce_sp", "sd_carry_sp", "sd_smooth_apply", "sd_smooth_fused",
                  "ld_rowmax", "ld_aggregate", "ld_product", "ld_carry", "ld_apply", "ld_combine", "ld_finalize", "ld_repair")
VITERBI_KERNELS = ("sd_reduce_mp", "sd_carry_mp", "sd_viterbi_forward", "sd_viterbi_suffix", "sd_viterbi_path",
                   "sd_viterbi_fused",
                   "lv_aggregate", "lv_tree_product", "lv_carry", "lv_forward", "lv_group_maps", "lv_suffix",
                   "lv_group_chase", "lv_path")
WORKLOADS = {
    "C2": ("config2", "single HMM, D=4, T=2^20, burst-channel-style model, binary observations", 24, 300, 30),
    "C3": ("config3", "single HMM, D=32, T=2^18, Dirichlet(0.5) transitions, Gaussian emissions", 8, 40, 5),
    "C4": ("config4", "256 independent HMMs, D=16, T=4096 each, categorical emissions over 8 symbols", 6, 40, 5),
    "C5": ("config5", "single HMM, D=128, T=2^16, banded-plus-noise transitions, Gaussian emissions on a grid", 8, 20, 3),
}


def kernel_roofline(name: str, avg_us: float, B: int, T: int, D: int) -> dict:
    """Roofline entry of one kernel: what bounds it, its algorithmic work per launch, the rate achieved."""
    sec = avg_us * 1e-6
    if name == "ld_aggregate":
        # one D x D by D x D product per element of the sequence (Definition 3): 2 D^3 flops
        work = 2.0 * D ** 3 * B * T
        ach = work / sec / 1e12
        return {"bound": "mfma", "kernel": name, "avg_us": avg_us, "achieved": ach, "peak": MFMA_F32_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / MFMA_F32_PEAK_TFLOPS, "traffic": None,
                "algorithmic_flops_per_launch": work}
    if name == "lv_aggregate":
        # one max-plus D x D by D x D product per element (Definition 5): D^3 adds and D^3 maxima
        work = 2.0 * D ** 3 * B * T
        ach = work / sec / 1e12
        return {"bound": "alu", "kernel": name, "avg_us": avg_us, "achieved": ach, "peak": VALU_F32_PEAK_TOPS,
                "unit": "TOP/s", "frac": ach / VALU_F32_PEAK_TOPS, "traffic": None,
                "algorithmic_ops_per_launch": work}
    # streaming kernels: smoother reads log-likelihoods and writes marginals (8 D bytes per step of the
    # sequence), Viterbi reads log-likelihoods and writes the int32 path (4 D + 4)
    alg_bytes = B * T * (8 * D if name in SMOOTH_KERNELS else 4 * D + 4)
    ach = alg_bytes / sec / 1e9
    return {"bound": "hbm", "kernel": name, "avg_us": avg_us, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_launch": alg_bytes}


def c5_leg(steps: int = 10, warmup: int = 3) -> dict:
    """The compute-bound configuration beside the headline one: hmm_smooth on C5 (D=128, T=2^16), timed the same way
    (inputs resident, `steps` calls between two synchronisations, then the same calls with per-kernel events).
    The D x D element products of the sum-product scan run on the matrix cores: ld_aggregate's rate, and the whole
    call's, against the published dense FP32 matrix rate."""
    import torch

    import paper_2102_05743_amd as hmm
    from paper_2102_05743_amd import workloads as wl

    dev = torch.device("cuda:0")
    p = wl.config5()
    T, D, B = p.T, p.D, p.batch
    prior, A = torch.from_numpy(p.prior).to(dev), torch.from_numpy(p.A).to(dev)
    nsets = 4
    ll0 = torch.from_numpy(p.loglik).to(dev)
    lls = [ll0] + [ll0.clone() for _ in range(nsets - 1)]
    margs = [torch.empty((B, T, D), dtype=torch.float32, device=dev) for _ in range(nsets)]
    logliks = torch.empty((nsets, B), dtype=torch.float64, device=dev)
    ws = hmm.new_workspace(hmm.hmm_workspace_bytes(T, D, B)[0], dev)
    calls = [hmm.hmm_smooth_prepare(prior, A, lls[s], marginals=margs[s], loglik_out=logliks[s], workspace=ws)
             for s in range(nsets)]
    for i in range(warmup):
        calls[i % nsets]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        calls[(warmup + i) % nsets]()
    torch.cuda.synchronize()
    smooth_ms = (time.perf_counter() - t0) * 1e3 / steps
    hmm.hmm_kernel_timing_enable(True)
    for i in range(steps):
        calls[(warmup + i) % nsets]()
    torch.cuda.synchronize()
    kt = hmm.hmm_kernel_timing_get()
    hmm.hmm_kernel_timing_enable(False)
    agg_ms, agg_n = kt.get("ld_aggregate", (0.0, 0))
    agg_us = 1e3 * agg_ms / max(agg_n, 1)
    call_us = sum(1e3 * ms for ms, _ in kt.values()) / steps
    flops = 2.0 * D ** 3 * B * T        # one D x D by D x D product per element (Definition 3)
    return {"workload": "C5: " + WORKLOADS["C5"][1], "steps": steps, "warmup": warmup, "smooth_ms": smooth_ms,
            "ld_aggregate_us": agg_us, "call_kernel_us": call_us,
            "mfma_frac_kernel": flops / (agg_us * 1e-6) / 1e12 / MFMA_F32_PEAK_TFLOPS if agg_us > 0 else None,
            "mfma_frac_call": flops / (call_us * 1e-6) / 1e12 / MFMA_F32_PEAK_TFLOPS if call_us > 0 else None,
            "mfma_frac_call_wall": flops / (smooth_ms * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS,
            "peak_TFLOPs": MFMA_F32_PEAK_TFLOPS, "loglik": float(logliks[0, 0])}


def ge_sweep() -> int:
    """Run time against sequence length on the paper's Gilbert-Elliott model (Sec. VI, Figs. 5-6):
    one JSON line with, per T, the median time of an hmm_smooth and an hmm_viterbi call (inputs
    resident, back-to-back enqueue of `reps` calls / reps) and the sequential fp64 oracle beside it."""
    import numpy as np
    import torch

    import paper_2102_05743_amd as hmm
    from paper_2102_05743_amd import workloads as wl
    import oracle

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    hmm.load_library()
    dev = torch.device("cuda:0")
    rows = []
    for T in (100, 1000, 10_000, 100_000, 1 << 20, 1 << 22, 1 << 24):
        p = wl.gilbert_elliott(T=T)
        prior = torch.from_numpy(p.prior).to(dev)
        A = torch.from_numpy(p.A).to(dev)
        ll = torch.from_numpy(p.loglik).to(dev)
        marg = torch.empty_like(ll)
        path = torch.empty((1, T), dtype=torch.int32, device=dev)
        out = torch.empty((2, 1), dtype=torch.float64, device=dev)
        ws_s, ws_v = hmm.hmm_workspace_bytes(T, p.D, 1)
        ws = hmm.new_workspace(max(ws_s, ws_v), dev)
        calls = {"smooth": hmm.hmm_smooth_prepare(prior, A, ll, marginals=marg, loglik_out=out[0], workspace=ws),
                 "viterbi": hmm.hmm_viterbi_prepare(prior, A, ll, path=path, logprob_out=out[1], workspace=ws)}
        row = {"T": T}
        reps = 100 if T <= (1 << 20) else 20
        for name, fn in calls.items():
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            times = []
            for _ in range(5):
                t0 = time.perf_counter()
                for _ in range(reps):
                    fn()
                torch.cuda.synchronize()
                times.append((time.perf_counter() - t0) / reps)
            row[name + "_us"] = 1e6 * float(np.median(times))
        if T <= (1 << 22):
            c0 = time.perf_counter()
            oracle.smooth(p.prior[0], p.A[0], p.loglik[0], want_filtered=False)
            c1 = time.perf_counter()
            oracle.viterbi(p.prior[0], p.A[0], p.loglik[0])
            c2 = time.perf_counter()
            row["oracle_smooth_us"] = 1e6 * (c1 - c0)
            row["oracle_viterbi_us"] = 1e6 * (c2 - c1)
        rows.append(row)
    print(json.dumps({"sweep": "Gilbert-Elliott model (Sec. VI), D=4, one sequence", "unit": "us per call",
                      "rows": rows}))
    return 0


def machine_peaks() -> int:
    """What this GPU sustains on plain library kernels, beside the published peaks the rooflines use: device
    copy, fill and read bandwidth over 1 GiB buffers and an FP32 GEMM.  Context for the roofline fractions (a
    fraction of the published peak understates a kernel that runs at the rate the memory system can deliver)."""
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    props = torch.cuda.get_device_properties(0)
    n = 1 << 28                                   # 1 GiB of float32, four times the Infinity Cache
    a = torch.ones(n, dtype=torch.float32, device=dev)
    b = torch.empty_like(a)

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    t_copy = timed(lambda: b.copy_(a))
    t_fill = timed(lambda: b.fill_(1.0))
    t_read = timed(lambda: torch.max(a))
    m = 8192
    x = torch.randn((m, m), dtype=torch.float32, device=dev)
    y = torch.randn((m, m), dtype=torch.float32, device=dev)
    z = torch.empty_like(x)
    prev = torch.backends.cuda.matmul.allow_tf32
    torch.backends.cuda.matmul.allow_tf32 = False
    t_gemm = timed(lambda: torch.matmul(x, y, out=z), reps=10)
    torch.backends.cuda.matmul.allow_tf32 = prev
    out = {"device": props.name, "compute_units": props.multi_processor_count,
           "memory_GiB": round(props.total_memory / 2 ** 30, 1),
           "copy_GBs": 2 * 4 * n / t_copy / 1e9, "fill_GBs": 4 * n / t_fill / 1e9, "read_GBs": 4 * n / t_read / 1e9,
           "sgemm_8192_TFLOPs": 2.0 * m ** 3 / t_gemm / 1e12,
           "published": {"hbm_GBs": HBM_PEAK_GBS, "mfma_f32_TFLOPs": MFMA_F32_PEAK_TFLOPS, "valu_f32_TOPs": VALU_F32_PEAK_TOPS}}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="C2")
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--sets", type=int, default=None, help="distinct buffer sets rotated over (cold-cache timing)")
    ap.add_argument("--T", type=int, default=None, help="sequence length (default: the configuration's own)")
    ap.add_argument("--batch-copies", type=int, default=1,
                    help="run this many copies of the workload's sequences as one batch (a scaled run that shows the "
                         "kernels' streaming rate; supporting evidence, not the configured shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-c5", action="store_true", help="skip the short C5 (D=128) leg that a default C2 run appends")
    ap.add_argument("--two-streams", action="store_true",
                    help="also replay a graph that runs the two calls of a step on two streams (supporting figure; left out "
                         "by default so that every launch of a default run is an undisturbed one)")
    ap.add_argument("--repeats", type=int, default=5, help="further timed regions of K steps, for the spread in `extra`")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 32 MiB per step (a kernel of known traffic, for scaling "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--ge-sweep", action="store_true",
                    help="time both calls on the paper's Gilbert-Elliott model for T = 1e2 ... 2^24 instead")
    ap.add_argument("--machine-peaks", action="store_true",
                    help="measure what plain library kernels sustain on this GPU (copy / fill / read bandwidth, FP32 GEMM)")
    args = ap.parse_args()
    if args.machine_peaks:
        return machine_peaks()
    if args.ge_sweep:
        if args.gpus != 1:
            print("bench.py: this build runs on ONE GPU only; run it with --gpus 1", file=sys.stderr)
            return 2
        return ge_sweep()
    gen_name, wl_text, d_sets, d_steps, d_warmup = WORKLOADS[args.workload]
    args.steps = d_steps if args.steps is None else args.steps
    args.warmup = d_warmup if args.warmup is None else args.warmup
    args.sets = d_sets if args.sets is None else args.sets
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
    gen = getattr(wl, gen_name)
    p = gen() if args.T is None else gen(T=args.T)
    if args.batch_copies > 1:
        p.loglik = np.ascontiguousarray(np.tile(p.loglik, (args.batch_copies, 1, 1)))
        if not p.shared_model:
            p.prior = np.ascontiguousarray(np.tile(p.prior, (args.batch_copies, 1)))
            p.A = np.ascontiguousarray(np.tile(p.A, (args.batch_copies, 1, 1)))
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
    ws_smooth = hmm.new_workspace(ws_s, dev)       # allocated and prepared once, outside every timed region
    ws_viterbi = hmm.new_workspace(ws_v, dev)

    cal_src = cal_dst = None
    if args.copy_calibration:
        cal_src = torch.ones((8 << 20,), dtype=torch.float32, device=dev)     # 32 MiB
        cal_dst = torch.empty_like(cal_src)

    # arguments marshalled once per buffer set: a step is then two bare C-ABI calls
    smooth_calls = [hmm.hmm_smooth_prepare(prior, A, lls[s], marginals=margs[s], loglik_out=logliks[s],
                                           workspace=ws_smooth) for s in range(nsets)]
    viterbi_calls = [hmm.hmm_viterbi_prepare(prior, A, lls[s], path=paths[s], logprob_out=logprobs[s],
                                             workspace=ws_viterbi) for s in range(nsets)]

    def step(i: int) -> None:
        s = i % nsets
        if cal_src is not None:
            cal_dst.copy_(cal_src)
        smooth_calls[s]()
        viterbi_calls[s]()

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

    # ---- the spread: the same region a few more times (the headline stays the first one)
    region_ms = [ms_per_step]
    for _ in range(max(0, args.repeats)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        region_ms.append((time.perf_counter() - t0) * 1e3 / args.steps)

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

    # ---- the same steps recorded once into a HIP graph and replayed (every launch of the library is a
    # kernel, so calls can be captured): what a serving loop pays per step without per-launch host work.
    # One graph holds a step on every buffer set, so replays stay cold-cache.  Supporting figure only.
    ms_per_step_graph = None
    ms_per_step_two_streams = None
    if not args.copy_calibration:
        try:
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for s in range(nsets):
                    hmm.hmm_smooth(prior, A, lls[s], marginals=margs[s], loglik_out=logliks[s], workspace=ws_smooth)
                    hmm.hmm_viterbi(prior, A, lls[s], path=paths[s], logprob_out=logprobs[s], workspace=ws_viterbi)
            reps = max(1, args.steps // nsets)
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                graph.replay()
            torch.cuda.synchronize()
            ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / (reps * nsets)
        except Exception as e:   # never let the supporting figure break the benchmark line
            print(f"bench.py: graph replay skipped ({e})", file=sys.stderr)
        # ---- the same graph with the two calls of a step on two streams (they are independent: both only read the
        # inputs), joined before the next step: the two kernels share the compute units.  Supporting figure only.
        try:
            if not args.two_streams:
                raise StopIteration
            side, side2 = torch.cuda.Stream(), torch.cuda.Stream()
            graph2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph2, stream=side):
                for s in range(nsets):
                    side2.wait_stream(side)
                    hmm.hmm_smooth(prior, A, lls[s], marginals=margs[s], loglik_out=logliks[s], workspace=ws_smooth)
                    with torch.cuda.stream(side2):
                        hmm.hmm_viterbi(prior, A, lls[s], path=paths[s], logprob_out=logprobs[s], workspace=ws_viterbi)
                    side.wait_stream(side2)
            reps = max(1, args.steps // nsets)
            graph2.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                graph2.replay()
            torch.cuda.synchronize()
            ms_per_step_two_streams = (time.perf_counter() - t0) * 1e3 / (reps * nsets)
            for ws_ in (ws_smooth, ws_viterbi):   # both kernels need all their tiles resident: check that they were
                if hmm.hmm_workspace_status(ws_) != 0:
                    ms_per_step_two_streams = None
                    hmm.hmm_workspace_init(ws_)
            torch.cuda.synchronize()
        except StopIteration:
            pass
        except Exception as e:
            print(f"bench.py: two-stream graph replay skipped ({e})", file=sys.stderr)

    state_steps = B * T * D
    value = state_steps / (ms_per_step * 1e-3)

    per_kernel = {k: {"avg_us": 1e3 * ms / max(n, 1), "launches": n} for k, (ms, n) in ktimes.items()}
    smooth_us = sum(v["avg_us"] * v["launches"] for k, v in per_kernel.items() if k in SMOOTH_KERNELS) / args.steps
    viterbi_us = sum(v["avg_us"] * v["launches"] for k, v in per_kernel.items() if k in VITERBI_KERNELS) / args.steps
    dom = max(per_kernel.items(), key=lambda kv: kv[1]["avg_us"] * kv[1]["launches"])
    dom_name, dom_us = dom[0], dom[1]["avg_us"]
    def with_traffic(r, name):
        """HBM bytes per launch from the committed rocprofv3 counter summary of this kernel and workload, if there is one."""
        tfile = os.path.join(ROOT, "profiles", "traffic_" + name + "_" + args.workload + ".json")
        if os.path.exists(tfile):
            try:
                r["traffic"] = json.load(open(tfile)).get("traffic_bytes_per_launch")
            except Exception:
                pass
        return r

    def with_issue(r, name):
        """Vector-issue view beside the HBM one: wave instructions per launch (committed counter summary) x 4 cycles
        (a 64-lane instruction on a 16-lane SIMD) against the launch's duration on all SIMDs."""
        vfile = os.path.join(ROOT, "profiles", "valu_instr_" + args.workload + ".json")
        if os.path.exists(vfile):
            try:
                n = json.load(open(vfile))["valu_instr_per_launch"].get(name)
                if n:
                    simds, clock = 256 * 4, 2.4e9
                    r["valu_issue"] = {"bound": "alu", "wave_instr_per_launch": n,
                                       "frac": n * 4.0 / (r["avg_us"] * 1e-6 * clock * simds)}
            except Exception:
                pass
        return r

    roofline = with_issue(with_traffic(kernel_roofline(dom_name, dom_us, B, T, D), dom_name), dom_name)
    roofline["smooth_call"] = {"kernel_us": smooth_us,
                               "frac": (B * T * 8 * D) / (smooth_us * 1e-6) / 1e9 / HBM_PEAK_GBS if smooth_us > 0 else None}
    roofline["viterbi_call"] = {"kernel_us": viterbi_us,
                                "frac": (B * T * (4 * D + 4)) / (viterbi_us * 1e-6) / 1e9 / HBM_PEAK_GBS
                                if viterbi_us > 0 else None}
    # every kernel that takes at least a tenth of the step, against its own bound
    other_rooflines = [with_issue(with_traffic(kernel_roofline(k, v["avg_us"], B, T, D), k), k) for k, v in per_kernel.items()
                       if k != dom_name and v["avg_us"] * v["launches"] / args.steps >= 0.1 * (smooth_us + viterbi_us)]

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        best_s, best_v = float("inf"), float("inf")
        reps = 3 if args.workload == "C2" else 1
        nseq = min(B, 64)          # bounded sample of a batched workload: its first sequences
        for _ in range(reps):
            c0 = time.perf_counter()
            for b in range(nseq):
                m = 0 if p.shared_model else b
                oracle.smooth(p.prior[m], p.A[m], p.loglik[b], want_filtered=False)
            c1 = time.perf_counter()
            for b in range(nseq):
                m = 0 if p.shared_model else b
                oracle.viterbi(p.prior[m], p.A[m], p.loglik[b])
            c2 = time.perf_counter()
            best_s, best_v = min(best_s, c1 - c0), min(best_v, c2 - c1)
        sample = (f"the full workload (one sequence, T={T}, D={D})" if B == 1 else
                  f"{nseq} of the {B} sequences (T={T}, D={D} each)")
        cpu_baseline = {"value": nseq * T * D / (best_s + best_v), "unit": "state-steps/s", "cores": 1,
                        "kind": "oracle", "sample": sample + f", smoother + Viterbi, best of {reps}; the recursion is "
                        "sequential in T so one thread is all it can use",
                        "smooth_s": best_s, "viterbi_s": best_v}

    t_text = f"2^{T.bit_length() - 1}" if T & (T - 1) == 0 else str(T)
    out = {
        "metric": f"state-steps/sec (T*D/s), smoother + Viterbi, D={D}, T={t_text}" + (f", batch {B}" if B > 1 else ""),
        "value": value, "unit": "state-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {wl_text}" + ("" if args.T is None else f" (T overridden: {T})") +
                   ("" if args.batch_copies == 1 else f" (scaled run: {args.batch_copies} copies as one batch)"),
                   "batch": B, "buffer_sets": nsets, "step": "hmm_smooth + hmm_viterbi"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "extra": {"ms_per_step_regions": {"n": len(region_ms), "median": float(np.median(region_ms)),
                                          "min": min(region_ms), "max": max(region_ms)},
                  "ms_per_step_graph_replay_two_streams": ms_per_step_two_streams,
                  "ms_per_step_with_kernel_events": ms_per_step_events, "ms_per_step_warm_cache": ms_per_step_warm,
                  "ms_per_step_graph_replay": ms_per_step_graph,
                  "smooth_state_steps_per_s": state_steps / (smooth_us * 1e-6) if smooth_us > 0 else None,
                  "viterbi_state_steps_per_s": state_steps / (viterbi_us * 1e-6) if viterbi_us > 0 else None,
                  "per_kernel": per_kernel, "other_rooflines": other_rooflines,
                  "loglik": float(logliks[0, 0]), "logprob": float(logprobs[0, 0])},
    }
    if args.workload == "C2" and not args.no_c5 and args.T is None and args.batch_copies == 1 and not args.copy_calibration:
        del lls, margs, paths
        torch.cuda.empty_cache()
        try:
            out["extra"]["c5"] = c5_leg()
        except Exception as e:
            print(f"bench.py: C5 leg failed ({e})", file=sys.stderr)
            out["extra"]["c5"] = None
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
