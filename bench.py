#!/usr/bin/env python3
"""Benchmark of the MaaSO scoring path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is already resident in
HBM: maaso_placement_sweep over every candidate deployment (profile evaluation, queue wait, SLO
fetch, per-triple latency, SLO check, per-request feasibility, per-candidate reduction, best
candidate) followed by maaso_score_assign of the same requests on the winning deployment (best
instance per request, admitted count).  For the two distributor workloads a step is
maaso_score_assign alone (windowed for the online distributor).

With no --workload the run is the five-workload report: the headline (`value`, `roofline`,
`cpu_baseline`) is the skewed-stress sweep (8192 candidates x 131,072 requests x 128 instances, the
largest of the five), timed with exactly --steps steps after --warmup warm-up steps, and `per_config`
carries the same fields for the other four workloads and for the streaming distributor shape on
which HBM, not the VALU, binds.  Every entry is compared with the CPU oracle in the same run
(`oracle_check`): satisfied counts per candidate for the sweeps, chosen instance / slack / admitted
count / final state for the distributors.

Prints ONE JSON line.  The roofline of each entry is that of its dominant kernel, timed with HIP
events recorded inside the library directly around that kernel, on the stream it is launched on.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

# MI355X fp32 vector peak: 157.3 TFLOP/s published = 256 compute units x 4 SIMDs x 32 lanes per clock
# x 2.4 GHz x 2 flop per fused multiply-add, i.e. 78.6e12 VALU lane operations per second.  A
# min, add or compare occupies a lane slot exactly as an fma does, so the kernels are priced in lane
# operations; the flop figure (an fma counts two, everything else one) is given beside it.
VALU_PEAK_TLANEOPS = 256 * 4 * 32 * 2.4e9 / 1e12
FP32_VECTOR_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0

# Sweep, per (request, instance) pair that reaches the latency loop: prefill fma, queue-wait add, and
# half of a three-input minimum (one v_min3_f32 folds two pairs into the running minimum): 2.5
# instruction slots per pair is the least this instruction set needs.  Where an instance's queue wait
# is exactly zero (fresh instances, the placer's usual candidates) the add changes nothing and the
# kernel leaves it out: 1.5 slots.  The roofline fraction uses these figures with the kernel's own
# counts of both kinds of pair.  Counted as operations of the model (fma, add, min) a pair is 3; that
# figure is reported beside it and exceeds the slot fraction.
SWEEP_SLOTS_PER_PAIR = 2.5
SWEEP_SLOTS_PER_PAIR_NO_WAIT = 1.5
SWEEP_OPERATIONS_PER_PAIR = 3
SWEEP_FLOP_PER_PAIR = 4          # fma = 2
SWEEP_FLOP_PER_PAIR_NO_WAIT = 3
# Distributor, per triple: 2 fma, 1 add, 2 sub, 2 mul, 2 min, 1 compare, 2 selects (the between-token
# margin comes from a per-(class, instance) table).
ASSIGN_LANEOPS_PER_TRIPLE = 12
# Algorithmic HBM bytes of the distributor per request: prompt_len 4 + out_len 4 + class 1 in,
# chosen 4 + slack 4 out.
ASSIGN_BYTES_PER_REQUEST = 17
# Composite serving score (Sec. IV-D, Eq. 6): alpha and beta as in the paper's evaluation; gamma_T a
# throughput no deployment of these workloads exceeds (tokens/s), gamma_L the largest acceptable wait (s).
SCORE_WEIGHTS = (4.0, 0.3, 16384.0, 2.0)

# What the paper itself reports (its abstract; Sec. V-A "Hardware Environment" and "Workloads";
# Sec. V-B "Solver Overhead").  It prints no throughput of the scoring path, so none of this is a
# target for the figures of this run.
PAPER_CONTEXT = (
    "MaaSO (arXiv 2509.06362) reports +15-30 % SLO-satisfaction ratio and -40-60 % response latency "
    "(time to first token) against AlpaServe and Selective Replication (abstract), on a SIMULATED "
    "cluster of AWS p3.16xlarge nodes (8x V100 16 GB) driven by profiles measured with vLLM in "
    "bfloat16 on 8x H20 96 GB (2x Xeon Platinum 8468V) and 2x RTX 3090 24 GB (2x Xeon E5-2680) servers "
    "(Sec. V-A); default scale 24 GPUs, 17,000 arrivals per 3600 s, CV 2 (Sec. V-A); solver overhead "
    "of the baselines above 1000 s on 32-GPU clusters, MaaSO 'substantially lower' without a number "
    "(Sec. V-B, Solver Overhead). The paper prints no triples/s or per-evaluation time for this "
    "path: context, not a target.")

# HBM bytes per launch of the dominant kernel, from rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by the
# readings of a 1 GiB copy kernel (the summaries named here hold the readings and the factor).  A
# figure only holds for the kernel it was taken with: it is reported while the digest of that kernel's
# source files matches and as null - with both digests, so that the staleness is visible - afterwards.
KERNEL_SOURCES = {
    "sweep_kernel": ("device_model.hpp", "sweep_kernels.hpp"),
    "assign_static_kernel": ("device_model.hpp", "sweep_kernels.hpp", "assign_kernels.hpp"),
    "assign_window_kernel": ("device_model.hpp", "sweep_kernels.hpp", "assign_kernels.hpp",
                             "window_kernels.hpp"),
}
TRAFFIC = {
    # workload name: (kernel, bytes per launch, digest of the kernel's sources at measurement, summary)
    "cfg4_skewed_stress": ("sweep_kernel", 3.0879e7, "4a4d88dd875e78ec", "profiles/sweep_kernel_cfg4.md"),
    "cfg1_placer_sweep": ("sweep_kernel", 5.641e6, "4a4d88dd875e78ec", "profiles/sweep_kernel_cfg1.md"),
    "streaming_i4": ("assign_static_kernel", 1.1410e9, "db880294941b8bee",
                     "profiles/assign_static_kernel_stream.md"),
}

REPORT_OTHERS = ("cfg0", "cfg1", "cfg2", "cfg3", "stream")
CHECK_THREADS = 8      # oracle instances run side by side over disjoint candidate ranges (checks only)


def kernel_source_digest(kernel: str) -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES[kernel]:
        h.update((ROOT / "paper_2509_06362_amd" / "csrc" / name).read_bytes())
    return h.hexdigest()[:16]


def measured_traffic(workload_name: str):
    """(bytes or None, provenance) of the dominant kernel's measured HBM traffic per launch."""
    entry = TRAFFIC.get(workload_name)
    if entry is None:
        return None, {"source": None, "note": "no counter run on record for this workload"}
    kernel, nbytes, digest, source = entry
    now = kernel_source_digest(kernel)
    info = {"source": source, "kernel_digest_at_measurement": digest, "kernel_digest_now": now,
            "stale": now != digest, "bytes_at_measurement": nbytes}
    return (None if now != digest else nbytes), info


def make_workload(name: str):
    from dataclasses import replace
    from paper_2509_06362_amd import workloads as W
    if name == "cfg1":
        return W.config1()
    if name == "cfg3":
        return W.config3()
    if name == "cfg4":
        return W.config4()
    if name == "cfg0":
        return W.config0()
    if name == "cfg2":
        return W.config2()
    if name == "stream":
        return W.streaming_shape()
    if name == "cfg4w":  # config 4 scored capacity-aware: windows of 4096 over its bursty arrivals
        w = W.config4()
        return replace(w, name=w.name + "_windowed", window=4096)
    if name == "cfg4w1":  # config 4 request by request: every request meets the state left by all earlier ones
        w = W.config4()
        return replace(w, name=w.name + "_request_by_request", window=1)
    if name == "cfg4score":  # the same, every candidate scored with the composite serving score
        w = W.config4()
        return replace(w, name=w.name + "_windowed_score", window=4096)
    raise SystemExit(f"unknown workload {name}")


# ------------------------------------------------------------------------------------------------
# the oracle leg: a timed single-threaded sample (cpu_baseline) and the comparison with the GPU
# ------------------------------------------------------------------------------------------------

def _sweep_oracle(w, lo, hi):
    import oracle
    if w.name.endswith("_score"):
        return oracle.placement_score(w, *SCORE_WEIGHTS, window=int(w.window), c_begin=lo, c_end=hi)["sat_count"]
    if w.window:
        return oracle.placement_sweep_windowed(w, window=int(w.window), c_begin=lo, c_end=hi)["sat_count"]
    return oracle.placement_sweep(w, lo, hi)["sat_count"]


def _sweep_oracle_parallel(w, lo, hi):
    """Counts of candidates [lo, hi): independent single-threaded oracle calls over disjoint ranges."""
    import numpy as np
    out = np.zeros(w.n_cand, np.uint32)
    if hi <= lo:
        return out
    n = min(CHECK_THREADS, hi - lo)
    cuts = [lo + (hi - lo) * i // n for i in range(n + 1)]
    with ThreadPoolExecutor(max_workers=n) as pool:
        for (a, b), cnt in zip(zip(cuts[:-1], cuts[1:]),
                               pool.map(lambda ab: _sweep_oracle(w, ab[0], ab[1]), zip(cuts[:-1], cuts[1:]))):
            out[a:b] = cnt[a:b]
    return out


def sweep_cpu_leg(w, gpu_counts, budget_triples: float, min_checked: int):
    """Timed single-threaded oracle on candidates [0, n) (about budget_triples triples), then the
    comparison of the GPU's satisfied counts with the oracle's on candidates [0, max(n, min_checked))."""
    import numpy as np
    per_cand = w.n_req * w.n_inst.astype(np.int64)
    n = int(np.searchsorted(np.cumsum(per_cand), budget_triples)) + 1
    n = max(1, min(n, w.n_cand))
    t0 = time.perf_counter()
    ref = _sweep_oracle(w, 0, n)
    dt = time.perf_counter() - t0
    triples = int(per_cand[:n].sum())
    base = {"value": triples / dt, "unit": "triples/s", "cores": 1, "kind": "oracle",
            "sample": f"candidates [0,{n}) of {w.n_cand} x all {w.n_req} requests, {triples:.3e} triples",
            "seconds": dt}
    m = min(w.n_cand, max(n, min_checked))
    if m > n:
        more = _sweep_oracle_parallel(w, n, m)
        ref = ref.copy()
        ref[n:m] = more[n:m]
    agrees = bool(np.array_equal(gpu_counts[:m], ref[:m]))
    check = {"agrees": agrees, "compared": f"sat_count of candidates [0,{m}) of {w.n_cand}",
             "candidates_compared": m, "distinct_counts": int(len(np.unique(ref[:m]))),
             "mismatches": int((gpu_counts[:m] != ref[:m]).sum())}
    return base, check


def stressed_check(w_name: str, seed: int, n_check: int):
    """The same shape with queued prefill, occupancy up to 2B and deadlines x 0.25 - a variant whose
    candidates differ, so that a wrong count cannot hide behind ratios that are all 1.0.  Untimed."""
    import numpy as np
    import torch
    from paper_2509_06362_amd import binding, workloads as W
    w = W.stressed(make_workload(w_name), seed=seed)
    dw = binding.DeviceWorkload(w)
    try:
        cnt, _, best = dw.sweep()
        torch.cuda.synchronize()
        cnt = cnt.cpu().numpy().view(np.uint32)
        status = binding.maaso_ctx_device_status(dw.ctx)
    finally:
        dw.close()
    m = min(n_check, w.n_cand)
    ref = _sweep_oracle_parallel(w, 0, m)
    return {"agrees": bool(np.array_equal(cnt[:m], ref[:m])) and status == 0,
            "compared": f"sat_count of candidates [0,{m}) of {w.n_cand}, stressed variant (untimed)",
            "candidates_compared": m, "distinct_counts": int(len(np.unique(ref[:m]))),
            "mismatches": int((cnt[:m] != ref[:m]).sum())}


def assign_cpu_leg(w, got, budget_triples: float):
    """Timed single-threaded oracle on the first n requests; chosen instance, slack and (when the
    sample is the whole stream) admitted count and final state compared with the GPU's."""
    import numpy as np
    import oracle
    I = max(1, int(w.n_inst[0]))
    n = int(min(w.n_req, max(1, budget_triples // I)))
    if w.window:
        n = min(w.n_req, max(int(w.window), (n // int(w.window)) * int(w.window)))
    ws = w.with_requests(0, n)
    t0 = time.perf_counter()
    ref = oracle.score_assign(ws, latencies=False)
    dt = time.perf_counter() - t0
    triples = n * I
    base = {"value": triples / dt, "unit": "triples/s", "cores": 1, "kind": "oracle",
            "sample": f"requests [0,{n}) of {w.n_req} x {I} instances, {triples:.3e} triples",
            "seconds": dt}
    chosen = got["chosen"][:n].cpu().numpy()
    slack = got["slack"][:n].cpu().numpy()
    same_chosen = bool(np.array_equal(chosen, ref["chosen"]))
    same_slack = bool(np.array_equal(slack, ref["slack"]))
    what = ["chosen", "slack"]
    agrees = same_chosen and same_slack
    if n == w.n_req:
        what += ["n_satisfied"]
        agrees = agrees and int(got["n_satisfied"].item()) == ref["n_satisfied"]
        if w.window:
            what += ["final occ", "final q_ticks"]
            agrees = agrees and bool(np.array_equal(got["occ"].cpu().numpy()[0], ref["occ"]))
            agrees = agrees and bool(np.array_equal(got["q_ticks"].cpu().numpy()[0].view(np.uint64),
                                                    ref["q_ticks"]))
    check = {"agrees": agrees, "compared": f"{', '.join(what)} of requests [0,{n}) of {w.n_req}",
             "requests_compared": n, "mismatches": int((chosen != ref["chosen"]).sum()),
             "admitted_in_sample": int(ref["n_satisfied"])}
    return base, check


# ------------------------------------------------------------------------------------------------
# one workload
# ------------------------------------------------------------------------------------------------

def duration_stats(durs):
    """The dominant kernel's durations in issue order: a clock that was still rising shows as a first
    launch well above the median and the last."""
    if not durs:
        return {}
    s = sorted(durs)
    return {"kernel_ms_first": durs[0], "kernel_ms_median": s[len(s) // 2], "kernel_ms_last": durs[-1],
            "kernel_ms_min": s[0], "kernel_ms_max": s[-1]}


def measure(name: str, steps: int, warmup: int, args, min_gpu_warm_ms: float = 0.0):
    """Times one workload; returns (entry, context for the oracle leg).  GPU work only."""
    import numpy as np
    import torch
    from paper_2509_06362_amd import binding
    w = make_workload(name)
    kind = "sweep" if w.n_cand > 1 else "assign"
    sweep_window = int(w.window) if kind == "sweep" else 0
    dw = binding.DeviceWorkload(w)
    binding.maaso_ctx_set_launch_shape(dw.ctx, args.sweep_q, args.sweep_group, args.sweep_bq,
                                       args.window_blocks)
    if args.plain_launch:
        binding.maaso_ctx_set_cooperative(dw.ctx, False)
    dev = dw.prompt_len.device
    stream = torch.cuda.current_stream()

    # outputs allocated once, outside the timed region
    sweep_out = (torch.empty(w.n_cand, dtype=torch.int32, device=dev),
                 torch.empty(w.n_cand, dtype=torch.float32, device=dev),
                 torch.empty(1, dtype=torch.int32, device=dev))
    assign_out = dict(chosen=torch.empty(w.n_req, dtype=torch.int32, device=dev),
                      slack=torch.empty(w.n_req, dtype=torch.float32, device=dev),
                      n_satisfied=torch.empty(1, dtype=torch.int64, device=dev))

    if kind == "sweep" and w.name.endswith("_score"):
        score_out = dict(sat_count=sweep_out[0], best_cand=sweep_out[2])
        for k in ("phi_s", "phi_t", "phi_l", "score"):
            score_out[k] = torch.empty(w.n_cand, dtype=torch.float32, device=dev)
        cw = dict(zip(("alpha", "beta", "gamma_t", "gamma_l"), SCORE_WEIGHTS))

        def run_sweep():
            binding.maaso_placement_score(
                dw.ctx, n_cand=w.n_cand, i_pad=w.i_pad, n_inst=dw.n_inst, tp_idx=dw.tp_idx,
                max_batch=dw.max_batch, occ=dw.occ, q_ticks=dw.q_ticks, **dw.request_args(),
                arrival_ticks=dw.arrival_ticks, window=sweep_window, **dw.param_args(), **cw,
                stream=stream, **score_out)
    else:
        def run_sweep():
            dw.sweep(out=sweep_out, stream=stream, window=sweep_window)

    last = {}
    if kind == "sweep":
        # the distributor runs on the winning deployment; a first sweep tells the host which one that
        # is (for the triple count only)
        run_sweep()
        torch.cuda.synchronize()
        best = int(sweep_out[2].item())
        triples_sweep = w.valid_triples()
        triples_assign = w.n_req * int(w.n_inst[best])

        def step():
            # the distributor reads the sweep's best candidate on the device: no host round trip
            run_sweep()
            last["assign"] = dw.assign_selected(sweep_out[2], window=0, latencies=False, out=assign_out,
                                                stream=stream)
        dominant = run_sweep
        step_text = (("placement_score" if w.name.endswith("_score") else "placement_sweep")
                     + " + score_assign(best candidate)")
    elif name == "cfg0":
        # the tiny check runs both entry points on its one placement
        best = 0
        triples_sweep = w.valid_triples()
        triples_assign = w.n_req * int(w.n_inst[0])

        def dominant():
            last["assign"] = dw.assign(cand=0, window=w.window, latencies=False, out=assign_out, stream=stream)

        def step():
            run_sweep()
            dominant()
        step_text = "placement_sweep (one candidate) + score_assign"
    else:
        best = 0
        triples_sweep = 0
        triples_assign = w.n_req * int(w.n_inst[0])

        def step():
            last["assign"] = dw.assign(cand=0, window=w.window, latencies=False, out=assign_out, stream=stream)
        dominant = step
        step_text = "score_assign"

    triples_step = triples_sweep + triples_assign
    n_warm = warmup
    if min_gpu_warm_ms > 0.0:
        # enough untimed work for the device's clock to have risen before a short series is timed
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        est_ms = max((time.perf_counter() - t0) * 1e3, 1e-3)
        n_warm = max(warmup, min(2000, int(math.ceil(min_gpu_warm_ms / est_ms))))
    for _ in range(n_warm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    value = triples_step * steps / dt

    # dominant kernel: event pairs recorded inside the library around that kernel only, launched back
    # to back right behind the timed steps
    binding.maaso_ctx_kernel_timing(dw.ctx, True)
    n_timed = min(steps, 100)
    for _ in range(n_timed):
        dominant()
    torch.cuda.synchronize()
    durs = binding.maaso_ctx_kernel_durations(dw.ctx)
    binding.maaso_ctx_kernel_timing(dw.ctx, False)
    k_n = len(durs)
    k_avg_s = sum(durs) / max(k_n, 1) * 1e-3
    traffic, traffic_info = measured_traffic(w.name)
    if kind == "sweep" and sweep_window:
        ops = ASSIGN_LANEOPS_PER_TRIPLE * triples_sweep
        roofline = {
            "kernel": "sweep_seq_kernel" if sweep_window == 1 else "sweep_window_kernel", "bound": "alu",
            "achieved": ops / k_avg_s / 1e12, "peak": VALU_PEAK_TLANEOPS, "unit": "Tlaneop/s",
            "frac": ops / k_avg_s / 1e12 / VALU_PEAK_TLANEOPS, "traffic": traffic,
            "kernel_ms": k_avg_s * 1e3, "launches_timed": k_n,
            "laneops_per_triple": ASSIGN_LANEOPS_PER_TRIPLE,
            "kernel_triples_per_s": triples_sweep / k_avg_s,
        }
    elif kind == "sweep":
        # pairs that reached the latency loop, and those of them on an instance without a wait
        pairs, pairs_nowait = binding.maaso_ctx_sweep_evaluated(dw.ctx, split=True)
        ops = (SWEEP_SLOTS_PER_PAIR * (pairs - pairs_nowait)
               + SWEEP_SLOTS_PER_PAIR_NO_WAIT * pairs_nowait)
        flop = (SWEEP_FLOP_PER_PAIR * (pairs - pairs_nowait)
                + SWEEP_FLOP_PER_PAIR_NO_WAIT * pairs_nowait)
        roofline = {
            "kernel": "sweep_kernel", "bound": "alu",
            "achieved": ops / k_avg_s / 1e12, "peak": VALU_PEAK_TLANEOPS, "unit": "Tlaneop/s",
            "frac": ops / k_avg_s / 1e12 / VALU_PEAK_TLANEOPS, "traffic": traffic,
            "kernel_ms": k_avg_s * 1e3, "launches_timed": k_n,
            "slots_per_pair": SWEEP_SLOTS_PER_PAIR,
            "slots_per_pair_without_wait": SWEEP_SLOTS_PER_PAIR_NO_WAIT,
            "operations_per_pair": SWEEP_OPERATIONS_PER_PAIR,
            "frac_counting_operations": SWEEP_OPERATIONS_PER_PAIR * pairs / k_avg_s / 1e12
            / VALU_PEAK_TLANEOPS,
            "pairs_evaluated": pairs, "pairs_without_wait": pairs_nowait,
            "valid_triples": triples_sweep,
            "settled_per_class_instance": triples_sweep - pairs,
            "tflops": flop / k_avg_s / 1e12,
            "frac_of_fp32_vector_peak": flop / k_avg_s / 1e12 / FP32_VECTOR_PEAK_TFLOPS,
            "kernel_triples_per_s": triples_sweep / k_avg_s,
        }
        # the metric also asks for the fraction of the HBM roofline: each request record (9 B), each
        # instance slot (15 B) and each candidate result (8 B) once per call, over the same kernel time
        alg_bytes = 9 * w.n_req + 15 * w.n_cand * w.i_pad + 8 * w.n_cand
        roofline["hbm"] = {
            "algorithmic_bytes": alg_bytes, "achieved_GBps": alg_bytes / k_avg_s / 1e9,
            "frac_of_peak": alg_bytes / k_avg_s / 1e9 / HBM_PEAK_GBS,
            "measured_frac_of_peak": None if traffic is None else traffic / k_avg_s / 1e9 / HBM_PEAK_GBS,
            "note": "the sweep moves about 1e-3 B per triple: it is bound by the VALU, not by HBM; the "
                    "60 %-of-HBM target is literal only on the streaming distributor shape",
        }
    else:
        nbytes = ASSIGN_BYTES_PER_REQUEST * w.n_req
        ops = ASSIGN_LANEOPS_PER_TRIPLE * triples_assign
        hbm_frac = nbytes / k_avg_s / 1e9 / HBM_PEAK_GBS
        alu_frac = ops / k_avg_s / 1e12 / VALU_PEAK_TLANEOPS
        kname = "assign_window_kernel" if w.window else "assign_static_kernel"
        roofline = {
            "kernel": kname, "bound": "hbm", "achieved": nbytes / k_avg_s / 1e9,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac, "traffic": traffic,
            "kernel_ms": k_avg_s * 1e3, "launches_timed": k_n, "alu_frac": alu_frac,
            "bytes_per_request": ASSIGN_BYTES_PER_REQUEST,
        }
        if w.window:
            n_win = (w.n_req + int(w.window) - 1) // int(w.window)
            roofline["note"] = ("a chain of dependent windows: neither HBM nor the VALU binds, the time "
                                "is windows x per-window latency")
            roofline["windows"] = n_win
            roofline["us_per_window"] = k_avg_s * 1e6 / n_win
            # where a window's time goes: one more call with the kernel's profiling variant (block 0
            # sums its cycles per phase); shares of its loop, scaled to the unprofiled time per window
            binding.maaso_ctx_window_profile(dw.ctx, True)
            dominant()
            ph = binding.maaso_ctx_window_phases(dw.ctx)
            binding.maaso_ctx_window_profile(dw.ctx, False)
            if ph["loop"]:
                roofline["phase_us_per_window"] = {
                    k: ph[k] / ph["loop"] * roofline["us_per_window"]
                    for k in ("stage", "score", "exchange", "update")}
        elif w.n_req < (1 << 20):
            roofline["note"] = "launch latency: a single short kernel"
    roofline["traffic_info"] = traffic_info
    roofline.update(duration_stats(durs))

    if args.copy_calibration:
        # a plain elementwise copy of known size (1 GiB read + 1 GiB written per launch), so that
        # FETCH_SIZE / WRITE_SIZE readings of the kernels above can be scaled to bytes
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    status = binding.maaso_ctx_device_status(dw.ctx)
    entry = {
        "workload": w.name, "value": value, "unit": "triples/s", "steps": steps, "warmup": n_warm,
        "ms_per_step": ms_per_step,
        "config": {"workload": w.name, "n_cand": w.n_cand, "i_pad": w.i_pad, "n_req": w.n_req,
                   "n_slo": w.n_slo, "window": int(w.window), "seed": w.seed,
                   "triples_per_step": triples_step, "padded_triples": w.padded_triples(),
                   "step": step_text},
        "roofline": roofline,
        "device_status": status,
    }
    ctx = {"w": w, "kind": kind, "name": name}
    if kind == "sweep" or name == "cfg0":
        cnt = sweep_out[0].cpu().numpy().view(np.uint32).copy()
        entry["config"]["best_cand"] = best
        entry["config"]["best_ratio"] = float(cnt[best]) / max(w.n_req, 1)
        entry["config"]["distinct_ratios"] = int(len(np.unique(cnt)))
        ctx["counts"] = cnt
    if kind == "assign":
        ctx["got"] = {k: v.clone() for k, v in last["assign"].items() if v is not None}
    dw.close()
    return entry, ctx


def oracle_leg(entry, ctx, args):
    """cpu_baseline and oracle_check of one measured workload (CPU work; the GPU's results are in ctx)."""
    w, kind, name = ctx["w"], ctx["kind"], ctx["name"]
    if kind == "sweep":
        min_checked = {"cfg4": 512, "cfg3": 4096}.get(name, w.n_cand if name in ("cfg0", "cfg1") else 0)
        base, check = sweep_cpu_leg(w, ctx["counts"], args.cpu_triples, min_checked)
        if name in ("cfg1", "cfg3") or check["distinct_counts"] == 1:
            # every candidate of these workloads serves every request: add a variant that can fail
            if name in ("cfg1", "cfg3", "cfg4"):
                check["stressed"] = stressed_check(name, seed=int(name[-1]), n_check=min_checked)
                check["agrees"] = check["agrees"] and check["stressed"]["agrees"]
    else:
        base, check = assign_cpu_leg(w, ctx["got"], args.cpu_triples)
        if name == "cfg0":   # its one-candidate sweep too
            import oracle
            ref = oracle.placement_sweep(w)["sat_count"]
            same = bool((ctx["counts"] == ref).all())
            check["compared"] += "; sat_count of the one-candidate sweep"
            check["agrees"] = check["agrees"] and same
    base["gpu_over_cpu"] = entry["value"] / base["value"]
    entry["cpu_baseline"] = base
    entry["oracle_check"] = check
    entry["oracle_agrees"] = bool(check["agrees"]) and entry["device_status"] == 0


PROBE_PATTERNS = (
    (0, "pair body without queue wait: fma, fma, min3 per request"),
    (1, "pair body with queue wait: fma, fma, add, add, min3 per request"),
    (2, "pair body without queue wait, four pairs per loop trip"),
    (3, "compare writing a lane mask + carry add"),
    (4, "fma with a scalar-register operand"),
)


def valu_probe():
    """What the chip sustains for the sweep's instruction mix (maaso_probe_valu): vector lane operations
    per second of loops that are nothing but the sweep's inner instruction sequence."""
    from paper_2509_06362_amd import binding
    out = {"peak_Tlaneops": VALU_PEAK_TLANEOPS, "patterns": []}
    for pat, text in PROBE_PATTERNS:
        rate, n = binding.maaso_probe_valu(pat, 65536)
        out["patterns"].append({"pattern": pat, "what": text, "instructions_per_trip": n,
                                "Tlaneops": rate / 1e12, "frac_of_peak": rate / 1e12 / VALU_PEAK_TLANEOPS})
    out["sustained_frac_of_peak"] = max(p["frac_of_peak"] for p in out["patterns"][:3])
    return out


ALG2_GPUS = 64
ALG2_SCORE_WEIGHTS = (4.0, 0.3, 4096.0, 2.0)


def bench_alg2(args) -> int:
    """Resource partition (Alg. 2) as one pipeline: split by SLO, every growth-chain deployment of
    Alg. 1 scored against R_t, R_l and R, best per GPU count, partition scan.  A step is the whole
    pipeline; its triples are those of the scoring launch, which carries the three request sets."""
    import numpy as np
    import torch
    from paper_2509_06362_amd import binding, workloads as W
    w = W.partition_case(n_req=131072, rate=400.0)
    tp, b = W.all_configs()
    cw, offs = W.growth_chains(w, tp, b, ALG2_GPUS)
    dw = binding.DeviceWorkload(cw)
    slots = int(cw.n_inst.astype(np.int64).sum())
    triples_step = 2 * cw.n_req * slots

    # one library call per step, working in arrays made once: nothing is allocated and nothing
    # comes back to the host inside the timed region
    work = dw.partition_work(ALG2_GPUS)
    offs_dev = torch.from_numpy(np.ascontiguousarray(offs).view(np.int32)).to(dw.prompt_len.device)

    def step():
        return dw.resource_partition(offs_dev, 0b1, ALG2_GPUS, *ALG2_SCORE_WEIGHTS, window=int(w.window),
                                     work=work)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    binding.maaso_ctx_kernel_timing(dw.ctx, True)
    n_timed = min(args.steps, 50)
    for _ in range(n_timed):
        step()
    torch.cuda.synchronize()
    k_ms, k_n = binding.maaso_ctx_kernel_elapsed(dw.ctx)
    binding.maaso_ctx_kernel_timing(dw.ctx, False)
    k_total_s = k_ms * 1e-3 / max(n_timed, 1)       # the scoring launch of one step (three request sets)
    ops = ASSIGN_LANEOPS_PER_TRIPLE * triples_step
    part = res["partition"].cpu().numpy()
    result = {
        "metric": "scored (candidate,request,instance) triples/sec",
        "value": triples_step * args.steps / dt, "unit": "triples/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "alg2_partition", "n_gpus_partitioned": ALG2_GPUS, "n_cand": cw.n_cand,
                   "i_pad": cw.i_pad, "n_req": cw.n_req, "n_chains": len(tp), "window": int(w.window),
                   "seed": w.seed, "triples_per_step": triples_step,
                   "step": "maaso_resource_partition_requests: split by SLO, one scoring launch over (R_t, R_l, R), "
                           "Alg. 1's selection per set, partition scan; |R_t| stays on the device",
                   "partition": {"g_t": int(part[0]), "g_l": int(part[1]),
                                 "heterogeneous": int(part[2]), "phi_opt": float(res["phi_opt"].item())}},
        "roofline": {"kernel": "sweep_window_kernel", "bound": "alu",
                     "achieved": ops / k_total_s / 1e12, "peak": VALU_PEAK_TLANEOPS, "unit": "Tlaneop/s",
                     "frac": ops / k_total_s / 1e12 / VALU_PEAK_TLANEOPS, "traffic": None,
                     "kernel_ms": k_ms / max(k_n, 1), "launches_timed": k_n,
                     "laneops_per_triple": ASSIGN_LANEOPS_PER_TRIPLE},
        "device_status": binding.maaso_ctx_device_status(dw.ctx),
    }
    if not args.no_cpu_baseline:
        # the oracle's sequential Alg. 1 + Alg. 2 on the first requests of the same stream; it scores
        # a chain only up to its first rejected deployment, so its triples are counted from its own run
        import oracle
        oracle.build()
        n = int(min(w.n_req, max(int(w.window), args.cpu_triples // (2 * slots))))
        ws = w.with_requests(0, n)
        t0 = time.perf_counter()
        r_t, r_l = oracle.split_by_slo(ws, 0b1)
        done = 0
        lists = {}
        for tag, wx in (("t", r_t), ("l", r_l), ("h", ws)):
            lists[tag] = oracle.ins_deploy(wx, ALG2_GPUS, tp, b, *ALG2_SCORE_WEIGHTS, window=int(w.window))
        oracle.resource_partition(ALG2_GPUS, lists["t"]["phi_star"], lists["l"]["phi_star"],
                                  lists["h"]["phi_star"], r_l.n_req, ws.n_req)
        cdt = time.perf_counter() - t0
        for tag, wx in (("t", r_t), ("l", r_l), ("h", ws)):
            cw_x, offs_x = W.growth_chains(wx, tp, b, ALG2_GPUS)
            sc = oracle.placement_score(cw_x, *ALG2_SCORE_WEIGHTS, window=int(w.window))["score"]
            for i in range(len(tp)):
                chain = sc[offs_x[i]:offs_x[i + 1]]
                prev = np.concatenate([[np.float32(0)], chain[:-1]])
                stop = np.nonzero(~(chain > prev))[0]
                m = int(stop[0]) + 1 if len(stop) else len(chain)     # deployments the greedy scored
                done += wx.n_req * (m * (m + 1) // 2)
        result["cpu_baseline"] = {
            "value": done / cdt, "unit": "triples/s", "cores": 1, "kind": "oracle",
            "sample": f"sequential Alg. 1 + Alg. 2 on requests [0,{n}) of {w.n_req}: {done:.3e} triples "
                      f"(chains cut at the first rejection) in the timed part", "seconds": cdt}
        result["cpu_baseline"]["gpu_over_cpu"] = result["value"] / result["cpu_baseline"]["value"]
    print(json.dumps(result))
    dw.close()
    return 0


def top_level(entry, args, steps, warmup):
    """An entry in the form of the one-line contract."""
    out = {
        "metric": "scored (candidate,request,instance) triples/sec; % of HBM roofline",
        "value": entry["value"], "unit": "triples/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": entry["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "value_counts": "valid (candidate, request, instance) triples SETTLED per second with inputs "
                        "resident in HBM: the sweep settles a triple whose instance fails the class's "
                        "between-token deadline per (class, instance) and evaluates first-token "
                        "latency and deadline for every other one (roofline.pairs_evaluated); it does "
                        "not compute three slacks per triple - the distributor does, on the winning "
                        "deployment",
        "config": entry["config"], "roofline": entry["roofline"],
        "device_status": entry["device_status"],
    }
    for k in ("cpu_baseline", "oracle_check", "oracle_agrees"):
        if k in entry:
            out[k] = entry[k]
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="report",
                    choices=["report", "cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "cfg4w", "cfg4w1",
                             "cfg4score", "alg2", "stream", "probe"],
                    help="report (default): config 4 as the headline and the other workloads in per_config")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-triples", type=float, default=3.0e9,
                    help="size of the oracle's timed single-threaded sample, in triples")
    ap.add_argument("--sweep-q", type=int, default=0)
    ap.add_argument("--sweep-group", type=int, default=0)
    ap.add_argument("--sweep-bq", type=int, default=0)
    ap.add_argument("--window-blocks", type=int, default=0)
    ap.add_argument("--plain-launch", action="store_true",
                    help="launch the windowed distributor's kernel as an ordinary grid, not cooperatively "
                         "(rocprofv3 crashes at exit after a cooperative launch)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB copy kernel five times (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import torch
    from paper_2509_06362_amd import binding

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    binding.load_library()
    if args.workload == "alg2":
        return bench_alg2(args)
    if args.workload == "probe":
        print(json.dumps(valu_probe()))
        return 0
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()

    if args.workload != "report":
        entry, ctx = measure(args.workload, args.steps, args.warmup, args)
        if not args.no_cpu_baseline:
            if ctx["name"] in ("cfg4w", "cfg4w1", "cfg4score"):
                base, check = sweep_cpu_leg(ctx["w"], ctx["counts"], args.cpu_triples, 0)
                base["gpu_over_cpu"] = entry["value"] / base["value"]
                entry.update(cpu_baseline=base, oracle_check=check,
                             oracle_agrees=check["agrees"] and entry["device_status"] == 0)
            else:
                oracle_leg(entry, ctx, args)
        print(json.dumps(top_level(entry, args, args.steps, args.warmup)))
        return 0

    # The report.  All GPU work first (the headline with exactly the steps and warm-up asked for, the
    # others behind it with at least 50 ms of untimed work each), then the oracle legs.
    t_start = time.perf_counter()
    head, head_ctx = measure("cfg4", args.steps, args.warmup, args)
    others = [measure(n, max(10, min(args.steps, 50)), args.warmup, args, min_gpu_warm_ms=50.0)
              for n in REPORT_OTHERS]
    t_gpu = time.perf_counter() - t_start
    if not args.no_cpu_baseline:
        oracle_leg(head, head_ctx, args)
        for entry, ctx in others:
            oracle_leg(entry, ctx, args)
    result = top_level(head, args, args.steps, args.warmup)
    result["per_config"] = [e for e, _ in others]
    if not args.no_cpu_baseline:
        result["oracle_agrees_all"] = bool(head["oracle_agrees"] and all(e["oracle_agrees"] for e, _ in others))
    stream = next(e for e, _ in others if e["config"]["workload"] == "streaming_i4")
    result["hbm_roofline"] = {
        "note": "the 60 %-of-peak-HBM target is meaningful where HBM binds: the streaming distributor "
                "shape (4 instances, 2^26 requests, 17 B per request); the sweeps move ~1e-3 B per "
                "triple and are priced against the VALU peak",
        "streaming_frac_of_hbm_peak": stream["roofline"]["frac"],
        "headline_frac_of_hbm_peak": head["roofline"]["hbm"]["frac_of_peak"],
    }
    result["valu_probe"] = valu_probe()
    result["paper_context"] = PAPER_CONTEXT
    result["seconds"] = {"gpu_part": t_gpu, "total": time.perf_counter() - t_start}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
