"""Seeded synthetic inputs: profile tables, request streams, candidate placements.

This module only *draws inputs*.  It holds none of the method's arithmetic (no latency model,
no SLO check, no selection) and is the one piece shared by the CPU oracle's tests and the HIP
path's tests and benchmark, so that both sides read byte-identical arrays.

All randomness comes from numpy's Philox counter-based bit generator, keyed by the seed.
Transcendentals (powers, exp, log) are evaluated in float64 and rounded once to float32.

The shapes follow the paper's setting: an instance is a (parallelism strategy, inference batch
size) pair holding a live workload level (Sec. IV-B, Eq. 1); a candidate deployment is a multiset
of instances whose GPU counts fit the cluster (Sec. IV-C, constraint (c)); requests carry a decode
length and a deadline class (Sec. III-C, Sec. V-A "Workload Traces"); arrivals follow a gamma
process (Sec. V-A).  The paper's own traces and measured profiles are not public, so the profile
is a synthetic linear-prefill / linear-in-batch decode form and lengths are log-uniform or
log-normal.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace  # noqa: F401  (replace is re-exported)
from typing import Optional

import numpy as np

TICKS_PER_SECOND = 1 << 20  # time unit of arrival_ticks and q_ticks

TP_DEGREES = np.array([1, 2, 4, 8], dtype=np.uint32)


@dataclass
class Workload:
    """Plain numpy arrays, laid out exactly as the C-ABI expects them (SoA, row-major)."""

    name: str
    seed: int
    # profile tables, [T, b_cap + 1]; column 0 is never read and holds NaN
    tp_degree: np.ndarray
    b_cap: int
    prefill_a: np.ndarray
    prefill_p: np.ndarray
    tbt: np.ndarray
    # SLO classes
    d_ttft: np.ndarray
    d_tbt: np.ndarray
    # requests
    prompt_len: np.ndarray
    out_len: np.ndarray
    slo_class: np.ndarray
    arrival_ticks: Optional[np.ndarray]
    # placements, [C, i_pad]
    n_inst: np.ndarray
    tp_idx: np.ndarray
    max_batch: np.ndarray
    occ: np.ndarray
    q_ticks: np.ndarray
    # parameters
    s_bar: np.float32
    pen_kappa: np.float32 = np.float32(0.0)
    tbt_mode: int = 0
    window: int = 0
    policy: int = 0   # 0: largest slack; 1: shortest request queue among the capable instances
    notes: dict = field(default_factory=dict)

    @property
    def n_req(self) -> int:
        return int(self.prompt_len.shape[0])

    @property
    def n_cand(self) -> int:
        return int(self.n_inst.shape[0])

    @property
    def i_pad(self) -> int:
        return int(self.tp_idx.shape[1])

    @property
    def n_slo(self) -> int:
        return int(self.d_ttft.shape[0])

    @property
    def n_tp(self) -> int:
        return int(self.tp_degree.shape[0])

    def valid_triples(self) -> int:
        return self.n_req * int(self.n_inst.astype(np.int64).sum())

    def padded_triples(self) -> int:
        return self.n_req * self.n_cand * self.i_pad

    def with_candidates(self, lo: int, hi: int) -> "Workload":
        """The same workload restricted to candidates [lo, hi)."""
        return replace(
            self,
            n_inst=np.ascontiguousarray(self.n_inst[lo:hi]),
            tp_idx=np.ascontiguousarray(self.tp_idx[lo:hi]),
            max_batch=np.ascontiguousarray(self.max_batch[lo:hi]),
            occ=np.ascontiguousarray(self.occ[lo:hi]),
            q_ticks=np.ascontiguousarray(self.q_ticks[lo:hi]),
        )

    def with_requests(self, lo: int, hi: int) -> "Workload":
        """The same workload restricted to requests [lo, hi) (s_bar is kept)."""
        return replace(
            self,
            prompt_len=np.ascontiguousarray(self.prompt_len[lo:hi]),
            out_len=np.ascontiguousarray(self.out_len[lo:hi]),
            slo_class=np.ascontiguousarray(self.slo_class[lo:hi]),
            arrival_ticks=None
            if self.arrival_ticks is None
            else np.ascontiguousarray(self.arrival_ticks[lo:hi]),
        )


# --------------------------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------------------------

def rng_for(seed: int, stream: int = 0) -> np.random.Generator:
    """Counter-based generator; `stream` separates independent draws of one workload."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def profile_tables(b_cap: int, jitter_rng: Optional[np.random.Generator] = None):
    """Synthetic profile for TP in {1,2,4,8} and batch sizes 1..b_cap.

    prefill seconds = a_TP + p_TP * prompt_len with a_TP = 0.02/TP^0.8, p_TP = 4e-5/TP^0.85;
    seconds per output token = d_TP * (1 + 0.03 b) with d_TP = 0.012/TP^0.7.
    With `jitter_rng`, every entry is scaled by its own uniform factor in [0.9, 1.1].
    """
    tp = TP_DEGREES.astype(np.float64)[:, None]
    b = np.arange(b_cap + 1, dtype=np.float64)[None, :]
    a = np.broadcast_to(0.02 / tp**0.8, (4, b_cap + 1)).copy()
    p = np.broadcast_to(4e-5 / tp**0.85, (4, b_cap + 1)).copy()
    t = (0.012 / tp**0.7) * (1.0 + 0.03 * b)
    if jitter_rng is not None:
        a *= jitter_rng.uniform(0.9, 1.1, size=a.shape)
        p *= jitter_rng.uniform(0.9, 1.1, size=p.shape)
        t *= jitter_rng.uniform(0.9, 1.1, size=t.shape)
    out = []
    for m in (a, p, t):
        m32 = m.astype(np.float32)
        m32[:, 0] = np.nan  # column 0 (batch size 0) does not exist
        out.append(np.ascontiguousarray(m32))
    return out


def slo_three_classes():
    """(TTFT, TBT) deadlines (0.5 s, 50 ms), (2 s, 100 ms), (10 s, 200 ms)."""
    return (np.array([0.5, 2.0, 10.0], dtype=np.float32),
            np.array([0.05, 0.1, 0.2], dtype=np.float32))


def slo_eight_classes():
    """Geometric ladders: TTFT 0.2 .. 60 s, TBT 20 .. 300 ms."""
    k = np.arange(8, dtype=np.float64) / 7.0
    return ((0.2 * 300.0**k).astype(np.float32), (0.02 * 15.0**k).astype(np.float32))


def log_uniform_int(rng: np.random.Generator, lo: int, hi: int, n: int) -> np.ndarray:
    u = rng.random(n)
    v = np.floor(lo * ((hi + 1) / lo) ** u)
    return np.minimum(v, hi).astype(np.uint32)


def lognormal_int(rng: np.random.Generator, mu: float, sigma: float, lo: int, hi: int, n: int):
    v = np.rint(np.exp(mu + sigma * rng.standard_normal(n)))
    return np.clip(v, lo, hi).astype(np.uint32)


def poisson_arrivals(rng: np.random.Generator, rate: float, n: int) -> np.ndarray:
    t = np.cumsum(rng.exponential(1.0 / rate, size=n))
    ticks = np.floor(t * TICKS_PER_SECOND)
    assert ticks[-1] < 2**32 if n else True
    return ticks.astype(np.uint32)


def bursty_arrivals(rng: np.random.Generator, rate: float, shape: float, n: int, block: int = 256):
    """Gamma-modulated Poisson: each block of requests draws its own rate multiplier."""
    nb = (n + block - 1) // block
    m = np.maximum(rng.gamma(shape, 1.0 / shape, size=nb), 1e-3)
    gaps = rng.exponential(1.0, size=n) / (rate * np.repeat(m, block)[:n])
    ticks = np.floor(np.cumsum(gaps) * TICKS_PER_SECOND)
    ticks = np.minimum(ticks, 2**32 - 1)
    return ticks.astype(np.uint32)


def mean_out_len(out_len: np.ndarray) -> np.float32:
    return np.float32(out_len.astype(np.float64).mean()) if out_len.size else np.float32(1.0)


BATCH_SET_128 = np.array([4, 8, 16, 32, 64, 128], dtype=np.uint16)
BATCH_SET_256 = np.array([4, 8, 16, 32, 64, 128, 256], dtype=np.uint16)


def candidates_sum_to_budget(rng, n_cand: int, budget: int, i_pad: int, batch_set):
    """Each candidate: draw TP uniformly from the degrees that still fit until the GPU budget is used."""
    remaining = np.full(n_cand, budget, dtype=np.int64)
    n_inst = np.zeros(n_cand, dtype=np.uint32)
    tp_idx = np.zeros((n_cand, i_pad), dtype=np.uint8)
    max_batch = np.ones((n_cand, i_pad), dtype=np.uint16)
    for _ in range(i_pad):
        live = remaining > 0
        if not live.any():
            break
        n_fit = np.floor(np.log2(np.minimum(np.maximum(remaining, 1), 8))).astype(np.int64) + 1
        t = np.minimum((rng.random(n_cand) * n_fit).astype(np.int64), n_fit - 1)
        b = batch_set[rng.integers(0, len(batch_set), size=n_cand)]
        rows = np.nonzero(live)[0]
        cols = n_inst[rows].astype(np.int64)
        tp_idx[rows, cols] = t[rows].astype(np.uint8)
        max_batch[rows, cols] = b[rows]
        n_inst[rows] += 1
        remaining[rows] -= (1 << t[rows])
    assert (remaining == 0).all(), "i_pad too small for the budget"
    return n_inst, tp_idx, max_batch


def candidates_fixed_count(rng, n_cand: int, n_per: int, budget: int, batch_set):
    """Exactly n_per instances whose TP degrees sum to `budget`: start all at TP1, keep doubling."""
    t = np.zeros((n_cand, n_per), dtype=np.int64)  # log2(TP)
    total = np.full(n_cand, n_per, dtype=np.int64)
    assert n_per <= budget <= 8 * n_per
    for _ in range(budget - n_per + 1):
        need = total < budget
        if not need.any():
            break
        tp = 1 << t
        ok = (t < 3) & (total[:, None] + tp <= budget) & need[:, None]
        score = np.where(ok, rng.random((n_cand, n_per)), -1.0)
        pick = score.argmax(axis=1)
        rows = np.nonzero(ok.any(axis=1))[0]
        total[rows] += tp[rows, pick[rows]]
        t[rows, pick[rows]] += 1
    assert (total == budget).all()
    b = batch_set[rng.integers(0, len(batch_set), size=(n_cand, n_per))]
    return (np.full(n_cand, n_per, dtype=np.uint32), t.astype(np.uint8),
            np.ascontiguousarray(b, dtype=np.uint16))


def occupancy_below_cap(rng, max_batch, n_inst):
    """occ uniform in [0, B-1] on valid slots, 0 on padding."""
    occ = np.floor(rng.random(max_batch.shape) * max_batch).astype(np.int32)
    valid = np.arange(max_batch.shape[1])[None, :] < n_inst[:, None]
    return np.where(valid, occ, 0).astype(np.int32)


def growth_chains(w: "Workload", cfg_tp, cfg_b, n_gpus: int, max_inst: int = 256):
    """Candidate layout for Alg. 1's growth of a deployment (Sec. IV-E): for every configuration
    (strategy row, batch size), in the given order, the deployments of 1, 2, ... identical fresh
    instances (empty, nothing queued) that fit into `n_gpus` GPUs, at most `max_inst` instances.

    Returns (workload with these candidates, chain_offsets): chain i is candidates
    [chain_offsets[i], chain_offsets[i+1]) and its m-th candidate has m + 1 instances."""
    cfg_tp = np.asarray(cfg_tp, dtype=np.uint8)
    cfg_b = np.asarray(cfg_b, dtype=np.uint16)
    lens = np.minimum(n_gpus // w.tp_degree[cfg_tp].astype(np.int64), max_inst)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint32)
    n_cand = int(offsets[-1])
    i_pad = max(int(lens.max()) if len(lens) else 1, 1)
    n_inst = np.concatenate([np.arange(1, n + 1) for n in lens] + [np.zeros(0)]).astype(np.uint32)
    chain = np.repeat(np.arange(len(lens)), lens)
    tp_idx = np.ascontiguousarray(np.broadcast_to(cfg_tp[chain][:, None], (n_cand, i_pad)))
    max_batch = np.ascontiguousarray(np.broadcast_to(cfg_b[chain][:, None], (n_cand, i_pad)))
    cw = replace(w, n_inst=n_inst, tp_idx=tp_idx, max_batch=max_batch,
                 occ=np.zeros((n_cand, i_pad), dtype=np.int32),
                 q_ticks=np.zeros((n_cand, i_pad), dtype=np.uint64))
    return cw, offsets


def all_configs(batch_set=BATCH_SET_128, n_tp: int = 4):
    """Every (strategy row, batch size) pair, strategy-major: the unpruned configuration list."""
    tp = np.repeat(np.arange(n_tp, dtype=np.uint8), len(batch_set))
    b = np.tile(np.asarray(batch_set, dtype=np.uint16), n_tp)
    return tp, b


def partition_case(n_req: int = 65536, rate: float = 400.0, seed: int = 5,
                   tight_share: float = 0.5) -> "Workload":
    """Requests for the resource-partition scan (Alg. 2): a strict class (0.5 s, 50 ms) and a relaxed
    one (10 s, 200 ms) mixed `tight_share` : 1 - `tight_share`, Poisson arrivals at `rate` requests/s,
    shorter prompts and outputs than the sweep workloads so that a few dozen GPUs can keep up.
    Carries one placeholder candidate; the placer's candidates come from growth_chains()."""
    a, p, t = profile_tables(128)
    rng = rng_for(seed, 1)
    prompt = log_uniform_int(rng, 16, 2048, n_req)
    out = log_uniform_int(rng, 8, 512, n_req)
    cls = (rng.random(n_req) >= tight_share).astype(np.uint8)
    return Workload(
        name="alg2_partition", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=128,
        prefill_a=a, prefill_p=p, tbt=t,
        d_ttft=np.array([0.5, 10.0], dtype=np.float32), d_tbt=np.array([0.05, 0.2], dtype=np.float32),
        prompt_len=prompt, out_len=out, slo_class=cls,
        arrival_ticks=poisson_arrivals(rng_for(seed, 3), rate, n_req),
        n_inst=np.array([1], dtype=np.uint32), tp_idx=np.zeros((1, 1), dtype=np.uint8),
        max_batch=np.full((1, 1), 4, dtype=np.uint16), occ=np.zeros((1, 1), dtype=np.int32),
        q_ticks=np.zeros((1, 1), dtype=np.uint64), s_bar=mean_out_len(out), window=256)


def throughput_samples(seed: int, levels=(1, 2, 4, 8, 16, 32, 64, 128), repeats: int = 3,
                       noise: float = 0.02, truth=None):
    """Synthetic profiler measurements for the least-squares fit of the throughput-decay function
    (Sec. IV-B): for every strategy, `repeats` noisy throughput readings at each workload level.
    truth: [T, 3] rows (T0 tokens/s, delta, eps); default: four strategies of decreasing sensitivity.
    Returns (offsets [T+1] uint32, level [N] float32, thr [N] float32, truth [T, 3] float64)."""
    if truth is None:
        truth = np.array([[80.0, 0.16, 0.5], [130.0, 0.14, 1.5], [210.0, 0.12, 3.0], [330.0, 0.09, 6.0]])
    truth = np.asarray(truth, dtype=np.float64)
    rng = rng_for(seed, 7)
    lv = np.tile(np.repeat(np.asarray(levels, dtype=np.float64), repeats), (truth.shape[0], 1))
    clean = truth[:, :1] * (1.0 - truth[:, 1:2] * np.log(truth[:, 2:3] + lv))
    thr = clean * (1.0 + noise * rng.standard_normal(lv.shape))
    n = lv.shape[1]
    offsets = (np.arange(truth.shape[0] + 1) * n).astype(np.uint32)
    return (offsets, np.ascontiguousarray(lv.reshape(-1), dtype=np.float32),
            np.ascontiguousarray(thr.reshape(-1), dtype=np.float32), truth)


# --------------------------------------------------------------------------------------------
# the five workloads (+ one bandwidth-bound shape)
# --------------------------------------------------------------------------------------------

def _requests_loguniform(rng, n_req, n_slo):
    prompt = log_uniform_int(rng, 16, 8192, n_req)
    out = log_uniform_int(rng, 8, 8192, n_req)
    cls = rng.integers(0, n_slo, size=n_req).astype(np.uint8)
    return prompt, out, cls


def config0(n_req: int = 1024, seed: int = 0) -> Workload:
    """Tiny distributor check: one candidate, instances (TP,B) = (1,8),(2,16),(4,32),(8,64)."""
    a, p, t = profile_tables(64)
    d_ttft, d_tbt = slo_three_classes()
    prompt, out, cls = _requests_loguniform(rng_for(seed, 1), n_req, 3)
    rng = rng_for(seed, 2)
    max_batch = np.array([[8, 16, 32, 64]], dtype=np.uint16)
    n_inst = np.array([4], dtype=np.uint32)
    return Workload(
        name="cfg0_tiny_distributor", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=64,
        prefill_a=a, prefill_p=p, tbt=t, d_ttft=d_ttft, d_tbt=d_tbt,
        prompt_len=prompt, out_len=out, slo_class=cls, arrival_ticks=None,
        n_inst=n_inst, tp_idx=np.array([[0, 1, 2, 3]], dtype=np.uint8), max_batch=max_batch,
        occ=occupancy_below_cap(rng, max_batch, n_inst),
        q_ticks=np.zeros((1, 4), dtype=np.uint64), s_bar=mean_out_len(out))


def config1(n_cand: int = 4096, n_req: int = 65536, seed: int = 1) -> Workload:
    """Placer sweep: candidates whose TP degrees sum to a 32-GPU budget, padded to 32 slots."""
    a, p, t = profile_tables(128)
    d_ttft, d_tbt = slo_three_classes()
    prompt, out, cls = _requests_loguniform(rng_for(seed, 1), n_req, 3)
    rng = rng_for(seed, 2)
    n_inst, tp_idx, max_batch = candidates_sum_to_budget(rng, n_cand, 32, 32, BATCH_SET_128)
    return Workload(
        name="cfg1_placer_sweep", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=128,
        prefill_a=a, prefill_p=p, tbt=t, d_ttft=d_ttft, d_tbt=d_tbt,
        prompt_len=prompt, out_len=out, slo_class=cls, arrival_ticks=None,
        n_inst=n_inst, tp_idx=tp_idx, max_batch=max_batch,
        occ=occupancy_below_cap(rng, max_batch, n_inst),
        q_ticks=np.zeros((n_cand, 32), dtype=np.uint64), s_bar=mean_out_len(out))


def config2(n_req: int = 4_194_304, window: int = 4096, n_inst_total: int = 64,
            seed: int = 2) -> Workload:
    """Online distributor: 64 mixed instances, Poisson arrivals at 2000 req/s, windows of 4096."""
    a, p, t = profile_tables(128)
    d_ttft, d_tbt = slo_three_classes()
    prompt, out, cls = _requests_loguniform(rng_for(seed, 1), n_req, 3)
    rng = rng_for(seed, 2)
    tp_idx = rng.integers(0, 4, size=(1, n_inst_total)).astype(np.uint8)
    max_batch = BATCH_SET_128[rng.integers(0, 6, size=(1, n_inst_total))].astype(np.uint16)
    arrivals = poisson_arrivals(rng_for(seed, 3), 2000.0, n_req)
    return Workload(
        name="cfg2_online_distributor", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=128,
        prefill_a=a, prefill_p=p, tbt=t, d_ttft=d_ttft, d_tbt=d_tbt,
        prompt_len=prompt, out_len=out, slo_class=cls, arrival_ticks=arrivals,
        n_inst=np.array([n_inst_total], dtype=np.uint32), tp_idx=tp_idx, max_batch=max_batch,
        occ=np.zeros((1, n_inst_total), dtype=np.int32),
        q_ticks=np.zeros((1, n_inst_total), dtype=np.uint64),
        s_bar=mean_out_len(out), window=window)


def config3(n_cand: int = 65536, n_req: int = 16384, seed: int = 3) -> Workload:
    """Large sweep: exactly 32 instances per candidate over a 64-GPU budget, jittered tables."""
    a, p, t = profile_tables(128, jitter_rng=rng_for(seed, 0))
    d_ttft, d_tbt = slo_three_classes()
    prompt, out, cls = _requests_loguniform(rng_for(seed, 1), n_req, 3)
    rng = rng_for(seed, 2)
    n_inst, tp_idx, max_batch = candidates_fixed_count(rng, n_cand, 32, 64, BATCH_SET_128)
    return Workload(
        name="cfg3_large_sweep", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=128,
        prefill_a=a, prefill_p=p, tbt=t, d_ttft=d_ttft, d_tbt=d_tbt,
        prompt_len=prompt, out_len=out, slo_class=cls, arrival_ticks=None,
        n_inst=n_inst, tp_idx=tp_idx, max_batch=max_batch,
        occ=occupancy_below_cap(rng, max_batch, n_inst),
        q_ticks=np.zeros((n_cand, 32), dtype=np.uint64), s_bar=mean_out_len(out))


def config4(n_cand: int = 8192, n_req: int = 131072, n_per: int = 128, seed: int = 4) -> Workload:
    """Skewed stress: log-normal lengths, 8 SLO classes, 128 instances, occupancy penalty 0.5."""
    a, p, t = profile_tables(256)
    d_ttft, d_tbt = slo_eight_classes()
    rng = rng_for(seed, 1)
    prompt = lognormal_int(rng, 6.0, 1.5, 1, 32768, n_req)
    out = lognormal_int(rng, 6.0, 1.5, 1, 32768, n_req)
    cls = rng.integers(0, 8, size=n_req).astype(np.uint8)
    rng = rng_for(seed, 2)
    tp_idx = rng.integers(0, 4, size=(n_cand, n_per)).astype(np.uint8)
    max_batch = BATCH_SET_256[rng.integers(0, 7, size=(n_cand, n_per))].astype(np.uint16)
    # occupancy up to 5B/4: about a fifth of the instances sit past their batch cap
    occ = np.floor(rng.random((n_cand, n_per)) * (max_batch.astype(np.int64) * 5 // 4 + 1))
    q_ticks = rng.integers(0, 1 << 19, size=(n_cand, n_per), dtype=np.uint64)
    arrivals = bursty_arrivals(rng_for(seed, 3), 5000.0, 0.3, n_req)
    return Workload(
        name="cfg4_skewed_stress", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=256,
        prefill_a=a, prefill_p=p, tbt=t, d_ttft=d_ttft, d_tbt=d_tbt,
        prompt_len=prompt, out_len=out, slo_class=cls, arrival_ticks=arrivals,
        n_inst=np.full(n_cand, n_per, dtype=np.uint32), tp_idx=tp_idx, max_batch=max_batch,
        occ=occ.astype(np.int32), q_ticks=q_ticks,
        s_bar=mean_out_len(out), pen_kappa=np.float32(0.5))


def streaming_shape(n_req: int = 1 << 26, seed: int = 5) -> Workload:
    """Bandwidth-bound shape: config 0's four instances against a long request stream."""
    w = config0(n_req=n_req, seed=seed)
    return replace(w, name="streaming_i4")


def random_small(seed: int, n_cand: int, i_pad: int, n_req: int, n_slo: int = 3,
                 b_cap: int = 32, over_cap: bool = True, queued: bool = True,
                 pen_kappa: float = 0.0, jitter: bool = True) -> Workload:
    """Small irregular workload for edge-case tests: ragged n_inst (zero included), queues, overflow."""
    a, p, t = profile_tables(b_cap, jitter_rng=rng_for(seed, 0) if jitter else None)
    rng = rng_for(seed, 1)
    if n_slo == 3:
        d_ttft, d_tbt = slo_three_classes()
    else:
        d_ttft = np.sort(rng.uniform(0.2, 20.0, size=n_slo)).astype(np.float32)
        d_tbt = np.sort(rng.uniform(0.02, 0.3, size=n_slo)).astype(np.float32)
    prompt = log_uniform_int(rng, 1, 16384, n_req)
    out = log_uniform_int(rng, 1, 8192, n_req)
    cls = rng.integers(0, n_slo, size=n_req).astype(np.uint8)
    rng = rng_for(seed, 2)
    n_inst = rng.integers(0, i_pad + 1, size=n_cand).astype(np.uint32)
    tp_idx = rng.integers(0, 4, size=(n_cand, i_pad)).astype(np.uint8)
    max_batch = rng.integers(1, b_cap + 1, size=(n_cand, i_pad)).astype(np.uint16)
    hi = max_batch.astype(np.int64) * (2 if over_cap else 1)
    occ = np.floor(rng.random((n_cand, i_pad)) * hi).astype(np.int32)
    if queued:
        q_ticks = rng.integers(0, 1 << 22, size=(n_cand, i_pad), dtype=np.uint64)
        big = rng.random((n_cand, i_pad)) < 0.05  # a few queues beyond 2^24 ticks (16 s)
        q_ticks = np.where(big, q_ticks * np.uint64(37) + np.uint64((1 << 24) + 1), q_ticks)
    else:
        q_ticks = np.zeros((n_cand, i_pad), dtype=np.uint64)
    arrivals = poisson_arrivals(rng_for(seed, 3), 500.0, n_req) if n_req else np.zeros(0, np.uint32)
    return Workload(
        name=f"random_small_{seed}", seed=seed, tp_degree=TP_DEGREES.copy(), b_cap=b_cap,
        prefill_a=a, prefill_p=p, tbt=t, d_ttft=d_ttft, d_tbt=d_tbt,
        prompt_len=prompt, out_len=out, slo_class=cls, arrival_ticks=arrivals,
        n_inst=n_inst, tp_idx=tp_idx, max_batch=max_batch, occ=occ,
        q_ticks=np.ascontiguousarray(q_ticks, dtype=np.uint64),
        s_bar=mean_out_len(out), pen_kappa=np.float32(pen_kappa))


CONFIGS = {0: config0, 1: config1, 2: config2, 3: config3, 4: config4}


def stressed(w: Workload, seed: int = 99, deadline_scale: float = 0.25) -> Workload:
    """A harder variant of a workload with the same shapes: queued prefill work of up to a few
    seconds, occupancy of up to twice the batch cap, tighter deadlines.  Satisfaction then varies
    from candidate to candidate, which the plain placer workloads (every request servable) do not
    offer to a parity test."""
    rng = rng_for(seed, 7)
    shape = w.occ.shape
    q = np.floor(2.0 ** rng.uniform(14.0, 23.0, size=shape)).astype(np.uint64)
    q = np.where(rng.random(shape) < 0.05, np.uint64(0), q)
    occ = np.floor(rng.random(shape) * w.max_batch.astype(np.int64) * 2).astype(np.int32)
    return replace(
        w, name=w.name + "_stressed", occ=occ, q_ticks=np.ascontiguousarray(q, dtype=np.uint64),
        d_ttft=(w.d_ttft.astype(np.float64) * deadline_scale).astype(np.float32),
        d_tbt=(w.d_tbt.astype(np.float64) * deadline_scale).astype(np.float32))
