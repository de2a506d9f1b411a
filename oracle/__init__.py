"""ctypes front end of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Imported by the tests, by the smoke check and by the benchmark's CPU-baseline leg; never by the
product package.  `build()` compiles maaso_oracle.cpp with g++ (no contraction, no fast-math) and
`load()` returns the wrapped library.  The wrappers take a workload (plain numpy arrays) and return
numpy arrays; they do no arithmetic of their own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

from .batch_prune import batch_size_prune  # noqa: F401  (definition of the batch-size pruning)
from .profile_fit import profile_fit  # noqa: F401  (numpy oracle of the profiler's fit)

_HERE = Path(__file__).resolve().parent
SRC = _HERE / "maaso_oracle.cpp"
LIB = _HERE / "libmaaso_oracle.so"
CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
            "-Wall", "-Wextra"]


def build(force: bool = False) -> Path:
    if force or not LIB.exists() or LIB.stat().st_mtime < SRC.stat().st_mtime:
        tmp = LIB.with_suffix(f".so.tmp{os.getpid()}")
        subprocess.run(["g++", *CXXFLAGS, str(SRC), "-o", str(tmp)], check=True)
        os.replace(tmp, LIB)
    return LIB


_lib = None


def _ptr(a, ctype):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(ctype))


def load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(str(LIB))
        _lib.oracle_triple.restype = None
        for name in ("oracle_stage", "oracle_score_assign", "oracle_placement_sweep",
                     "oracle_placement_sweep_windowed", "oracle_placement_score",
                     "oracle_threshold_sweep", "oracle_ins_deploy", "oracle_resource_partition"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _profile_args(w):
    return (C.c_uint32(w.n_tp), C.c_uint32(w.b_cap), _ptr(w.prefill_a, C.c_float),
            _ptr(w.prefill_p, C.c_float), _ptr(w.tbt, C.c_float))


def _slo_args(w):
    return (C.c_uint32(w.n_slo), _ptr(w.d_ttft, C.c_float), _ptr(w.d_tbt, C.c_float))


def stage(w, cand: int = 0, tbt_mode=None):
    """Profile evaluation of candidate `cand`'s valid instances -> dict of float32 arrays."""
    lib = load()
    n = int(w.n_inst[cand])
    outs = {k: np.empty(n, np.float32) for k in ("a", "p", "tbt", "svc", "wait")}
    rc = lib.oracle_stage(
        *_profile_args(w), C.c_uint32(n), _ptr(np.ascontiguousarray(w.tp_idx[cand]), C.c_uint8),
        _ptr(np.ascontiguousarray(w.max_batch[cand]), C.c_uint16),
        _ptr(np.ascontiguousarray(w.occ[cand]), C.c_int32),
        _ptr(np.ascontiguousarray(w.q_ticks[cand]), C.c_uint64),
        C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode),
        *(_ptr(outs[k], C.c_float) for k in ("a", "p", "tbt", "svc", "wait")))
    assert rc == 0
    return outs


def triple(a, p, tbt_j, wait, prompt_len, out_len, d_ttft, d_tbt):
    """One (request, instance) evaluation -> dict(pre, ttft, e2e, s1, s2, s3, slack)."""
    lib = load()
    out = np.empty(7, np.float32)
    lib.oracle_triple(C.c_float(float(a)), C.c_float(float(p)), C.c_float(float(tbt_j)),
                      C.c_float(float(wait)), C.c_uint32(int(prompt_len)), C.c_uint32(int(out_len)),
                      C.c_float(float(d_ttft)), C.c_float(float(d_tbt)), _ptr(out, C.c_float))
    return dict(zip(("pre", "ttft", "e2e", "s1", "s2", "s3", "slack"), out))


def score_assign(w, cand: int = 0, window=None, tbt_mode=None, latencies: bool = True):
    """Distributor over candidate `cand`.  Returns a dict; `occ`/`q_ticks` are the final state."""
    lib = load()
    n_inst = int(w.n_inst[cand])
    occ = np.ascontiguousarray(w.occ[cand]).copy()
    q = np.ascontiguousarray(w.q_ticks[cand]).copy()
    R = w.n_req
    chosen = np.empty(R, np.int32)
    slack = np.empty(R, np.float32)
    lt, lb, le = (np.empty(R, np.float32) if latencies else None for _ in range(3))
    n_sat = C.c_uint64(0)
    window = w.window if window is None else window
    arr = w.arrival_ticks
    if window and arr is None:
        raise ValueError("windowed scoring needs arrival_ticks")
    rc = lib.oracle_score_assign(
        *_profile_args(w), *_slo_args(w), C.c_uint32(n_inst),
        _ptr(np.ascontiguousarray(w.tp_idx[cand]), C.c_uint8),
        _ptr(np.ascontiguousarray(w.max_batch[cand]), C.c_uint16),
        _ptr(occ, C.c_int32), _ptr(q, C.c_uint64), C.c_uint32(R),
        _ptr(w.prompt_len, C.c_uint32), _ptr(w.out_len, C.c_uint32), _ptr(w.slo_class, C.c_uint8),
        _ptr(arr, C.c_uint32), C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode), C.c_uint32(window), C.c_uint32(int(w.policy)),
        _ptr(chosen, C.c_int32), _ptr(slack, C.c_float), _ptr(lt, C.c_float), _ptr(lb, C.c_float),
        _ptr(le, C.c_float), C.byref(n_sat))
    if rc != 0:
        raise ValueError(f"oracle_score_assign rejected the profile (rc={rc})")
    return dict(chosen=chosen, slack=slack, ttft=lt, tbt=lb, e2e=le, n_satisfied=int(n_sat.value),
                occ=occ, q_ticks=q)


def placement_sweep(w, c_begin: int = 0, c_end=None, tbt_mode=None):
    """Static sweep over candidates [c_begin, c_end).  Entries outside the range are zero."""
    lib = load()
    c_end = w.n_cand if c_end is None else c_end
    cnt = np.zeros(w.n_cand, np.uint32)
    ratio = np.zeros(w.n_cand, np.float32)
    best = C.c_uint32(0)
    rc = lib.oracle_placement_sweep(
        *_profile_args(w), *_slo_args(w), C.c_uint32(w.n_cand), C.c_uint32(w.i_pad),
        _ptr(w.n_inst, C.c_uint32), _ptr(w.tp_idx, C.c_uint8), _ptr(w.max_batch, C.c_uint16),
        _ptr(w.occ, C.c_int32), _ptr(w.q_ticks, C.c_uint64), C.c_uint32(w.n_req),
        _ptr(w.prompt_len, C.c_uint32), _ptr(w.out_len, C.c_uint32), _ptr(w.slo_class, C.c_uint8),
        C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode),
        C.c_uint32(c_begin), C.c_uint32(c_end), _ptr(cnt, C.c_uint32), _ptr(ratio, C.c_float),
        C.byref(best))
    if rc != 0:
        raise ValueError(f"oracle_placement_sweep rejected its arguments (rc={rc})")
    return dict(sat_count=cnt, sat_ratio=ratio, best_cand=int(best.value))


def placement_sweep_windowed(w, window=None, c_begin: int = 0, c_end=None, tbt_mode=None):
    """Capacity-aware sweep: each candidate of [c_begin, c_end) through the windowed distributor."""
    lib = load()
    c_end = w.n_cand if c_end is None else c_end
    window = w.window if window is None else window
    if w.arrival_ticks is None:
        raise ValueError("windowed scoring needs arrival_ticks")
    cnt = np.zeros(w.n_cand, np.uint32)
    ratio = np.zeros(w.n_cand, np.float32)
    best = C.c_uint32(0)
    rc = lib.oracle_placement_sweep_windowed(
        *_profile_args(w), *_slo_args(w), C.c_uint32(w.n_cand), C.c_uint32(w.i_pad),
        _ptr(w.n_inst, C.c_uint32), _ptr(w.tp_idx, C.c_uint8), _ptr(w.max_batch, C.c_uint16),
        _ptr(w.occ, C.c_int32), _ptr(w.q_ticks, C.c_uint64), C.c_uint32(w.n_req),
        _ptr(w.prompt_len, C.c_uint32), _ptr(w.out_len, C.c_uint32), _ptr(w.slo_class, C.c_uint8),
        _ptr(w.arrival_ticks, C.c_uint32), C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode), C.c_uint32(window), C.c_uint32(int(w.policy)),
        C.c_uint32(c_begin), C.c_uint32(c_end), _ptr(cnt, C.c_uint32), _ptr(ratio, C.c_float),
        C.byref(best))
    if rc != 0:
        raise ValueError(f"oracle_placement_sweep_windowed rejected its arguments (rc={rc})")
    return dict(sat_count=cnt, sat_ratio=ratio, best_cand=int(best.value))


def placement_score(w, alpha, beta, gamma_t, gamma_l, window=0, c_begin: int = 0, c_end=None,
                    tbt_mode=None):
    """Composite serving score of candidates [c_begin, c_end) (window 0 = static)."""
    lib = load()
    c_end = w.n_cand if c_end is None else c_end
    if window and w.arrival_ticks is None:
        raise ValueError("windowed scoring needs arrival_ticks")
    cnt = np.zeros(w.n_cand, np.uint32)
    ps, pt, pl, sc = (np.zeros(w.n_cand, np.float32) for _ in range(4))
    best = C.c_uint32(0)
    rc = lib.oracle_placement_score(
        *_profile_args(w), *_slo_args(w), C.c_uint32(w.n_cand), C.c_uint32(w.i_pad),
        _ptr(w.n_inst, C.c_uint32), _ptr(w.tp_idx, C.c_uint8), _ptr(w.max_batch, C.c_uint16),
        _ptr(w.occ, C.c_int32), _ptr(w.q_ticks, C.c_uint64), C.c_uint32(w.n_req),
        _ptr(w.prompt_len, C.c_uint32), _ptr(w.out_len, C.c_uint32), _ptr(w.slo_class, C.c_uint8),
        _ptr(w.arrival_ticks, C.c_uint32), C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode), C.c_uint32(window), C.c_uint32(int(w.policy)),
        C.c_float(alpha), C.c_float(beta), C.c_float(gamma_t), C.c_float(gamma_l),
        C.c_uint32(c_begin), C.c_uint32(c_end), _ptr(cnt, C.c_uint32), _ptr(ps, C.c_float),
        _ptr(pt, C.c_float), _ptr(pl, C.c_float), _ptr(sc, C.c_float), C.byref(best))
    if rc != 0:
        raise ValueError(f"oracle_placement_score rejected its arguments (rc={rc})")
    return dict(sat_count=cnt, phi_s=ps, phi_t=pt, phi_l=pl, score=sc, best_cand=int(best.value))


def threshold_sweep(w, tbt_mode=None):
    """Counts of the static sweep by the prompt-length-threshold route (all candidates)."""
    lib = load()
    cnt = np.zeros(w.n_cand, np.uint32)
    rc = lib.oracle_threshold_sweep(
        *_profile_args(w), *_slo_args(w), C.c_uint32(w.n_cand), C.c_uint32(w.i_pad),
        _ptr(w.n_inst, C.c_uint32), _ptr(w.tp_idx, C.c_uint8), _ptr(w.max_batch, C.c_uint16),
        _ptr(w.occ, C.c_int32), _ptr(w.q_ticks, C.c_uint64), C.c_uint32(w.n_req),
        _ptr(w.prompt_len, C.c_uint32), _ptr(w.slo_class, C.c_uint8),
        C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode), _ptr(cnt, C.c_uint32))
    if rc != 0:
        raise ValueError("oracle_threshold_sweep rejected the profile")
    return cnt


def ins_deploy(w, n_gpus: int, cfg_tp, cfg_b, alpha, beta, gamma_t, gamma_l, window=0,
               max_inst: int = 256, tbt_mode=None):
    """Alg. 1 for one model over the requests of `w` (its candidates are ignored): score list and
    best deployment per GPU count, as (configuration index, instance count)."""
    lib = load()
    cfg_tp = np.ascontiguousarray(cfg_tp, np.uint8)
    cfg_b = np.ascontiguousarray(cfg_b, np.uint16)
    if window and w.arrival_ticks is None:
        raise ValueError("windowed scoring needs arrival_ticks")
    phi = np.zeros(n_gpus + 1, np.float32)
    cfg = np.zeros(n_gpus + 1, np.int32)
    cnt = np.zeros(n_gpus + 1, np.uint32)
    n_eval = C.c_uint64(0)
    deg = np.ascontiguousarray(w.tp_degree, np.uint32)
    rc = lib.oracle_ins_deploy(
        *_profile_args(w), *_slo_args(w), _ptr(deg, C.c_uint32), C.c_uint32(w.n_req),
        _ptr(w.prompt_len, C.c_uint32), _ptr(w.out_len, C.c_uint32), _ptr(w.slo_class, C.c_uint8),
        _ptr(w.arrival_ticks, C.c_uint32), C.c_float(float(w.s_bar)), C.c_float(float(w.pen_kappa)),
        C.c_uint32(w.tbt_mode if tbt_mode is None else tbt_mode), C.c_uint32(window), C.c_uint32(int(w.policy)),
        C.c_float(alpha), C.c_float(beta), C.c_float(gamma_t), C.c_float(gamma_l),
        C.c_uint32(n_gpus), C.c_uint32(len(cfg_tp)), _ptr(cfg_tp, C.c_uint8), _ptr(cfg_b, C.c_uint16),
        C.c_uint32(max_inst), _ptr(phi, C.c_float), _ptr(cfg, C.c_int32), _ptr(cnt, C.c_uint32),
        C.byref(n_eval))
    if rc != 0:
        raise ValueError(f"oracle_ins_deploy rejected its arguments (rc={rc})")
    return dict(phi_star=phi, cfg_star=cfg, cnt_star=cnt, n_evaluated=int(n_eval.value))


def resource_partition(n_gpus: int, phi_t_star, phi_l_star, phi_h_star, n_req_l: int, n_req: int):
    """Alg. 2's partition scan -> dict(g_t, g_l, heterogeneous, k_h, phi_opt)."""
    lib = load()
    pt = np.ascontiguousarray(phi_t_star, np.float32)
    pl = np.ascontiguousarray(phi_l_star, np.float32)
    ph = None if phi_h_star is None else np.ascontiguousarray(phi_h_star, np.float32)
    assert len(pt) == n_gpus + 1 and len(pl) == n_gpus + 1 and (ph is None or len(ph) == n_gpus + 1)
    out = np.zeros(4, np.uint32)
    opt = C.c_float(0.0)
    rc = lib.oracle_resource_partition(C.c_uint32(n_gpus), _ptr(pt, C.c_float), _ptr(pl, C.c_float),
                                       _ptr(ph, C.c_float), C.c_uint64(n_req_l), C.c_uint64(n_req),
                                       _ptr(out, C.c_uint32), C.byref(opt))
    if rc != 0:
        raise ValueError("oracle_resource_partition rejected its arguments")
    return dict(g_t=int(out[0]), g_l=int(out[1]), heterogeneous=int(out[2]), k_h=int(out[3]),
                phi_opt=float(np.float32(opt.value)))


def split_by_slo(w, tight_classes: int):
    """Alg. 2's first step: the requests whose class has its bit set in `tight_classes` (R_t) and the
    others (R_l), each in arrival order.  Pure selection; returns two workloads."""
    tight = ((np.uint32(tight_classes) >> w.slo_class.astype(np.uint32)) & 1).astype(bool)

    def pick(m):
        from dataclasses import replace
        return replace(w, prompt_len=np.ascontiguousarray(w.prompt_len[m]),
                       out_len=np.ascontiguousarray(w.out_len[m]),
                       slo_class=np.ascontiguousarray(w.slo_class[m]),
                       arrival_ticks=None if w.arrival_ticks is None
                       else np.ascontiguousarray(w.arrival_ticks[m]))
    return pick(tight), pick(~tight)
