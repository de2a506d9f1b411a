"""Thin ctypes binding of libmaaso (include/maaso.h).  Argument marshalling only.

Functions carry the names of the C entry points.  Device buffers are torch tensors (PyTorch is used
for device memory and streams, nothing else); every step of the scoring path runs in the library's
HIP kernels.  There is no fallback: if the shared library has not been built, or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional

import numpy as np

LIB_PATH = Path(__file__).resolve().parent / "libmaaso.so"

MAASO_MAX_INSTANCES = 256
MAASO_MAX_SLO = 16
MAASO_MAX_TABLE_CELLS = 2048
MAASO_NOALLOC_SCRATCH_BYTES = 8 << 20

EXPORTS = (
    "maaso_profile_tables_load", "maaso_ctx_destroy", "maaso_ctx_device_status", "maaso_strerror",
    "maaso_ctx_set_launch_shape", "maaso_ctx_set_wait_limit", "maaso_ctx_kernel_timing",
    "maaso_ctx_kernel_elapsed", "maaso_ctx_sweep_evaluated", "maaso_score_assign",
    "maaso_placement_sweep", "maaso_placement_score", "maaso_split_by_slo",
    "maaso_ins_deploy_select", "maaso_resource_partition", "maaso_profile_fit",
    "maaso_score_assign_selected", "maaso_placement_score_sets", "maaso_placement_sweep_noalloc",
    "maaso_ctx_reserve", "maaso_ctx_workspace", "maaso_ctx_kernel_durations",
    "maaso_ctx_window_profile", "maaso_ctx_window_phases", "maaso_probe_valu",
    "maaso_ctx_set_cooperative", "maaso_resource_partition_requests", "maaso_batch_size_prune",
)


class MaasoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class ProfileDesc(C.Structure):
    _fields_ = [("n_tp", C.c_uint32), ("b_cap", C.c_uint32), ("tp_degree", C.c_void_p),
                ("prefill_a", C.c_void_p), ("prefill_p", C.c_void_p), ("tbt", C.c_void_p),
                ("n_slo", C.c_uint32), ("d_ttft", C.c_void_p), ("d_tbt", C.c_void_p)]


class Requests(C.Structure):
    _fields_ = [("n_req", C.c_uint32), ("prompt_len", C.c_void_p), ("out_len", C.c_void_p),
                ("slo_class", C.c_void_p), ("arrival_ticks", C.c_void_p)]


class Placements(C.Structure):
    _fields_ = [("n_cand", C.c_uint32), ("i_pad", C.c_uint32), ("n_inst", C.c_void_p),
                ("tp_idx", C.c_void_p), ("max_batch", C.c_void_p), ("occ", C.c_void_p),
                ("q_ticks", C.c_void_p)]


class Params(C.Structure):
    _fields_ = [("s_bar", C.c_float), ("pen_kappa", C.c_float), ("tbt_mode", C.c_uint32),
                ("window", C.c_uint32), ("policy", C.c_uint32)]


class AssignOut(C.Structure):
    _fields_ = [("chosen", C.c_void_p), ("slack", C.c_void_p), ("ttft", C.c_void_p),
                ("tbt", C.c_void_p), ("e2e", C.c_void_p), ("n_satisfied", C.c_void_p)]


class ScoreWeights(C.Structure):
    _fields_ = [("alpha", C.c_float), ("beta", C.c_float), ("gamma_t", C.c_float),
                ("gamma_l", C.c_float)]


class ScoreOut(C.Structure):
    _fields_ = [("sat_count", C.c_void_p), ("phi_s", C.c_void_p), ("phi_t", C.c_void_p),
                ("phi_l", C.c_void_p), ("score", C.c_void_p), ("best_cand", C.c_void_p)]


# field name -> element type name of maaso_partition_work, in declaration order
PARTITION_WORK_FIELDS = (
    ("prompt_len_split", "int32"), ("out_len_split", "int32"), ("slo_class_split", "uint8"),
    ("arrival_ticks_split", "int32"), ("n_tight", "int32"), ("sat_t", "int32"), ("sat_l", "int32"),
    ("sat_h", "int32"), ("score_t", "float32"), ("score_l", "float32"), ("score_h", "float32"),
    ("phi_t_star", "float32"), ("phi_l_star", "float32"), ("phi_h_star", "float32"),
    ("cand_t_star", "int32"), ("cand_l_star", "int32"), ("cand_h_star", "int32"),
    ("partition", "int32"), ("phi_opt", "float32"),
)


class PartitionWork(C.Structure):
    _fields_ = [(name, C.c_void_p) for name, _ in PARTITION_WORK_FIELDS]


_lib = None


def load_library() -> C.CDLL:
    """Loads libmaaso.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2509_06362_amd.build); "
                "there is no fallback path")
        lib = C.CDLL(str(LIB_PATH))
        lib.maaso_strerror.restype = C.c_char_p
        lib.maaso_strerror.argtypes = [C.c_int]
        lib.maaso_profile_tables_load.argtypes = [C.POINTER(ProfileDesc), C.c_int,
                                                  C.POINTER(C.c_void_p)]
        lib.maaso_ctx_destroy.argtypes = [C.c_void_p]
        lib.maaso_ctx_destroy.restype = None
        lib.maaso_ctx_device_status.argtypes = [C.c_void_p, C.POINTER(C.c_uint32)]
        lib.maaso_ctx_set_launch_shape.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32,
                                                   C.c_uint32]
        lib.maaso_ctx_set_wait_limit.argtypes = [C.c_void_p, C.c_uint32]
        lib.maaso_ctx_set_cooperative.argtypes = [C.c_void_p, C.c_int]
        lib.maaso_ctx_reserve.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32]
        lib.maaso_ctx_workspace.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)]
        lib.maaso_ctx_kernel_timing.argtypes = [C.c_void_p, C.c_int]
        lib.maaso_ctx_kernel_elapsed.argtypes = [C.c_void_p, C.POINTER(C.c_float),
                                                 C.POINTER(C.c_uint32)]
        lib.maaso_ctx_kernel_durations.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_uint32,
                                                   C.POINTER(C.c_uint32)]
        lib.maaso_ctx_window_profile.argtypes = [C.c_void_p, C.c_int]
        lib.maaso_ctx_window_phases.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
        lib.maaso_probe_valu.argtypes = [C.c_int, C.c_uint32, C.c_uint32, C.POINTER(C.c_double),
                                         C.POINTER(C.c_uint32)]
        lib.maaso_ctx_sweep_evaluated.argtypes = [C.c_void_p, C.POINTER(C.c_uint64),
                                                  C.POINTER(C.c_uint64)]
        lib.maaso_score_assign.argtypes = [C.c_void_p, C.POINTER(Placements), C.POINTER(Requests),
                                           C.POINTER(Params), C.POINTER(AssignOut), C.c_void_p]
        lib.maaso_score_assign_selected.argtypes = [C.c_void_p, C.POINTER(Placements), C.c_void_p,
                                                    C.POINTER(Requests), C.POINTER(Params),
                                                    C.POINTER(AssignOut), C.c_void_p]
        lib.maaso_placement_sweep.argtypes = [C.c_void_p, C.POINTER(Placements), C.POINTER(Requests),
                                              C.POINTER(Params), C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p]
        lib.maaso_placement_sweep_noalloc.argtypes = lib.maaso_placement_sweep.argtypes
        lib.maaso_placement_score.argtypes = [C.c_void_p, C.POINTER(Placements), C.POINTER(Requests),
                                              C.POINTER(Params), C.POINTER(ScoreWeights),
                                              C.POINTER(ScoreOut), C.c_void_p]
        lib.maaso_placement_score_sets.argtypes = [C.c_void_p, C.POINTER(Placements), C.c_uint32,
                                                   C.POINTER(Requests), C.POINTER(Params),
                                                   C.POINTER(ScoreWeights), C.POINTER(ScoreOut),
                                                   C.c_void_p]
        lib.maaso_profile_fit.argtypes = [C.c_int, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_uint32, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        lib.maaso_split_by_slo.argtypes = [C.c_void_p, C.POINTER(Requests), C.c_uint32] + [C.c_void_p] * 6
        lib.maaso_ins_deploy_select.argtypes = [C.c_void_p, C.POINTER(Placements), C.c_void_p,
                                                C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p,
                                                C.c_void_p, C.c_void_p]
        lib.maaso_resource_partition.argtypes = [C.c_void_p, C.c_uint32] + [C.c_void_p] * 6 + [
            C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.maaso_resource_partition_requests.argtypes = [
            C.c_void_p, C.POINTER(Placements), C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(Requests),
            C.c_uint32, C.POINTER(Params), C.POINTER(ScoreWeights), C.POINTER(PartitionWork), C.c_void_p]
        lib.maaso_batch_size_prune.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        missing = [n for n in EXPORTS if n != "maaso_strerror" and getattr(lib, n).argtypes is None]
        if missing:  # an undeclared signature would pass pointers as C ints
            raise RuntimeError(f"binding.py declares no argument types for {missing}")
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load_library().maaso_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise MaasoError(status, where)


def _host(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _dptr(t, dtype=None) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device buffers must be contiguous GPU tensors"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


class Context:
    """Owns a maaso_ctx*."""

    def __init__(self, handle: int, device: int, n_slo: int):
        self.handle, self.device, self.n_slo = handle, device, n_slo

    def close(self) -> None:
        if self.handle:
            load_library().maaso_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def maaso_profile_tables_load(n_tp, b_cap, prefill_a, prefill_p, tbt, d_ttft, d_tbt,
                              tp_degree=None, device: int = 0) -> Context:
    """Host numpy tables -> context on `device`."""
    lib = load_library()
    keep = [_host(prefill_a, np.float32), _host(prefill_p, np.float32), _host(tbt, np.float32),
            _host(d_ttft, np.float32), _host(d_tbt, np.float32)]
    deg = None if tp_degree is None else _host(tp_degree, np.uint32)
    desc = ProfileDesc(int(n_tp), int(b_cap), None if deg is None else deg.ctypes.data,
                       keep[0].ctypes.data, keep[1].ctypes.data, keep[2].ctypes.data,
                       int(keep[3].shape[0]), keep[3].ctypes.data, keep[4].ctypes.data)
    out = C.c_void_p()
    _check(lib.maaso_profile_tables_load(C.byref(desc), int(device), C.byref(out)),
           "maaso_profile_tables_load")
    return Context(out.value, int(device), int(keep[3].shape[0]))


def maaso_ctx_device_status(ctx: Context) -> int:
    """Synchronises; returns and clears the MAASO_DEV_* bits.  Raises on a wait timeout."""
    bits = C.c_uint32(0)
    rc = load_library().maaso_ctx_device_status(ctx.handle, C.byref(bits))
    if rc == -6:
        raise MaasoError(rc, "maaso_ctx_device_status")
    if rc not in (0, -1):
        raise MaasoError(rc, "maaso_ctx_device_status")
    return int(bits.value)


def maaso_ctx_set_launch_shape(ctx: Context, sweep_requests_per_lane=0, sweep_group=0,
                               sweep_blocks_per_queue=0, window_blocks=0) -> None:
    _check(load_library().maaso_ctx_set_launch_shape(ctx.handle, sweep_requests_per_lane,
                                                     sweep_group, sweep_blocks_per_queue,
                                                     window_blocks),
           "maaso_ctx_set_launch_shape")


def maaso_ctx_set_cooperative(ctx: Context, enable: bool) -> None:
    _check(load_library().maaso_ctx_set_cooperative(ctx.handle, int(bool(enable))), "maaso_ctx_set_cooperative")


def maaso_ctx_set_wait_limit(ctx: Context, polls: int) -> None:
    _check(load_library().maaso_ctx_set_wait_limit(ctx.handle, polls), "maaso_ctx_set_wait_limit")


def maaso_ctx_reserve(ctx: Context, max_cand: int, i_pad: int, max_req: int) -> None:
    _check(load_library().maaso_ctx_reserve(ctx.handle, int(max_cand), int(i_pad), int(max_req)),
           "maaso_ctx_reserve")


def maaso_ctx_workspace(ctx: Context):
    """(bytes of workspace held, times it has been allocated)."""
    b, n = C.c_uint64(0), C.c_uint32(0)
    _check(load_library().maaso_ctx_workspace(ctx.handle, C.byref(b), C.byref(n)), "maaso_ctx_workspace")
    return int(b.value), int(n.value)


def maaso_ctx_kernel_timing(ctx: Context, enable: bool) -> None:
    _check(load_library().maaso_ctx_kernel_timing(ctx.handle, int(bool(enable))),
           "maaso_ctx_kernel_timing")


def maaso_ctx_kernel_elapsed(ctx: Context):
    """(sum of dominant-kernel durations in ms, number of launches) since the last call."""
    ms, n = C.c_float(0), C.c_uint32(0)
    _check(load_library().maaso_ctx_kernel_elapsed(ctx.handle, C.byref(ms), C.byref(n)),
           "maaso_ctx_kernel_elapsed")
    return float(ms.value), int(n.value)


def maaso_ctx_kernel_durations(ctx: Context, cap: int = 256):
    """Durations (ms) of the dominant kernel of each timed call since the last read, in issue order."""
    buf = (C.c_float * cap)()
    n = C.c_uint32(0)
    _check(load_library().maaso_ctx_kernel_durations(ctx.handle, buf, cap, C.byref(n)),
           "maaso_ctx_kernel_durations")
    return [float(buf[i]) for i in range(n.value)]


def maaso_ctx_window_profile(ctx: Context, enable: bool) -> None:
    _check(load_library().maaso_ctx_window_profile(ctx.handle, int(bool(enable))), "maaso_ctx_window_profile")


def maaso_ctx_window_phases(ctx: Context):
    """Cycles block 0 of the last profiled windowed call spent on (stage, score, exchange, update),
    the whole loop, and the number of windows."""
    buf = (C.c_uint64 * 6)()
    _check(load_library().maaso_ctx_window_phases(ctx.handle, buf), "maaso_ctx_window_phases")
    v = [int(x) for x in buf]
    return dict(stage=v[0], score=v[1], exchange=v[2], update=v[3], loop=v[4], windows=v[5])


def maaso_probe_valu(pattern: int, trips: int = 65536, device: int = 0):
    """(vector lane operations per second, vector instructions per loop trip) of a probe pattern."""
    rate, n = C.c_double(0.0), C.c_uint32(0)
    _check(load_library().maaso_probe_valu(int(device), int(pattern), int(trips), C.byref(rate), C.byref(n)),
           "maaso_probe_valu")
    return float(rate.value), int(n.value)


def maaso_ctx_sweep_evaluated(ctx: Context, split: bool = False):
    """(request, instance) pairs the last sweep evaluated in its latency loop (synchronises); with
    `split` also how many of them belong to an instance without a queue wait."""
    v, z = C.c_uint64(0), C.c_uint64(0)
    _check(load_library().maaso_ctx_sweep_evaluated(ctx.handle, C.byref(v), C.byref(z)),
           "maaso_ctx_sweep_evaluated")
    return (int(v.value), int(z.value)) if split else int(v.value)


def _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks) -> Requests:
    import torch
    return Requests(int(n_req), _dptr(prompt_len, torch.int32), _dptr(out_len, torch.int32),
                    _dptr(slo_class, torch.uint8), _dptr(arrival_ticks, torch.int32))


def _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks) -> Placements:
    import torch
    return Placements(int(n_cand), int(i_pad), _dptr(n_inst, torch.int32), _dptr(tp_idx, torch.uint8),
                      _dptr(max_batch, torch.int16), _dptr(occ, torch.int32),
                      _dptr(q_ticks, torch.int64))


def maaso_score_assign(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks,
                       n_req, prompt_len, out_len, slo_class, arrival_ticks=None,
                       s_bar, pen_kappa=0.0, tbt_mode=0, window=0, policy=0,
                       chosen=None, slack=None, ttft=None, tbt=None, e2e=None, n_satisfied=None,
                       stream=None) -> None:
    """All array arguments are GPU torch tensors holding the C types' bit patterns
    (uint32 as int32, uint16 as int16, uint64 as int64)."""
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    out = AssignOut(_dptr(chosen, torch.int32), _dptr(slack, torch.float32),
                    _dptr(ttft, torch.float32), _dptr(tbt, torch.float32),
                    _dptr(e2e, torch.float32), _dptr(n_satisfied, torch.int64))
    _check(load_library().maaso_score_assign(ctx.handle, C.byref(pl), C.byref(rq), C.byref(prm),
                                             C.byref(out), _stream_handle(stream)),
           "maaso_score_assign")


def maaso_score_assign_selected(ctx: Context, *, cand, n_cand, i_pad, n_inst, tp_idx, max_batch, occ,
                                q_ticks, n_req, prompt_len, out_len, slo_class, arrival_ticks=None,
                                s_bar, pen_kappa=0.0, tbt_mode=0, window=0, policy=0,
                                chosen=None, slack=None, ttft=None, tbt=None, e2e=None,
                                n_satisfied=None, stream=None) -> None:
    """maaso_score_assign on the row whose index is the device word `cand` (an int32 tensor)."""
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    out = AssignOut(_dptr(chosen, torch.int32), _dptr(slack, torch.float32),
                    _dptr(ttft, torch.float32), _dptr(tbt, torch.float32),
                    _dptr(e2e, torch.float32), _dptr(n_satisfied, torch.int64))
    _check(load_library().maaso_score_assign_selected(
        ctx.handle, C.byref(pl), _dptr(cand, torch.int32), C.byref(rq), C.byref(prm), C.byref(out),
        _stream_handle(stream)), "maaso_score_assign_selected")


def maaso_placement_sweep(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks,
                          n_req, prompt_len, out_len, slo_class, arrival_ticks=None, s_bar,
                          pen_kappa=0.0, tbt_mode=0, window=0, policy=0, sat_count, sat_ratio=None,
                          best_cand=None, stream=None) -> None:
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    _check(load_library().maaso_placement_sweep(
        ctx.handle, C.byref(pl), C.byref(rq), C.byref(prm), _dptr(sat_count, torch.int32),
        _dptr(sat_ratio, torch.float32), _dptr(best_cand, torch.int32), _stream_handle(stream)),
        "maaso_placement_sweep")


def maaso_placement_sweep_noalloc(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks,
                                  n_req, prompt_len, out_len, slo_class, arrival_ticks=None, s_bar,
                                  pen_kappa=0.0, tbt_mode=0, window=0, policy=0, sat_count,
                                  sat_ratio=None, best_cand=None, stream=None) -> None:
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    _check(load_library().maaso_placement_sweep_noalloc(
        ctx.handle, C.byref(pl), C.byref(rq), C.byref(prm), _dptr(sat_count, torch.int32),
        _dptr(sat_ratio, torch.float32), _dptr(best_cand, torch.int32), _stream_handle(stream)),
        "maaso_placement_sweep_noalloc")


def maaso_placement_score(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks,
                          n_req, prompt_len, out_len, slo_class, arrival_ticks=None, s_bar,
                          pen_kappa=0.0, tbt_mode=0, window=0, policy=0, alpha, beta, gamma_t, gamma_l,
                          sat_count, score, phi_s=None, phi_t=None, phi_l=None, best_cand=None,
                          stream=None) -> None:
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    wts = ScoreWeights(float(alpha), float(beta), float(gamma_t), float(gamma_l))
    out = ScoreOut(_dptr(sat_count, torch.int32), _dptr(phi_s, torch.float32),
                   _dptr(phi_t, torch.float32), _dptr(phi_l, torch.float32),
                   _dptr(score, torch.float32), _dptr(best_cand, torch.int32))
    _check(load_library().maaso_placement_score(ctx.handle, C.byref(pl), C.byref(rq), C.byref(prm),
                                                C.byref(wts), C.byref(out), _stream_handle(stream)),
           "maaso_placement_score")


def maaso_placement_score_sets(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks,
                               sets, s_bar, pen_kappa=0.0, tbt_mode=0, window=0, policy=0, alpha, beta,
                               gamma_t, gamma_l, stream=None) -> None:
    """`sets`: one dict per request set with the request keywords (n_req, prompt_len, out_len,
    slo_class, arrival_ticks) and the output keywords (sat_count, score, phi_s, phi_t, phi_l,
    best_cand) of maaso_placement_score."""
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    wts = ScoreWeights(float(alpha), float(beta), float(gamma_t), float(gamma_l))
    n = len(sets)
    rqs = (Requests * max(n, 1))()
    outs = (ScoreOut * max(n, 1))()
    for k, d in enumerate(sets):
        rqs[k] = _requests(d["n_req"], d["prompt_len"], d["out_len"], d["slo_class"],
                           d.get("arrival_ticks"))
        outs[k] = ScoreOut(_dptr(d["sat_count"], torch.int32), _dptr(d.get("phi_s"), torch.float32),
                           _dptr(d.get("phi_t"), torch.float32), _dptr(d.get("phi_l"), torch.float32),
                           _dptr(d["score"], torch.float32), _dptr(d.get("best_cand"), torch.int32))
    _check(load_library().maaso_placement_score_sets(
        ctx.handle, C.byref(pl), n, rqs, C.byref(prm), C.byref(wts), outs, _stream_handle(stream)),
        "maaso_placement_score_sets")


def maaso_profile_fit(offsets, level, thr, b_cap: int, eps_lo: float = 2.0 ** -10,
                      eps_hi: float = 2.0 ** 10, device: int = 0):
    """Host numpy samples -> (params [T, 4] float64: T0, delta, eps, sse; tbt [T, b_cap + 1] float32).
    Raises MaasoError; on MAASO_E_TABLE the partial outputs are attached to the exception."""
    off = _host(offsets, np.uint32)
    lv, th = _host(level, np.float32), _host(thr, np.float32)
    n_tp = off.shape[0] - 1
    params = np.full((n_tp, 4), np.nan, np.float64)
    tbt = np.full((n_tp, b_cap + 1), np.nan, np.float32)
    rc = load_library().maaso_profile_fit(int(device), n_tp, off.ctypes.data, lv.ctypes.data,
                                          th.ctypes.data, int(b_cap), float(eps_lo), float(eps_hi),
                                          params.ctypes.data, tbt.ctypes.data)
    if rc != 0:
        err = MaasoError(rc, "maaso_profile_fit")
        err.partial = (params, tbt)
        raise err
    return params, tbt


def maaso_split_by_slo(ctx: Context, *, n_req, prompt_len, out_len, slo_class, arrival_ticks=None,
                       tight_classes, prompt_len_out, out_len_out, slo_class_out,
                       arrival_ticks_out=None, n_tight, stream=None) -> None:
    import torch
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    _check(load_library().maaso_split_by_slo(
        ctx.handle, C.byref(rq), int(tight_classes), _dptr(prompt_len_out, torch.int32),
        _dptr(out_len_out, torch.int32), _dptr(slo_class_out, torch.uint8),
        _dptr(arrival_ticks_out, torch.int32), _dptr(n_tight, torch.int32), _stream_handle(stream)),
        "maaso_split_by_slo")


def maaso_ins_deploy_select(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, score, chain_offsets=None,
                            n_gpus, phi_star, cand_star, stream=None) -> None:
    import torch
    pl = Placements(int(n_cand), int(i_pad), _dptr(n_inst, torch.int32), _dptr(tp_idx, torch.uint8),
                    None, None, None)
    n_chains = 0 if chain_offsets is None else int(chain_offsets.numel()) - 1
    _check(load_library().maaso_ins_deploy_select(
        ctx.handle, C.byref(pl), _dptr(score, torch.float32), _dptr(chain_offsets, torch.int32),
        n_chains, int(n_gpus), _dptr(phi_star, torch.float32), _dptr(cand_star, torch.int32),
        _stream_handle(stream)), "maaso_ins_deploy_select")


def maaso_resource_partition(ctx: Context, *, n_gpus, phi_t_star, phi_l_star, phi_h_star=None,
                             cand_t_star=None, cand_l_star=None, cand_h_star=None, n_req_l, n_req,
                             partition, phi_opt, stream=None) -> None:
    import torch
    _check(load_library().maaso_resource_partition(
        ctx.handle, int(n_gpus), _dptr(phi_t_star, torch.float32), _dptr(phi_l_star, torch.float32),
        _dptr(phi_h_star, torch.float32), _dptr(cand_t_star, torch.int32),
        _dptr(cand_l_star, torch.int32), _dptr(cand_h_star, torch.int32), int(n_req_l), int(n_req),
        _dptr(partition, torch.int32), _dptr(phi_opt, torch.float32), _stream_handle(stream)),
        "maaso_resource_partition")


def maaso_batch_size_prune(ctx: Context, *, n_cand, group_offsets, sat_count, latency, keep, n_kept,
                           stream=None) -> None:
    import torch
    n_groups = int(group_offsets.numel()) - 1
    _check(load_library().maaso_batch_size_prune(
        ctx.handle, int(n_cand), _dptr(group_offsets, torch.int32), n_groups,
        _dptr(sat_count, torch.int32), _dptr(latency, torch.float32), _dptr(keep, torch.uint8),
        _dptr(n_kept, torch.int32), _stream_handle(stream)), "maaso_batch_size_prune")


def maaso_resource_partition_requests(ctx: Context, *, n_cand, i_pad, n_inst, tp_idx, max_batch, occ,
                                      q_ticks, chain_offsets=None, n_gpus, n_req, prompt_len, out_len,
                                      slo_class, arrival_ticks=None, tight_classes, s_bar,
                                      pen_kappa=0.0, tbt_mode=0, window=0, policy=0, alpha, beta,
                                      gamma_t, gamma_l, work, stream=None) -> None:
    """`work`: dict of tensors keyed by the fields of maaso_partition_work (absent or None = NULL)."""
    import torch
    pl = _placements(n_cand, i_pad, n_inst, tp_idx, max_batch, occ, q_ticks)
    rq = _requests(n_req, prompt_len, out_len, slo_class, arrival_ticks)
    prm = Params(float(s_bar), float(pen_kappa), int(tbt_mode), int(window), int(policy))
    wts = ScoreWeights(float(alpha), float(beta), float(gamma_t), float(gamma_l))
    wk = PartitionWork(*[_dptr(work.get(name), getattr(torch, dt)) for name, dt in PARTITION_WORK_FIELDS])
    n_chains = 0 if chain_offsets is None else int(chain_offsets.numel()) - 1
    _check(load_library().maaso_resource_partition_requests(
        ctx.handle, C.byref(pl), _dptr(chain_offsets, torch.int32), n_chains, int(n_gpus), C.byref(rq),
        int(tight_classes), C.byref(prm), C.byref(wts), C.byref(wk), _stream_handle(stream)),
        "maaso_resource_partition_requests")


# ------------------------------------------------------------------------------------------------
# plumbing for tests and the benchmark: a workload's arrays as GPU tensors
# ------------------------------------------------------------------------------------------------

class DeviceWorkload:
    """Uploads the numpy arrays of a `workloads.Workload` once and keeps the tensors resident."""

    def __init__(self, w, device: int = 0):
        import torch
        dev = torch.device("cuda", device)
        self.w = w
        self.device = device

        def up(a, view):
            a = np.ascontiguousarray(a)
            if not a.flags.writeable:  # e.g. a broadcast view: torch wants a buffer of its own
                a = a.copy()
            return torch.from_numpy(a.view(view)).to(dev)

        self.prompt_len = up(w.prompt_len, np.int32)
        self.out_len = up(w.out_len, np.int32)
        self.slo_class = up(w.slo_class, np.uint8)
        self.arrival_ticks = None if w.arrival_ticks is None else up(w.arrival_ticks, np.int32)
        self.n_inst = up(w.n_inst, np.int32)
        self.tp_idx = up(w.tp_idx, np.uint8)
        self.max_batch = up(w.max_batch, np.int16)
        self.occ = up(w.occ, np.int32)
        self.q_ticks = up(w.q_ticks, np.int64)
        self.ctx = maaso_profile_tables_load(w.n_tp, w.b_cap, w.prefill_a, w.prefill_p, w.tbt,
                                             w.d_ttft, w.d_tbt, w.tp_degree, device)

    def request_args(self):
        return dict(n_req=self.w.n_req, prompt_len=self.prompt_len, out_len=self.out_len,
                    slo_class=self.slo_class)

    def param_args(self):
        return dict(s_bar=float(self.w.s_bar), pen_kappa=float(self.w.pen_kappa),
                    tbt_mode=int(self.w.tbt_mode), policy=int(self.w.policy))

    def sweep(self, stream=None, out=None, window=0, noalloc=False):
        """maaso_placement_sweep over all candidates; returns (sat_count, sat_ratio, best_cand).
        window > 0 selects the capacity-aware form; noalloc the entry point that works in the
        library's static scratch array."""
        import torch
        dev = self.prompt_len.device
        C_ = self.w.n_cand
        if out is None:
            out = (torch.empty(C_, dtype=torch.int32, device=dev),
                   torch.empty(C_, dtype=torch.float32, device=dev),
                   torch.empty(1, dtype=torch.int32, device=dev))
        (maaso_placement_sweep_noalloc if noalloc else maaso_placement_sweep)(
            self.ctx, n_cand=C_, i_pad=self.w.i_pad, n_inst=self.n_inst, tp_idx=self.tp_idx,
            max_batch=self.max_batch, occ=self.occ, q_ticks=self.q_ticks, **self.request_args(),
            arrival_ticks=self.arrival_ticks if window else None, window=window,
            **self.param_args(), sat_count=out[0], sat_ratio=out[1], best_cand=out[2], stream=stream)
        return out

    def score(self, alpha, beta, gamma_t, gamma_l, window=0, stream=None):
        """maaso_placement_score over all candidates; returns a dict of tensors."""
        import torch
        dev = self.prompt_len.device
        C_ = self.w.n_cand
        out = dict(sat_count=torch.empty(C_, dtype=torch.int32, device=dev),
                   best_cand=torch.empty(1, dtype=torch.int32, device=dev))
        for k in ("phi_s", "phi_t", "phi_l", "score"):
            out[k] = torch.empty(C_, dtype=torch.float32, device=dev)
        maaso_placement_score(
            self.ctx, n_cand=C_, i_pad=self.w.i_pad, n_inst=self.n_inst, tp_idx=self.tp_idx,
            max_batch=self.max_batch, occ=self.occ, q_ticks=self.q_ticks, **self.request_args(),
            arrival_ticks=self.arrival_ticks if window else None, window=window,
            **self.param_args(), alpha=alpha, beta=beta, gamma_t=gamma_t, gamma_l=gamma_l,
            stream=stream, **out)
        return out

    def score_sets(self, ranges, alpha, beta, gamma_t, gamma_l, window=0, stream=None):
        """maaso_placement_score_sets: the resident candidates against the request ranges
        [(lo, hi), ...] of the resident requests, one launch; returns one dict of tensors per range."""
        import torch
        dev = self.prompt_len.device
        C_ = self.w.n_cand
        sets, outs = [], []
        for lo, hi in ranges:
            out = dict(sat_count=torch.empty(C_, dtype=torch.int32, device=dev),
                       best_cand=torch.empty(1, dtype=torch.int32, device=dev))
            for k in ("phi_s", "phi_t", "phi_l", "score"):
                out[k] = torch.empty(C_, dtype=torch.float32, device=dev)
            outs.append(out)
            sets.append(dict(
                n_req=hi - lo, prompt_len=self.prompt_len[lo:hi], out_len=self.out_len[lo:hi],
                slo_class=self.slo_class[lo:hi],
                arrival_ticks=self.arrival_ticks[lo:hi] if window else None, **out))
        maaso_placement_score_sets(
            self.ctx, n_cand=C_, i_pad=self.w.i_pad, n_inst=self.n_inst, tp_idx=self.tp_idx,
            max_batch=self.max_batch, occ=self.occ, q_ticks=self.q_ticks, sets=sets, window=window,
            **self.param_args(), alpha=alpha, beta=beta, gamma_t=gamma_t, gamma_l=gamma_l,
            stream=stream)
        return outs

    def split_by_slo(self, tight_classes: int, stream=None):
        """maaso_split_by_slo of the resident requests; returns the four reordered streams (arrival
        None when the workload has none) and the device word holding |R_t|."""
        import torch
        dev = self.prompt_len.device
        out = dict(prompt_len_out=torch.empty_like(self.prompt_len),
                   out_len_out=torch.empty_like(self.out_len),
                   slo_class_out=torch.empty_like(self.slo_class),
                   arrival_ticks_out=None if self.arrival_ticks is None
                   else torch.empty_like(self.arrival_ticks),
                   n_tight=torch.empty(1, dtype=torch.int32, device=dev))
        maaso_split_by_slo(self.ctx, **self.request_args(), arrival_ticks=self.arrival_ticks,
                           tight_classes=tight_classes, stream=stream, **out)
        return out

    def partition_work(self, n_gpus: int, homogeneous: bool = True):
        """The arrays maaso_resource_partition_requests works in, for this workload's shape."""
        import torch
        dev = self.prompt_len.device
        C_, R = self.w.n_cand, self.w.n_req
        shape = dict(prompt_len_split=R, out_len_split=R, slo_class_split=R, arrival_ticks_split=R,
                     n_tight=1, partition=6, phi_opt=1)
        wk = {}
        for name, dt in PARTITION_WORK_FIELDS:
            if name.endswith("_h") or name.endswith("_h_star"):
                if not homogeneous:
                    continue
            if name == "arrival_ticks_split" and self.arrival_ticks is None:
                continue
            n = shape.get(name, n_gpus + 1 if name.endswith("_star") else C_)
            wk[name] = torch.empty(n, dtype=getattr(torch, dt), device=dev)
        return wk

    def resource_partition(self, chain_offsets, tight_classes: int, n_gpus: int, alpha, beta, gamma_t,
                           gamma_l, window=0, homogeneous=True, stream=None, work=None):
        """Alg. 2 over the resident candidates (growth chains of Alg. 1) and requests in ONE call of
        the library (maaso_resource_partition_requests): nothing comes back to the host in between.
        `chain_offsets`: numpy array or a device tensor; `work`: arrays from partition_work (made
        here when absent).  Returns the work dict (tensors)."""
        import torch
        dev = self.prompt_len.device
        if work is None:
            work = self.partition_work(n_gpus, homogeneous)
        offs = chain_offsets
        if not isinstance(offs, torch.Tensor):
            offs = torch.from_numpy(np.ascontiguousarray(chain_offsets).view(np.int32)).to(dev)
        maaso_resource_partition_requests(
            self.ctx, n_cand=self.w.n_cand, i_pad=self.w.i_pad, n_inst=self.n_inst, tp_idx=self.tp_idx,
            max_batch=self.max_batch, occ=self.occ, q_ticks=self.q_ticks, chain_offsets=offs,
            n_gpus=n_gpus, **self.request_args(),
            arrival_ticks=self.arrival_ticks if window else None,
            tight_classes=tight_classes, window=window, **self.param_args(), alpha=alpha, beta=beta,
            gamma_t=gamma_t, gamma_l=gamma_l, work=work, stream=stream)
        return work

    def resource_partition_steps(self, chain_offsets, tight_classes: int, n_gpus: int, alpha, beta,
                                 gamma_t, gamma_l, window=0, homogeneous=True, stream=None):
        """The same through the five separate entry points, with |R_t| read back by the host in the
        middle (what a caller composing Alg. 2 by hand would do).  Returns a dict of tensors."""
        import torch
        dev = self.prompt_len.device
        C_, R = self.w.n_cand, self.w.n_req
        sp = self.split_by_slo(tight_classes, stream=stream)
        n_t = int(sp["n_tight"].item())
        offs = torch.from_numpy(np.ascontiguousarray(chain_offsets).view(np.int32)).to(dev)
        res = dict(n_tight=n_t)

        split = (sp["prompt_len_out"], sp["out_len_out"], sp["slo_class_out"], sp["arrival_ticks_out"])
        runs = [("t", 0, n_t, split), ("l", n_t, R, split)]
        if homogeneous:
            runs.append(("h", 0, R, (self.prompt_len, self.out_len, self.slo_class, self.arrival_ticks)))
        sets = []
        for tag, lo, hi, src in runs:
            res[f"score_{tag}"] = torch.empty(C_, dtype=torch.float32, device=dev)
            sets.append(dict(
                n_req=hi - lo, prompt_len=src[0][lo:hi], out_len=src[1][lo:hi], slo_class=src[2][lo:hi],
                arrival_ticks=None if (src[3] is None or not window) else src[3][lo:hi],
                sat_count=torch.empty(C_, dtype=torch.int32, device=dev), score=res[f"score_{tag}"]))
        # one launch scores every candidate against every set
        maaso_placement_score_sets(
            self.ctx, n_cand=C_, i_pad=self.w.i_pad, n_inst=self.n_inst, tp_idx=self.tp_idx,
            max_batch=self.max_batch, occ=self.occ, q_ticks=self.q_ticks, sets=sets, window=window,
            **self.param_args(), alpha=alpha, beta=beta, gamma_t=gamma_t, gamma_l=gamma_l,
            stream=stream)
        for tag, _, _, _ in runs:
            phi = torch.empty(n_gpus + 1, dtype=torch.float32, device=dev)
            cand = torch.empty(n_gpus + 1, dtype=torch.int32, device=dev)
            maaso_ins_deploy_select(self.ctx, n_cand=C_, i_pad=self.w.i_pad, n_inst=self.n_inst,
                                    tp_idx=self.tp_idx, score=res[f"score_{tag}"], chain_offsets=offs,
                                    n_gpus=n_gpus, phi_star=phi, cand_star=cand, stream=stream)
            res[f"phi_{tag}_star"], res[f"cand_{tag}_star"] = phi, cand
        res["partition"] = torch.empty(6, dtype=torch.int32, device=dev)
        res["phi_opt"] = torch.empty(1, dtype=torch.float32, device=dev)
        maaso_resource_partition(
            self.ctx, n_gpus=n_gpus, phi_t_star=res["phi_t_star"], phi_l_star=res["phi_l_star"],
            phi_h_star=res.get("phi_h_star"), cand_t_star=res["cand_t_star"],
            cand_l_star=res["cand_l_star"], cand_h_star=res.get("cand_h_star"), n_req_l=R - n_t,
            n_req=R, partition=res["partition"], phi_opt=res["phi_opt"], stream=stream)
        res["split"] = sp
        return res

    def assign(self, cand: int = 0, window=None, latencies: bool = True, stream=None, out=None,
               tbt_mode=None):
        """maaso_score_assign on candidate `cand` (state tensors are cloned, so the workload's own
        copies stay as uploaded).  Returns a dict of tensors, plus the state after the call."""
        import torch
        dev = self.prompt_len.device
        R = self.w.n_req
        window = self.w.window if window is None else window
        if out is None:
            out = dict(chosen=torch.empty(R, dtype=torch.int32, device=dev),
                       slack=torch.empty(R, dtype=torch.float32, device=dev),
                       n_satisfied=torch.empty(1, dtype=torch.int64, device=dev))
            if latencies:
                for k in ("ttft", "tbt", "e2e"):
                    out[k] = torch.empty(R, dtype=torch.float32, device=dev)
        occ, q = self.occ[cand:cand + 1], self.q_ticks[cand:cand + 1]
        if window:  # only the windowed form writes the state
            occ, q = occ.clone(), q.clone()
        prm = self.param_args()
        if tbt_mode is not None:
            prm["tbt_mode"] = tbt_mode
        maaso_score_assign(
            self.ctx, n_cand=1, i_pad=self.w.i_pad, n_inst=self.n_inst[cand:cand + 1],
            tp_idx=self.tp_idx[cand:cand + 1], max_batch=self.max_batch[cand:cand + 1], occ=occ,
            q_ticks=q, **self.request_args(), arrival_ticks=self.arrival_ticks, **prm,
            window=window, stream=stream,
            **{k: out.get(k) for k in ("chosen", "slack", "ttft", "tbt", "e2e", "n_satisfied")})
        res = dict(out)
        res["occ"], res["q_ticks"] = occ, q
        return res

    def assign_selected(self, cand, window=None, latencies: bool = True, stream=None, out=None):
        """maaso_score_assign_selected over all resident candidates, the row named by the device
        word `cand` (int32 tensor [1]).  With window > 0 the whole state is cloned first."""
        import torch
        dev = self.prompt_len.device
        R = self.w.n_req
        window = self.w.window if window is None else window
        if out is None:
            out = dict(chosen=torch.empty(R, dtype=torch.int32, device=dev),
                       slack=torch.empty(R, dtype=torch.float32, device=dev),
                       n_satisfied=torch.empty(1, dtype=torch.int64, device=dev))
            if latencies:
                for k in ("ttft", "tbt", "e2e"):
                    out[k] = torch.empty(R, dtype=torch.float32, device=dev)
        occ, q = self.occ, self.q_ticks
        if window:
            occ, q = occ.clone(), q.clone()
        maaso_score_assign_selected(
            self.ctx, cand=cand, n_cand=self.w.n_cand, i_pad=self.w.i_pad, n_inst=self.n_inst,
            tp_idx=self.tp_idx, max_batch=self.max_batch, occ=occ, q_ticks=q, **self.request_args(),
            arrival_ticks=self.arrival_ticks, **self.param_args(), window=window, stream=stream,
            **{k: out.get(k) for k in ("chosen", "slack", "ttft", "tbt", "e2e", "n_satisfied")})
        res = dict(out)
        res["occ"], res["q_ticks"] = occ, q
        return res

    def close(self):
        self.ctx.close()
