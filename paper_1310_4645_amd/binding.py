"""ctypes binding of libprs.so: argument marshalling only.

Tensors are torch CUDA(HIP) tensors used as plain device buffers; the stream
is torch's current stream.  Function names and argument order follow
include/prs.h.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

PRS_UNI, PRS_BI = 0, 1
PRS_COST_I64, PRS_COST_F64 = 0, 1
PRS_I32, PRS_F32, PRS_F64, PRS_I64 = 0, 1, 2, 3
PRS_OP_SUM, PRS_OP_MAX = 0, 0x100
PRS_CALL_SIMULATE, PRS_CALL_SCHEDULE, PRS_CALL_REPLAY, PRS_CALL_OFFSETS, PRS_CALL_SEARCH, PRS_CALL_UNEQUAL = 0, 1, 2, 3, 4, 5

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = ("prs_abi_version", "prs_workspace_bytes", "simulate_completion_batch", "prs_pair_offsets",
           "greedy_schedule_batch", "replay_reduction", "replay_reduction_static", "optimal_segmentation_batch",
           "unequal_segmentation_batch", "butterfly_threshold_batch", "prs_measure_alu_ceiling")


class PrsError(RuntimeError):
    pass


class _Configs(C.Structure):
    _fields_ = [("p", C.c_void_p), ("q_req", C.c_void_p), ("m", C.c_void_p),
                ("alpha", C.c_void_p), ("beta", C.c_void_p), ("gamma", C.c_void_p)]


class _Times(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("greedy", "binomial", "pipeline", "binary", "revopt", "butterfly",
                                          "lower_bound", "q_eff", "cfg_status")]


class _Best(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("T_greedy", "T_pipeline", "T_binary", "T_revopt", "q_greedy", "q_pipeline",
                                          "q_binary", "q_revopt", "cfg_status")]


class _Unequal(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("T_all", "T_best", "cuts_best", "n_best", "T_equi", "cuts_equi",
                                          "equi_optimal", "cfg_status")]


class _Tuning(C.Structure):
    _fields_ = [("uni_group_pairs", C.c_int64 * 3), ("uni_wave_log2", C.c_int32), ("bi_list_entries", C.c_int32),
                ("uni_wide_procs", C.c_int32), ("reserved", C.c_int32)]


def _tuning(t):
    """None, or a dict with any of uni_group_pairs (three limits), uni_wave_log2, bi_list_entries, uni_wide_procs
    -> prs_tuning*."""
    if t is None:
        return None
    unknown = set(t) - {"uni_group_pairs", "uni_wave_log2", "bi_list_entries", "uni_wide_procs"}
    if unknown:
        raise PrsError(f"unknown tuning fields {sorted(unknown)}")
    pairs = t.get("uni_group_pairs", (-1, -1, -1))
    return C.byref(_Tuning((C.c_int64 * 3)(*[int(v) for v in pairs]), int(t.get("uni_wave_log2", 0)),
                           int(t.get("bi_list_entries", 0)), int(t.get("uni_wide_procs", 0)), 0))


def library_path() -> str:
    return os.path.join(_HERE, "libprs.so")


def load_library():
    """Loads the in-tree libprs.so; raises if it has not been built."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise PrsError(f"{path} is missing: build it with `python -m paper_1310_4645_amd.build` "
                           "(there is no CPU fallback)")
        lib = C.CDLL(path)
        lib.prs_abi_version.restype = C.c_int
        lib.prs_workspace_bytes.restype = C.c_size_t
        lib.prs_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int32, C.c_int32]
        lib.simulate_completion_batch.restype = C.c_int
        lib.simulate_completion_batch.argtypes = [C.POINTER(_Configs), C.c_int64, C.c_int, C.c_int, C.c_int32, C.c_int32,
                                                  C.POINTER(_Times), C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.prs_pair_offsets.restype = C.c_int
        lib.prs_pair_offsets.argtypes = [C.POINTER(_Configs), C.c_int64, C.c_int, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
        lib.greedy_schedule_batch.restype = C.c_int
        lib.greedy_schedule_batch.argtypes = [C.POINTER(_Configs), C.c_int64, C.c_int, C.c_int, C.c_int32, C.c_int32,
                                              C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.replay_reduction.restype = C.c_int
        lib.replay_reduction.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                         C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
        lib.replay_reduction_static.restype = C.c_int
        lib.replay_reduction_static.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                                C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.butterfly_threshold_batch.restype = C.c_int
        lib.butterfly_threshold_batch.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_int32, C.c_int32, C.c_int32, C.c_double,
                                                  C.c_double, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.prs_measure_alu_ceiling.restype = C.c_int
        lib.prs_measure_alu_ceiling.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
        lib.optimal_segmentation_batch.restype = C.c_int
        lib.optimal_segmentation_batch.argtypes = [C.POINTER(_Configs), C.c_int64, C.c_int, C.c_int, C.c_int32, C.c_int32,
                                                   C.POINTER(_Best), C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.unequal_segmentation_batch.restype = C.c_int
        lib.unequal_segmentation_batch.argtypes = [C.POINTER(_Configs), C.c_int64, C.c_int, C.c_int32, C.c_int32,
                                                   C.POINTER(_Unequal), C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        _LIB = lib
    return _LIB


def exported_symbols():
    lib = load_library()
    return [s for s in EXPORTS if hasattr(lib, s)]


def _check(rc: int, what: str):
    if rc != 0:
        raise PrsError(f"{what} failed with prs_status {rc} "
                       f"({ {1: 'PRS_EINVAL', 2: 'PRS_ENOSPC', 3: 'PRS_EDEVICE'}.get(rc, '?') })")


def _dp(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class DeviceConfigs:
    """A batch of configurations resident in device memory (SoA)."""
    p: object
    q_req: object
    m: object
    alpha: object
    beta: object
    gamma: object
    cost: int

    @staticmethod
    def from_host(cfgs, device="cuda"):
        import torch
        cost = PRS_COST_I64 if cfgs.cost == "i64" else PRS_COST_F64
        tt = torch.int64 if cost == PRS_COST_I64 else torch.float64
        f = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), dtype=dt).to(device)
        return DeviceConfigs(f(cfgs.p, torch.int32), f(cfgs.q_req, torch.int32), f(cfgs.m, torch.int64),
                             f(cfgs.alpha, tt), f(cfgs.beta, tt), f(cfgs.gamma, tt), cost)

    def __len__(self):
        return int(self.p.shape[0])

    def struct(self) -> _Configs:
        return _Configs(self.p.data_ptr(), self.q_req.data_ptr(), self.m.data_ptr(),
                        self.alpha.data_ptr(), self.beta.data_ptr(), self.gamma.data_ptr())


def prs_workspace_bytes(call, model, cost, n, p_max, q_max) -> int:
    return int(load_library().prs_workspace_bytes(call, model, cost, n, p_max, q_max))


def _workspace(nbytes, device):
    import torch
    return torch.empty(max(int(nbytes), 256) + 256, dtype=torch.uint8, device=device)


def _aligned_ptr(ws):
    return (ws.data_ptr() + 255) // 256 * 256


def simulate_completion_batch(cfg: DeviceConfigs, model: int, p_max: int, q_max: int, out: dict | None = None,
                              workspace=None, tuning=None):
    """Returns a dict of device tensors: greedy, binomial, pipeline, binary, revopt (cost type), butterfly,
    lower_bound (float64), q_eff, cfg_status (int32).  `out` may pre-allocate any of them (None = skip)."""
    import torch
    lib = load_library()
    n = len(cfg)
    dev = cfg.p.device
    tt = torch.int64 if cfg.cost == PRS_COST_I64 else torch.float64
    if out is None:
        out = {k: torch.empty(n, dtype=tt, device=dev) for k in ("greedy", "binomial", "pipeline", "binary", "revopt")}
        out.update({k: torch.empty(n, dtype=torch.float64, device=dev) for k in ("butterfly", "lower_bound")})
        out.update({k: torch.empty(n, dtype=torch.int32, device=dev) for k in ("q_eff", "cfg_status")})
    need = prs_workspace_bytes(PRS_CALL_SIMULATE, model, cfg.cost, n, p_max, q_max)
    ws = workspace if workspace is not None else _workspace(need, dev)
    times = _Times(*[(out.get(k).data_ptr() if out.get(k) is not None else None) for k, _ in _Times._fields_])
    cs = cfg.struct()
    rc = lib.simulate_completion_batch(C.byref(cs), n, model, cfg.cost, p_max, q_max, C.byref(times),
                                       C.c_void_p(_aligned_ptr(ws)), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream(),
                                       _tuning(tuning))
    _check(rc, "simulate_completion_batch")
    out["_workspace"] = ws
    return out


def optimal_segmentation_batch(cfg: DeviceConfigs, model: int, p_max: int, q_max: int, workspace=None, tuning=None):
    """Best power-of-two segment count per algorithm.  Returns a dict of device tensors: T_greedy, T_pipeline,
    T_binary, T_revopt (cost type), q_greedy, q_pipeline, q_binary, q_revopt, cfg_status (int32).  cfg.q_req is
    not read."""
    import torch
    lib = load_library()
    n = len(cfg)
    dev = cfg.p.device
    tt = torch.int64 if cfg.cost == PRS_COST_I64 else torch.float64
    out = {k: torch.empty(n, dtype=tt, device=dev) for k in ("T_greedy", "T_pipeline", "T_binary", "T_revopt")}
    out.update({k: torch.empty(n, dtype=torch.int32, device=dev)
                for k in ("q_greedy", "q_pipeline", "q_binary", "q_revopt", "cfg_status")})
    need = prs_workspace_bytes(PRS_CALL_SEARCH, model, cfg.cost, n, p_max, q_max)
    ws = workspace if workspace is not None else _workspace(need, dev)
    best = _Best(*[out[k].data_ptr() for k, _ in _Best._fields_])
    cs = cfg.struct()
    rc = lib.optimal_segmentation_batch(C.byref(cs), n, model, cfg.cost, p_max, q_max, C.byref(best),
                                        C.c_void_p(_aligned_ptr(ws)), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream(),
                                        _tuning(tuning))
    _check(rc, "optimal_segmentation_batch")
    out["_workspace"] = ws
    return out


def unequal_segmentation_batch(cfg: DeviceConfigs, p_max: int, m_max: int, want_all=True, workspace=None, tuning=None):
    """Every segmentation of cfg.m <= m_max units through uni-greedy.  Returns a dict of device tensors: T_all
    (n x 2^(m_max-1), cost type, only if want_all), T_best, T_equi (cost type), cuts_best, cuts_equi (int32 holding
    the cut patterns), n_best, equi_optimal, cfg_status (int32).  cfg.q_req is not read."""
    import torch
    lib = load_library()
    n = len(cfg)
    dev = cfg.p.device
    tt = torch.int64 if cfg.cost == PRS_COST_I64 else torch.float64
    out = {k: torch.empty(n, dtype=tt, device=dev) for k in ("T_best", "T_equi")}
    out.update({k: torch.empty(n, dtype=torch.int32, device=dev)
                for k in ("cuts_best", "n_best", "cuts_equi", "equi_optimal", "cfg_status")})
    out["T_all"] = torch.empty((n, 1 << (m_max - 1)), dtype=tt, device=dev) if want_all else None
    need = prs_workspace_bytes(PRS_CALL_UNEQUAL, PRS_UNI, cfg.cost, n, p_max, m_max)
    ws = workspace if workspace is not None else _workspace(need, dev)
    res = _Unequal(*[None if out[k] is None else out[k].data_ptr() for k, _ in _Unequal._fields_])
    cs = cfg.struct()
    rc = lib.unequal_segmentation_batch(C.byref(cs), n, cfg.cost, p_max, m_max, C.byref(res),
                                        C.c_void_p(_aligned_ptr(ws)), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream(),
                                        _tuning(tuning))
    _check(rc, "unequal_segmentation_batch")
    out["_workspace"] = ws
    return out


def prs_pair_offsets(cfg: DeviceConfigs, p_max: int, q_max: int):
    import torch
    lib = load_library()
    n = len(cfg)
    off = torch.empty(n + 1, dtype=torch.int64, device=cfg.p.device)
    cs = cfg.struct()
    rc = lib.prs_pair_offsets(C.byref(cs), n, cfg.cost, p_max, q_max, _dp(off), None, 0, _stream())
    _check(rc, "prs_pair_offsets")
    return off


def greedy_schedule_batch(cfg: DeviceConfigs, model: int, p_max: int, q_max: int, pair_offset, pair_capacity: int,
                          src=None, dst=None, seg=None, t_start=None, want=("src", "dst", "seg", "t_start"),
                          workspace=None, tuning=None):
    """Returns dict(src, dst, seg, t_start, T_greedy, cfg_status) of device tensors."""
    import torch
    lib = load_library()
    n = len(cfg)
    dev = cfg.p.device
    tt = torch.int64 if cfg.cost == PRS_COST_I64 else torch.float64
    cap = int(pair_capacity)
    if src is None and "src" in want: src = torch.empty(cap, dtype=torch.int32, device=dev)
    if dst is None and "dst" in want: dst = torch.empty(cap, dtype=torch.int32, device=dev)
    if seg is None and "seg" in want: seg = torch.empty(cap, dtype=torch.int32, device=dev)
    if t_start is None and "t_start" in want: t_start = torch.empty(cap, dtype=tt, device=dev)
    T = torch.empty(n, dtype=tt, device=dev)
    st = torch.empty(n, dtype=torch.int32, device=dev)
    need = prs_workspace_bytes(PRS_CALL_SCHEDULE, model, cfg.cost, n, p_max, q_max)
    ws = workspace if workspace is not None else _workspace(need, dev)
    cs = cfg.struct()
    rc = lib.greedy_schedule_batch(C.byref(cs), n, model, cfg.cost, p_max, q_max, _dp(pair_offset), cap,
                                   _dp(src), _dp(dst), _dp(seg), _dp(t_start), _dp(T), _dp(st),
                                   C.c_void_p(_aligned_ptr(ws)), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream(),
                                   _tuning(tuning))
    _check(rc, "greedy_schedule_batch")
    return {"src": src, "dst": dst, "seg": seg, "t_start": t_start, "T_greedy": T, "cfg_status": st, "_workspace": ws}


def replay_reduction(p: int, q: int, seg_elem_offset, src, dst, seg, inp, out=None, workspace=None, op=PRS_OP_SUM):
    """inp: device tensor [p, n_elems] (int32, int64, float32 or float64, rows may be strided); seg_elem_offset:
    host int64 array of q+1 entries; op: PRS_OP_SUM or PRS_OP_MAX.  Returns (out, status) device tensors."""
    import torch
    lib = load_library()
    off = np.ascontiguousarray(seg_elem_offset, dtype=np.int64)
    n_elems = int(inp.shape[1])
    assert inp.stride(1) == 1
    kinds = {torch.int32: PRS_I32, torch.float32: PRS_F32, torch.float64: PRS_F64, torch.int64: PRS_I64}
    if inp.dtype not in kinds:
        raise PrsError(f"replay_reduction: unsupported element type {inp.dtype}")
    dtype = kinds[inp.dtype] | op
    if out is None:
        out = torch.empty(n_elems, dtype=inp.dtype, device=inp.device)
    status = torch.empty(1, dtype=torch.int32, device=inp.device)
    need = prs_workspace_bytes(PRS_CALL_REPLAY, PRS_UNI, 0, 1, p, q)
    ws = workspace if workspace is not None else _workspace(need, inp.device)
    rc = lib.replay_reduction(p, q, off.ctypes.data_as(C.c_void_p), _dp(src), _dp(dst), _dp(seg), int(src.shape[0]),
                              _dp(inp), int(inp.stride(0)), n_elems, dtype, _dp(out), _dp(status),
                              C.c_void_p(_aligned_ptr(ws)), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream())
    _check(rc, "replay_reduction")
    return out, status


def replay_reduction_static(p: int, q: int, seg_elem_offset, src, dst, seg, inp, out, status, op=PRS_OP_SUM):
    """replay_reduction without a workspace and without any allocation: `out` ([n_elems], dtype of inp) and
    `status` (one int32) are the caller's device tensors.  Raises PrsError (PRS_ENOSPC) for schedules beyond the
    library's fixed scratch array."""
    import torch
    lib = load_library()
    off = np.ascontiguousarray(seg_elem_offset, dtype=np.int64)
    n_elems = int(inp.shape[1])
    assert inp.stride(1) == 1
    kinds = {torch.int32: PRS_I32, torch.float32: PRS_F32, torch.float64: PRS_F64, torch.int64: PRS_I64}
    if inp.dtype not in kinds:
        raise PrsError(f"replay_reduction_static: unsupported element type {inp.dtype}")
    rc = lib.replay_reduction_static(p, q, off.ctypes.data_as(C.c_void_p), _dp(src), _dp(dst), _dp(seg), int(src.shape[0]),
                                     _dp(inp), int(inp.stride(0)), n_elems, kinds[inp.dtype] | op, _dp(out), _dp(status),
                                     _stream())
    _check(rc, "replay_reduction_static")
    return out, status


def butterfly_threshold_batch(p, alpha: float, q_max: int, m_log2_first: int, m_log2_last: int, ratio_lo: float,
                              ratio_hi: float, steps: int):
    """p: device int32 tensor of machine sizes.  Returns dict(ratio_below, ratio_above (float64), cfg_status (int32))
    of device tensors: the bracket of the largest beta/gamma at which the butterfly still beats bi-greedy's time for
    some message size 2^k, after `steps` bisection steps from [ratio_lo, ratio_hi]."""
    import torch
    lib = load_library()
    n = int(p.shape[0])
    out = {"ratio_below": torch.empty(n, dtype=torch.float64, device=p.device),
           "ratio_above": torch.empty(n, dtype=torch.float64, device=p.device),
           "cfg_status": torch.empty(n, dtype=torch.int32, device=p.device)}
    rc = lib.butterfly_threshold_batch(_dp(p), n, float(alpha), int(q_max), int(m_log2_first), int(m_log2_last), float(ratio_lo),
                                       float(ratio_hi), int(steps), _dp(out["ratio_below"]), _dp(out["ratio_above"]),
                                       _dp(out["cfg_status"]), _stream())
    _check(rc, "butterfly_threshold_batch")
    return out


def prs_measure_alu_ceiling(steps_per_lane: int, blocks: int, sink):
    """Enqueues the register-only microkernel (blocks x 256 lanes x steps_per_lane steps of Algorithm 1's arithmetic)."""
    _check(load_library().prs_measure_alu_ceiling(int(steps_per_lane), int(blocks), _dp(sink), _stream()), "prs_measure_alu_ceiling")
