"""ctypes binding of libdyn.so: same names as include/dyn.h, argument marshalling only.

DEVICE arguments are torch tensors on the GPU (PyTorch provides device memory and the
stream, nothing else); HOST arguments are NumPy arrays.  Every function raises DynError
when the library returns a negative status.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch

__all__ = ["DynError", "Profile", "dyn_profile_load", "dyn_profile_free", "dyn_trace_ingest",
           "dyn_trace_ingest_workspace", "dyn_eval_space", "dyn_eval_space_workspace", "dyn_cell_stats",
           "dyn_workspace_status", "dyn_select_config", "dyn_eval_select", "dyn_eval_select_static", "dyn_eval_tune",
           "DYN_STATIC_WORKSPACE_BYTES", "dyn_last_error", "lib_path",
           "dyn_timing_enable", "dyn_timing_reset", "dyn_timing_read", "DYN_K_CELL", "DYN_K_SPACE", "DYN_K_SELECT",
           "DYN_K_TOTALS",
           "DYN_F_FEASIBLE", "DYN_F_OVERLOAD", "DYN_F_TTFT", "DYN_F_TBT", "DYN_F_BUDGET", "DYN_F_EMPTY",
           "DYN_WS_BAD_OFFSETS", "DYN_WS_BAD_REQUEST", "DYN_WS_TICK_RANK", "DYN_WS_SORT_ABANDONED", "dyn_eval_select_ticks",
           "dyn_eval_ticks_workspace", "DYN_K_TICK_TOP", "DYN_K_TICK_SPACE", "DYN_K_TICK_MERGE", "DYN_K_MIXED_TYPES", "DYN_K_MIXED_COMBINE",
           "MixedPlan", "dyn_mixed_workspace", "dyn_eval_select_mixed", "DYN_K_PATH", "dyn_select_path_workspace",
           "dyn_select_path", "dyn_account_workspace", "dyn_account", "dyn_hierarchy_workspace", "dyn_hierarchy", "DYN_K_HIER", "DYN_TICK_LIMIT", "DYN_TICK_DEPTH"]

DYN_F_FEASIBLE, DYN_F_OVERLOAD, DYN_F_TTFT, DYN_F_TBT, DYN_F_BUDGET, DYN_F_EMPTY = 1, 2, 4, 8, 16, 32
DYN_WS_BAD_OFFSETS, DYN_WS_BAD_REQUEST, DYN_WS_TICK_RANK, DYN_WS_SORT_ABANDONED = 1, 2, 4, 8
DYN_TICK_LIMIT, DYN_TICK_DEPTH = 64, 8192
DYN_STATIC_WORKSPACE_BYTES = 16 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libdyn.so")


if not os.path.exists(lib_path()):
    raise ImportError(f"{lib_path()} is missing: build it with `python paper_2408_00741_amd/build.py` "
                      "(there is no fallback implementation)")
_lib = C.CDLL(lib_path())

_vp, _i32, _i64, _f64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_double, C.c_size_t


class _ProfileDesc(C.Structure):
    _fields_ = [("n_class", _i32), ("n_tp", _i32), ("tp", _vp), ("n_f", _i32), ("f_mhz", _vp),
                ("n_rho", _i32), ("rho", _vp), ("prefill_ms_per_tok", _vp), ("tbt_ms", _vp),
                ("power_w", _vp), ("max_load_tps", _vp)]


class _ClassEdges(C.Structure):
    _fields_ = [("n_model", _i32), ("n_in_bin", _i32), ("n_out_bin", _i32), ("in_edge", _vp), ("out_edge", _vp)]


class _TraceView(C.Structure):
    _fields_ = [("n_req", _i64), ("n_window", _i32), ("window_s", _f64), ("in_tok", _vp), ("out_tok", _vp),
                ("cell_off", _vp)]


class _Config(C.Structure):
    _fields_ = [("n_inst", _i32), ("tp_index", _i32), ("f_mhz", _f64)]


class _Objective(C.Structure):
    _fields_ = [("slo_ttft_ms", _vp), ("slo_tbt_ms", _vp), ("pct_num", _i32), ("pct_den", _i32),
                ("gpu_budget", _vp), ("idle_cost_weight", _f64)]


class _Space(C.Structure):
    _fields_ = [("energy_j", _vp), ("p99_ttft_ms", _vp), ("p99_tbt_ms", _vp), ("flags", _vp)]


class _Selection(C.Structure):
    _fields_ = [("sel", _vp), ("sel_energy_j", _vp), ("sel_cost", _vp), ("window_energy_j", _vp),
                ("window_infeasible", _vp)]


class _MixedSpace(C.Structure):
    _fields_ = [("n_share", _i32), ("n_max", _vp)]


class _MixedSelection(C.Structure):
    _fields_ = [("energy_j", _vp), ("n_inst", _vp), ("f_index", _vp), ("share", _vp), ("window_energy_j", _vp),
                ("window_infeasible", _vp)]


class _Transitions(C.Structure):
    _fields_ = [("n_layout", _i32), ("layout", _vp), ("transition_j", _vp)]


class _PathSelection(C.Structure):
    _fields_ = [("sel", _vp), ("sel_energy_j", _vp), ("path_cost", _vp), ("window_energy_j", _vp),
                ("window_infeasible", _vp)]


class _Rates(C.Structure):
    _fields_ = [("gpu_hour_price", _f64), ("kwh_price", _f64), ("carbon_g_per_kwh", _vp), ("gpus_per_server", _i32)]


class _Accounting(C.Structure):
    _fields_ = [("gpus", _vp), ("gpu_cost", _vp), ("energy_cost", _vp), ("carbon_g", _vp), ("totals", _vp)]


class _Controllers(C.Structure):
    _fields_ = [("epoch_windows", _i32), ("tp_ref_index", _i32), ("f_ref_index", _i32), ("gpus_per_node", _i32),
                ("n_layout", _i32), ("spill", _i32), ("lay_n", _vp), ("lay_tp_index", _vp), ("transition_j", _vp)]


class _HierarchyOut(C.Structure):
    _fields_ = [("nodes", _vp), ("layout_sel", _vp), ("f_sel", _vp), ("energy_j", _vp), ("violations", _vp),
                ("window_energy_j", _vp), ("window_infeasible", _vp), ("path_cost", _vp), ("keep", _vp)]


_lib.dyn_last_error.restype = C.c_char_p
_lib.dyn_profile_load.restype = C.c_int
_lib.dyn_profile_load.argtypes = [C.POINTER(_ProfileDesc), _vp, C.POINTER(_vp)]
_lib.dyn_profile_free.restype = None
_lib.dyn_profile_free.argtypes = [_vp]
_lib.dyn_trace_ingest_workspace.restype = _sz
_lib.dyn_trace_ingest_workspace.argtypes = [_i64, _i32, _i32]
_lib.dyn_trace_ingest.restype = C.c_int
_lib.dyn_trace_ingest.argtypes = [_vp, _vp, _vp, _vp, _i64, C.POINTER(_ClassEdges), _i32, _f64, _vp, _vp, _vp,
                                  _vp, _sz, _vp]
_lib.dyn_eval_space_workspace.restype = _sz
_lib.dyn_eval_space_workspace.argtypes = [_i32, _i32, _i32]
_lib.dyn_eval_space.restype = C.c_int
_lib.dyn_eval_space.argtypes = [_vp, C.POINTER(_TraceView), C.POINTER(_Config), _i32, C.POINTER(_Objective),
                                C.POINTER(_Space), _vp, _sz, _vp]
_lib.dyn_cell_stats.restype = C.c_int
_lib.dyn_cell_stats.argtypes = [_vp, _sz, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.dyn_workspace_status.restype = C.c_int
_lib.dyn_workspace_status.argtypes = [_vp, _vp, C.POINTER(C.c_uint32)]
_lib.dyn_select_config.restype = C.c_int
_lib.dyn_select_config.argtypes = [_vp, C.POINTER(_Space), C.POINTER(_Config), _i32, C.POINTER(_Objective), _i32,
                                   _f64, C.POINTER(_Selection), _vp]


_lib.dyn_eval_select.restype = C.c_int
_lib.dyn_eval_select.argtypes = [_vp, C.POINTER(_TraceView), C.POINTER(_Config), _i32, C.POINTER(_Objective),
                                 C.POINTER(_Space), C.POINTER(_Selection), _vp, _sz, _vp]
_lib.dyn_eval_tune.restype = C.c_int
_lib.dyn_eval_tune.argtypes = [_vp, C.POINTER(_TraceView), C.POINTER(_Config), _i32, C.POINTER(_Objective),
                               C.POINTER(_Space), C.POINTER(_Selection), _vp, _sz, _vp, C.POINTER(_i32)]
_lib.dyn_eval_select_static.restype = C.c_int
_lib.dyn_eval_select_static.argtypes = [_vp, C.POINTER(_TraceView), C.POINTER(_Config), _i32, C.POINTER(_Objective),
                                        C.POINTER(_Space), C.POINTER(_Selection), _vp, _vp]
_lib.dyn_eval_ticks_workspace.restype = _sz
_lib.dyn_eval_ticks_workspace.argtypes = [_i64, _i32, _i32, _i32, _i32]
_lib.dyn_eval_select_ticks.restype = C.c_int
_lib.dyn_eval_select_ticks.argtypes = [_vp, C.POINTER(_TraceView), _i32, C.POINTER(_Config), _i32,
                                       C.POINTER(_Objective), C.POINTER(_Space), C.POINTER(_Selection), _vp, _sz, _vp]
_lib.dyn_mixed_workspace.restype = _sz
_lib.dyn_mixed_workspace.argtypes = [_vp, _i32, C.POINTER(_MixedSpace)]
_lib.dyn_eval_select_mixed.restype = C.c_int
_lib.dyn_eval_select_mixed.argtypes = [_vp, C.POINTER(_TraceView), C.POINTER(_MixedSpace), C.POINTER(_Objective),
                                       C.POINTER(_MixedSelection), _vp, _sz, _vp]
_lib.dyn_select_path_workspace.restype = _sz
_lib.dyn_select_path_workspace.argtypes = [_i32, _i32, _i32, _i32]
_lib.dyn_select_path.restype = C.c_int
_lib.dyn_select_path.argtypes = [_vp, C.POINTER(_Space), C.POINTER(_Config), _i32, C.POINTER(_Objective),
                                 C.POINTER(_Transitions), _i32, _f64, C.POINTER(_PathSelection), _vp, _sz, _vp]
_lib.dyn_account_workspace.restype = _sz
_lib.dyn_account_workspace.argtypes = [_i32]
_lib.dyn_account.restype = C.c_int
_lib.dyn_account.argtypes = [_vp, _vp, _vp, C.POINTER(_Config), _i32, _i32, _f64, C.POINTER(_Rates),
                             C.POINTER(_Accounting), _vp, _sz, _vp]
_lib.dyn_hierarchy_workspace.restype = _sz
_lib.dyn_hierarchy_workspace.argtypes = [_i32, _i32, _i32, _i32]
_lib.dyn_hierarchy.restype = C.c_int
_lib.dyn_hierarchy.argtypes = [_vp, C.POINTER(_TraceView), C.POINTER(_TraceView), _i32, C.POINTER(_Controllers),
                               C.POINTER(_Objective), C.POINTER(_HierarchyOut), _vp, _sz, _vp]
_lib.dyn_timing_enable.restype = C.c_int
_lib.dyn_timing_enable.argtypes = [C.c_int, _i32]
_lib.dyn_timing_reset.restype = C.c_int
_lib.dyn_timing_read.restype = C.c_int
_lib.dyn_timing_read.argtypes = [_i32, C.POINTER(C.c_double), C.POINTER(_i64)]
(DYN_K_CELL, DYN_K_SPACE, DYN_K_SELECT, DYN_K_TOTALS, DYN_K_TICK_TOP, DYN_K_TICK_SPACE, DYN_K_TICK_MERGE,
 DYN_K_MIXED_TYPES, DYN_K_MIXED_COMBINE, DYN_K_PATH, DYN_K_HIER) = range(11)


def dyn_timing_enable(on: bool, max_launches: int = 4096):
    _check(_lib.dyn_timing_enable(1 if on else 0, max_launches), "dyn_timing_enable")


def dyn_timing_reset():
    _check(_lib.dyn_timing_reset(), "dyn_timing_reset")


def dyn_timing_read(kernel: int):
    """(summed duration in ms, number of launches) of one kernel since the last reset."""
    ms, n = C.c_double(0.0), _i64(0)
    _check(_lib.dyn_timing_read(kernel, C.byref(ms), C.byref(n)), "dyn_timing_read")
    return ms.value, n.value


class DynError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where} failed with status {status}: {dyn_last_error()}")


def dyn_last_error() -> str:
    return (_lib.dyn_last_error() or b"").decode()


def _check(rc: int, where: str):
    if rc != 0:
        raise DynError(rc, where)


def _host(a, dt) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dt)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _dp(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


class Profile:
    """Owner of a dyn_profile handle."""

    def __init__(self, handle: int, shape):
        self.handle = handle
        self.n_class, self.n_tp, self.n_f, self.n_rho = shape

    def free(self):
        if self.handle:
            _lib.dyn_profile_free(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def dyn_profile_load(profile: Dict[str, np.ndarray], stream=None) -> Profile:
    tp = _host(profile["tp"], np.int32); fg = _host(profile["f_mhz"], np.float64)
    rg = _host(profile["rho"], np.float64)
    pf = _host(profile["prefill_ms_per_tok"], np.float64); tb = _host(profile["tbt_ms"], np.float64)
    pw = _host(profile["power_w"], np.float64); ml = _host(profile["max_load_tps"], np.float64)
    G = pf.shape[0] if pf.ndim == 4 else 0
    want = (G, tp.size, fg.size, rg.size)
    if pf.shape != want or tb.shape != want or pw.shape != want or ml.shape != want[:3]:
        raise ValueError(f"profile tables must have shape {want} / {want[:3]}")
    d = _ProfileDesc(G, tp.size, _hp(tp), fg.size, _hp(fg), rg.size, _hp(rg), _hp(pf), _hp(tb), _hp(pw), _hp(ml))
    h = _vp()
    _check(_lib.dyn_profile_load(C.byref(d), _stream(stream), C.byref(h)), "dyn_profile_load")
    return Profile(h.value, want)


def dyn_profile_free(p: Profile):
    p.free()


def dyn_trace_ingest_workspace(n_req: int, n_window: int, n_class: int) -> int:
    return int(_lib.dyn_trace_ingest_workspace(n_req, n_window, n_class))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)   # torch allocations are 512 B aligned


def dyn_trace_ingest(t_s: torch.Tensor, in_tok: torch.Tensor, out_tok: torch.Tensor,
                     model: Optional[torch.Tensor], edges: Dict[str, np.ndarray], n_window: int, window_s: float,
                     workspace: Optional[torch.Tensor] = None, stream=None):
    """Returns (in_sorted, out_sorted, cell_off, workspace)."""
    ie = _host(edges["in_edge"], np.int32); oe = _host(edges["out_edge"], np.int32)
    if ie.ndim != 2 or oe.ndim != 2 or ie.shape[0] != oe.shape[0]:
        raise ValueError("edges must be [n_model][bins-1]")
    n_model, bi, bo = ie.shape[0], ie.shape[1] + 1, oe.shape[1] + 1
    G = n_model * bi * bo
    n = t_s.numel()
    dev = t_s.device
    e = _ClassEdges(n_model, bi, bo, _hp(ie), _hp(oe))
    need = dyn_trace_ingest_workspace(n, n_window, G)
    if workspace is None:
        workspace = _workspace(need, dev)
    ins = torch.empty(n, dtype=torch.int32, device=dev); outs = torch.empty(n, dtype=torch.int32, device=dev)
    off = torch.empty(n_window * G + 1, dtype=torch.int64, device=dev)
    _check(_lib.dyn_trace_ingest(_dp(t_s, torch.float64, "t_s"), _dp(in_tok, torch.int32, "in_tok"),
                                 _dp(out_tok, torch.int32, "out_tok"), _dp(model, torch.int32, "model"), n,
                                 C.byref(e), n_window, float(window_s), _dp(ins), _dp(outs), _dp(off),
                                 _dp(workspace), workspace.numel(), _stream(stream)), "dyn_trace_ingest")
    return ins, outs, off, workspace


def dyn_eval_space_workspace(n_window: int, n_class: int, n_config: int) -> int:
    return int(_lib.dyn_eval_space_workspace(n_window, n_class, n_config))


def _configs(configs: Dict[str, np.ndarray]):
    n = _host(configs["n_inst"], np.int32); t = _host(configs["tp_index"], np.int32)
    f = _host(configs["f_mhz"], np.float64)
    K = n.size
    arr = (_Config * K)()
    for k in range(K):
        arr[k].n_inst = int(n[k]); arr[k].tp_index = int(t[k]); arr[k].f_mhz = float(f[k])
    return arr, K


def _objective(slos: Dict[str, np.ndarray], pct: Sequence[int], gpu_budget, idle_cost_weight: float):
    st = _host(slos["slo_ttft_ms"], np.float64); sb = _host(slos["slo_tbt_ms"], np.float64)
    bud = None if gpu_budget is None else _host(gpu_budget, np.int32)
    o = _Objective(_hp(st), _hp(sb), int(pct[0]), int(pct[1]), _hp(bud), float(idle_cost_weight))
    return o, (st, sb, bud)      # keep the arrays alive


class Plan:
    """Marshalled candidate list and objective, reusable across calls (host side only)."""

    def __init__(self, configs, slos, pct=(99, 100), gpu_budget=None, idle_cost_weight=0.0):
        self.cfg, self.K = _configs(configs)
        self.obj, self._keep = _objective(slos, pct, gpu_budget, idle_cost_weight)
        self.n_class = self._keep[0].size


__all__.append("Plan")


def _space_tensors(cells, K, dev):
    return {"energy_j": torch.empty((cells, K), dtype=torch.float64, device=dev),
            "p99_ttft_ms": torch.empty((cells, K), dtype=torch.float64, device=dev),
            "p99_tbt_ms": torch.empty((cells, K), dtype=torch.float64, device=dev),
            "flags": torch.empty((cells, K), dtype=torch.uint8, device=dev)}


def _selection_tensors(cells, n_window, dev):
    return {"sel": torch.empty(cells, dtype=torch.int32, device=dev),
            "sel_energy_j": torch.empty(cells, dtype=torch.float64, device=dev),
            "sel_cost": torch.empty(cells, dtype=torch.float64, device=dev),
            "window_energy_j": torch.empty(n_window, dtype=torch.float64, device=dev),
            "window_infeasible": torch.empty(n_window, dtype=torch.int32, device=dev)}


def _selection_struct(out):
    return _Selection(_dp(out["sel"], torch.int32), _dp(out["sel_energy_j"], torch.float64),
                      _dp(out["sel_cost"], torch.float64), _dp(out["window_energy_j"], torch.float64),
                      _dp(out["window_infeasible"], torch.int32))


def _eval_args(profile, in_tok, out_tok, cell_off, n_window, window_s, plan, out, workspace):
    G, K = profile.n_class, plan.K
    if plan.n_class != G:
        raise ValueError("SLO arrays must have one entry per class")
    cells = n_window * G
    if cell_off.numel() != cells + 1:
        raise ValueError("cell_off must have n_window*G + 1 entries")
    dev = cell_off.device
    if out is None:
        out = _space_tensors(cells, K, dev)
    if workspace is None:
        workspace = _workspace(dyn_eval_space_workspace(n_window, G, K), dev)
    tv = _TraceView(in_tok.numel(), n_window, float(window_s), _dp(in_tok, torch.int32, "in_tok"),
                    _dp(out_tok, torch.int32, "out_tok"), _dp(cell_off, torch.int64, "cell_off"))
    sp = _Space(_dp(out["energy_j"], torch.float64), _dp(out["p99_ttft_ms"], torch.float64),
                _dp(out["p99_tbt_ms"], torch.float64), _dp(out["flags"], torch.uint8))
    for v in out.values():
        if v.numel() != cells * K:
            raise ValueError("space tensors must hold n_window*G*K entries")
    return tv, sp, out, workspace, cells, K


def dyn_eval_space(profile: Profile, in_tok: torch.Tensor, out_tok: torch.Tensor, cell_off: torch.Tensor,
                   n_window: int, window_s: float, plan: Plan, out: Optional[Dict[str, torch.Tensor]] = None,
                   workspace: Optional[torch.Tensor] = None, stream=None):
    """Returns (space dict of [cells, K] tensors, workspace)."""
    tv, sp, out, workspace, cells, K = _eval_args(profile, in_tok, out_tok, cell_off, n_window, window_s, plan, out,
                                                  workspace)
    _check(_lib.dyn_eval_space(profile.handle, C.byref(tv), plan.cfg, K, C.byref(plan.obj), C.byref(sp),
                               _dp(workspace), workspace.numel(), _stream(stream)), "dyn_eval_space")
    return out, workspace


def dyn_eval_select(profile: Profile, in_tok: torch.Tensor, out_tok: torch.Tensor, cell_off: torch.Tensor,
                    n_window: int, window_s: float, plan: Plan, out: Optional[Dict[str, torch.Tensor]] = None,
                    sel: Optional[Dict[str, torch.Tensor]] = None, workspace: Optional[torch.Tensor] = None,
                    stream=None):
    """Evaluation and selection in one pass.  Returns (space, selection, workspace)."""
    tv, sp, out, workspace, cells, K = _eval_args(profile, in_tok, out_tok, cell_off, n_window, window_s, plan, out,
                                                  workspace)
    if sel is None:
        sel = _selection_tensors(cells, n_window, cell_off.device)
    se = _selection_struct(sel)
    _check(_lib.dyn_eval_select(profile.handle, C.byref(tv), plan.cfg, K, C.byref(plan.obj), C.byref(sp), C.byref(se),
                                _dp(workspace), workspace.numel(), _stream(stream)), "dyn_eval_select")
    return out, sel, workspace


def dyn_eval_tune(profile: Profile, in_tok: torch.Tensor, out_tok: torch.Tensor, cell_off: torch.Tensor, n_window: int,
                  window_s: float, plan: Plan, out: Optional[Dict[str, torch.Tensor]] = None,
                  sel: Optional[Dict[str, torch.Tensor]] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> int:
    """Times the evaluation for several block shapes and keeps the fastest in the profile handle.  Returns the chosen
    number of windows per block."""
    tv, sp, out, workspace, cells, K = _eval_args(profile, in_tok, out_tok, cell_off, n_window, window_s, plan, out,
                                                  workspace)
    if sel is None:
        sel = _selection_tensors(cells, n_window, cell_off.device)
    se = _selection_struct(sel)
    chosen = _i32(0)
    _check(_lib.dyn_eval_tune(profile.handle, C.byref(tv), plan.cfg, K, C.byref(plan.obj), C.byref(sp), C.byref(se),
                              _dp(workspace), workspace.numel(), _stream(stream), C.byref(chosen)), "dyn_eval_tune")
    return int(chosen.value)


def dyn_eval_select_static(profile: Profile, in_tok: torch.Tensor, out_tok: torch.Tensor, cell_off: torch.Tensor,
                           n_window: int, window_s: float, plan: Plan, out: Dict[str, torch.Tensor],
                           sel: Dict[str, torch.Tensor], status: Optional[torch.Tensor] = None, stream=None):
    """dyn_eval_select on the library's fixed workspace: nothing is allocated, here or in the library, so `out` and
    `sel` (and `status`, one int32/uint32 word on the device, optional) are the caller's."""
    if out is None or sel is None:
        raise ValueError("dyn_eval_select_static allocates nothing: pass the output tensors")
    dummy = cell_off                      # any device tensor: _eval_args allocates a workspace only when given None
    tv, sp, out, _, cells, K = _eval_args(profile, in_tok, out_tok, cell_off, n_window, window_s, plan, out, dummy)
    se = _selection_struct(sel)
    if status is not None and (status.numel() != 1 or status.element_size() != 4):
        raise ValueError("status must be one 32-bit word")
    _check(_lib.dyn_eval_select_static(profile.handle, C.byref(tv), plan.cfg, K, C.byref(plan.obj), C.byref(sp),
                                       C.byref(se), _dp(status), _stream(stream)), "dyn_eval_select_static")
    return out, sel


def dyn_eval_ticks_workspace(n_req: int, n_window: int, n_tick: int, n_class: int, n_config: int) -> int:
    return int(_lib.dyn_eval_ticks_workspace(n_req, n_window, n_tick, n_class, n_config))


def dyn_eval_select_ticks(profile: Profile, in_tok: torch.Tensor, out_tok: torch.Tensor, cell_off: torch.Tensor,
                          n_window: int, n_tick: int, tick_s: float, plan: Plan,
                          out: Optional[Dict[str, torch.Tensor]] = None, sel: Optional[Dict[str, torch.Tensor]] = None,
                          workspace: Optional[torch.Tensor] = None, stream=None):
    """Tick-level evaluation and selection.  The trace arrays are those of dyn_trace_ingest with
    n_window*n_tick windows of tick_s seconds; outputs are per coarse cell.  Returns (space, selection, workspace)."""
    G, K = profile.n_class, plan.K
    if plan.n_class != G:
        raise ValueError("SLO arrays must have one entry per class")
    cells = n_window * G
    if cell_off.numel() != cells * n_tick + 1:
        raise ValueError("cell_off must have n_window*n_tick*G + 1 entries")
    dev = cell_off.device
    if out is None:
        out = _space_tensors(cells, K, dev)
    if sel is None:
        sel = _selection_tensors(cells, n_window, dev)
    if workspace is None:
        nbytes = dyn_eval_ticks_workspace(in_tok.numel(), n_window, n_tick, G, K)
        if nbytes == 0:
            raise DynError(-2, "dyn_eval_ticks_workspace")
        workspace = _workspace(nbytes, dev)
    for v in out.values():
        if v.numel() != cells * K:
            raise ValueError("space tensors must hold n_window*G*K entries")
    tv = _TraceView(in_tok.numel(), n_window * n_tick, float(tick_s), _dp(in_tok, torch.int32, "in_tok"),
                    _dp(out_tok, torch.int32, "out_tok"), _dp(cell_off, torch.int64, "cell_off"))
    sp = _Space(_dp(out["energy_j"], torch.float64), _dp(out["p99_ttft_ms"], torch.float64),
                _dp(out["p99_tbt_ms"], torch.float64), _dp(out["flags"], torch.uint8))
    se = _selection_struct(sel)
    _check(_lib.dyn_eval_select_ticks(profile.handle, C.byref(tv), n_tick, plan.cfg, K, C.byref(plan.obj), C.byref(sp),
                                      C.byref(se), _dp(workspace), workspace.numel(), _stream(stream)),
           "dyn_eval_select_ticks")
    return out, sel, workspace


class MixedPlan:
    """Marshalled mixed-pool search space (shares, instances per type) and objective (host side only)."""

    def __init__(self, n_share, n_max, slos, pct=(99, 100), gpu_budget=None):
        self._n_max = _host(n_max, np.int32)
        self.space = _MixedSpace(int(n_share), _hp(self._n_max))
        self.obj, self._keep = _objective(slos, pct, gpu_budget, 0.0)
        self.n_class = self._keep[0].size
        self.n_tp = self._n_max.size


def dyn_mixed_workspace(profile: Profile, n_window: int, plan: MixedPlan) -> int:
    return int(_lib.dyn_mixed_workspace(profile.handle, n_window, C.byref(plan.space)))


def dyn_eval_select_mixed(profile: Profile, in_tok: torch.Tensor, out_tok: torch.Tensor, cell_off: torch.Tensor,
                          n_window: int, window_s: float, plan: MixedPlan,
                          out: Optional[Dict[str, torch.Tensor]] = None, workspace: Optional[torch.Tensor] = None,
                          stream=None):
    """Least-energy assignment of instances, frequencies and load shares per cell.  Returns (selection, workspace)."""
    G, T = profile.n_class, profile.n_tp
    if plan.n_class != G or plan.n_tp != T:
        raise ValueError("SLO arrays need one entry per class and n_max one per TP degree")
    cells = n_window * G
    if cell_off.numel() != cells + 1:
        raise ValueError("cell_off must have n_window*G + 1 entries")
    dev = cell_off.device
    if out is None:
        out = {"energy_j": torch.empty(cells, dtype=torch.float64, device=dev),
               "n_inst": torch.empty((cells, T), dtype=torch.int32, device=dev),
               "f_index": torch.empty((cells, T), dtype=torch.int32, device=dev),
               "share": torch.empty((cells, T), dtype=torch.int32, device=dev),
               "window_energy_j": torch.empty(n_window, dtype=torch.float64, device=dev),
               "window_infeasible": torch.empty(n_window, dtype=torch.int32, device=dev)}
    if workspace is None:
        nbytes = dyn_mixed_workspace(profile, n_window, plan)
        if nbytes == 0:
            raise DynError(-2, "dyn_mixed_workspace")
        workspace = _workspace(nbytes, dev)
    tv = _TraceView(in_tok.numel(), n_window, float(window_s), _dp(in_tok, torch.int32, "in_tok"),
                    _dp(out_tok, torch.int32, "out_tok"), _dp(cell_off, torch.int64, "cell_off"))
    se = _MixedSelection(_dp(out["energy_j"], torch.float64), _dp(out["n_inst"], torch.int32),
                         _dp(out["f_index"], torch.int32), _dp(out["share"], torch.int32),
                         _dp(out["window_energy_j"], torch.float64), _dp(out["window_infeasible"], torch.int32))
    for k in ("n_inst", "f_index", "share"):
        if out[k].numel() != cells * T:
            raise ValueError("selection tensors must hold n_window*G*n_tp entries")
    _check(_lib.dyn_eval_select_mixed(profile.handle, C.byref(tv), C.byref(plan.space), C.byref(plan.obj), C.byref(se),
                                      _dp(workspace), workspace.numel(), _stream(stream)), "dyn_eval_select_mixed")
    return out, workspace


def dyn_select_path_workspace(n_window: int, n_class: int, n_config: int, n_layout: int) -> int:
    return int(_lib.dyn_select_path_workspace(n_window, n_class, n_config, n_layout))


def dyn_select_path(profile: Profile, space: Dict[str, torch.Tensor], n_window: int, window_s: float, plan: Plan,
                    layout, transition_j, out: Optional[Dict[str, torch.Tensor]] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None):
    """Selection with transition overheads between consecutive windows.  Returns (selection, workspace)."""
    G, K = profile.n_class, plan.K
    cells = n_window * G
    dev = space["energy_j"].device
    if space["energy_j"].numel() != cells * K or space["flags"].numel() != cells * K:
        raise ValueError("space tensors must hold n_window*G*K entries")
    lay = _host(layout, np.int32); tr = _host(transition_j, np.float64)
    if lay.size != K or tr.ndim != 2 or tr.shape[0] != tr.shape[1]:
        raise ValueError("layout needs K entries and transition_j must be square")
    if out is None:
        out = {"sel": torch.empty(cells, dtype=torch.int32, device=dev),
               "sel_energy_j": torch.empty(cells, dtype=torch.float64, device=dev),
               "path_cost": torch.empty(G, dtype=torch.float64, device=dev),
               "window_energy_j": torch.empty(n_window, dtype=torch.float64, device=dev),
               "window_infeasible": torch.empty(n_window, dtype=torch.int32, device=dev)}
    if workspace is None:
        workspace = _workspace(max(256, dyn_select_path_workspace(n_window, G, K, tr.shape[0])), dev)
    sp = _Space(_dp(space["energy_j"], torch.float64), _dp(space.get("p99_ttft_ms")), _dp(space.get("p99_tbt_ms")),
                _dp(space["flags"], torch.uint8))
    tt = _Transitions(int(tr.shape[0]), _hp(lay), _hp(tr))
    se = _PathSelection(_dp(out["sel"], torch.int32), _dp(out["sel_energy_j"], torch.float64),
                        _dp(out["path_cost"], torch.float64), _dp(out["window_energy_j"], torch.float64),
                        _dp(out["window_infeasible"], torch.int32))
    _check(_lib.dyn_select_path(profile.handle, C.byref(sp), plan.cfg, K, C.byref(plan.obj), C.byref(tt), n_window,
                                float(window_s), C.byref(se), _dp(workspace), workspace.numel(), _stream(stream)),
           "dyn_select_path")
    return out, workspace


def dyn_account_workspace(n_window: int) -> int:
    return int(_lib.dyn_account_workspace(n_window))


def dyn_account(profile: Profile, sel: torch.Tensor, window_energy_j: torch.Tensor, plan: Plan, n_window: int,
                window_s: float, gpu_hour_price: float, kwh_price: float, carbon_g_per_kwh: torch.Tensor,
                gpus_per_server: int = 8, stream=None):
    """Cost and carbon of a selection.  Returns (dict of per-window tensors + totals[5], workspace)."""
    dev = sel.device
    if sel.numel() != n_window * profile.n_class or window_energy_j.numel() != n_window or carbon_g_per_kwh.numel() != n_window:
        raise ValueError("sel needs n_window*G entries, window_energy_j and carbon_g_per_kwh n_window")
    out = {"gpus": torch.empty(n_window, dtype=torch.int64, device=dev),
           "gpu_cost": torch.empty(n_window, dtype=torch.float64, device=dev),
           "energy_cost": torch.empty(n_window, dtype=torch.float64, device=dev),
           "carbon_g": torch.empty(n_window, dtype=torch.float64, device=dev),
           "totals": torch.empty(5, dtype=torch.float64, device=dev)}
    ws = _workspace(dyn_account_workspace(n_window), dev)
    rates = _Rates(float(gpu_hour_price), float(kwh_price), _dp(carbon_g_per_kwh, torch.float64), int(gpus_per_server))
    acc = _Accounting(_dp(out["gpus"], torch.int64), _dp(out["gpu_cost"], torch.float64), _dp(out["energy_cost"], torch.float64),
                      _dp(out["carbon_g"], torch.float64), _dp(out["totals"], torch.float64))
    _check(_lib.dyn_account(profile.handle, _dp(sel, torch.int32), _dp(window_energy_j, torch.float64), plan.cfg, plan.K,
                            n_window, float(window_s), C.byref(rates), C.byref(acc), _dp(ws), ws.numel(), _stream(stream)),
           "dyn_account")
    return out, ws


def dyn_hierarchy_workspace(n_window: int, n_tick: int, n_class: int, n_layout: int) -> int:
    return int(_lib.dyn_hierarchy_workspace(n_window, n_tick, n_class, n_layout))


def dyn_hierarchy(profile: Profile, coarse, fine, n_window: int, n_tick: int, tick_s: float, epoch_windows: int,
                  tp_ref_index: int, f_ref_index: int, gpus_per_node: int, lay_n, lay_tp_index, slos, pct=(99, 100),
                  out: Optional[Dict[str, torch.Tensor]] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                  transition_j=None, spill: bool = False):
    """The three controllers top down.  `coarse` / `fine` are (in_tok, out_tok, cell_off) tensor triples of the trace
    sorted by window and by tick.  `transition_j` ([n_layout][n_layout] joules, host) makes the shard controller weigh
    re-sharding overheads (out["path_cost"] is then filled); `spill` applies the fragmentation rule (out["keep"] is
    then filled).  Returns (dict of output tensors, workspace)."""
    G = profile.n_class
    cells = n_window * G
    ci, co_, coff = coarse
    fi, fo_, foff = fine
    if coff.numel() != cells + 1 or foff.numel() != cells * n_tick + 1:
        raise ValueError("cell_off sizes do not match n_window, n_tick and the classes")
    dev = coff.device
    ln = _host(lay_n, np.int32); lt = _host(lay_tp_index, np.int32)
    tj = None
    if transition_j is not None:
        tj = _host(transition_j, np.float64)
        if tj.shape != (ln.size, ln.size):
            raise ValueError("transition_j must be [n_layout][n_layout]")
    n_epoch = -(-n_window // max(int(epoch_windows), 1))      # the library rejects epoch_windows < 1
    out = out or {"nodes": torch.empty((n_epoch, G), dtype=torch.int32, device=dev),
           "layout_sel": torch.empty(cells, dtype=torch.int32, device=dev),
           "f_sel": torch.empty((n_window * n_tick, G), dtype=torch.int32, device=dev),
           "energy_j": torch.empty(cells, dtype=torch.float64, device=dev),
           "violations": torch.empty(cells, dtype=torch.int32, device=dev),
           "window_energy_j": torch.empty(n_window, dtype=torch.float64, device=dev),
           "window_infeasible": torch.empty(n_window, dtype=torch.int32, device=dev)}
    if tj is not None and "path_cost" not in out:
        out["path_cost"] = torch.empty(G, dtype=torch.float64, device=dev)
    if spill and "keep" not in out:
        out["keep"] = torch.empty((n_epoch, G), dtype=torch.float64, device=dev)
    want = {"nodes": (n_epoch * G, torch.int32), "layout_sel": (cells, torch.int32), "f_sel": (cells * n_tick, torch.int32),
            "energy_j": (cells, torch.float64), "violations": (cells, torch.int32),
            "window_energy_j": (n_window, torch.float64), "window_infeasible": (n_window, torch.int32)}
    if tj is not None:
        want["path_cost"] = (G, torch.float64)
    if spill:
        want["keep"] = (n_epoch * G, torch.float64)
    for k, (n, dt) in want.items():
        if out[k].numel() != n or out[k].dtype != dt:
            raise ValueError(f"out[{k!r}] must hold {n} elements of {dt}")
    if workspace is None:
        workspace = _workspace(dyn_hierarchy_workspace(n_window, n_tick, G, ln.size), dev)
    obj, keep = _objective(slos, pct, None, 0.0)
    tc = _TraceView(ci.numel(), n_window, float(tick_s) * n_tick, _dp(ci, torch.int32), _dp(co_, torch.int32), _dp(coff, torch.int64))
    tf = _TraceView(fi.numel(), n_window * n_tick, float(tick_s), _dp(fi, torch.int32), _dp(fo_, torch.int32), _dp(foff, torch.int64))
    ctl = _Controllers(int(epoch_windows), int(tp_ref_index), int(f_ref_index), int(gpus_per_node), int(ln.size),
                       1 if spill else 0, _hp(ln), _hp(lt), _hp(tj))
    ho = _HierarchyOut(*[_dp(out[k]) for k in ("nodes", "layout_sel", "f_sel", "energy_j", "violations", "window_energy_j",
                                               "window_infeasible")], _dp(out.get("path_cost")), _dp(out.get("keep") if spill else None))
    _check(_lib.dyn_hierarchy(profile.handle, C.byref(tc), C.byref(tf), n_tick, C.byref(ctl), C.byref(obj), C.byref(ho),
                              _dp(workspace), workspace.numel(), _stream(stream)), "dyn_hierarchy")
    return out, workspace


def dyn_cell_stats(workspace: torch.Tensor, n_window: int, n_class: int, stream=None):
    """Returns (tok_in, tok_out, in_p99) of the last dyn_eval_space on `workspace`."""
    cells = n_window * n_class
    dev = workspace.device
    ti = torch.empty(cells, dtype=torch.int64, device=dev); to = torch.empty(cells, dtype=torch.int64, device=dev)
    p = torch.empty(cells, dtype=torch.int32, device=dev)
    _check(_lib.dyn_cell_stats(_dp(workspace), workspace.numel(), n_window, n_class, _dp(ti), _dp(to), _dp(p),
                               _stream(stream)), "dyn_cell_stats")
    return ti, to, p


def dyn_workspace_status(workspace: torch.Tensor, stream=None) -> int:
    st = C.c_uint32(0)
    _check(_lib.dyn_workspace_status(_dp(workspace), _stream(stream), C.byref(st)), "dyn_workspace_status")
    return int(st.value)


def dyn_select_config(profile: Profile, space: Dict[str, torch.Tensor], n_window: int, window_s: float, plan: Plan,
                      out: Optional[Dict[str, torch.Tensor]] = None, stream=None) -> Dict[str, torch.Tensor]:
    G, K = profile.n_class, plan.K
    cells = n_window * G
    dev = space["energy_j"].device
    if space["energy_j"].numel() != cells * K or space["flags"].numel() != cells * K:
        raise ValueError("space tensors must hold n_window*G*K entries")
    if out is None:
        out = _selection_tensors(cells, n_window, dev)
    sp = _Space(_dp(space["energy_j"], torch.float64), _dp(space.get("p99_ttft_ms")), _dp(space.get("p99_tbt_ms")),
                _dp(space["flags"], torch.uint8))
    se = _selection_struct(out)
    _check(_lib.dyn_select_config(profile.handle, C.byref(sp), plan.cfg, K, C.byref(plan.obj), n_window,
                                  float(window_s), C.byref(se), _stream(stream)), "dyn_select_config")
    return out
