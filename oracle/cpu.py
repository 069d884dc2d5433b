"""ctypes front end of the CPU oracle (oracle/dyn_oracle.cpp).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's CPU-baseline leg
may import this.  Argument marshalling only; all arithmetic is in the C++ file.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

from .build_oracle import build

_lib = None

_P = C.c_void_p


def _load():
    global _lib
    if _lib is None:
        # DYNORACLE_LIB: another build of the same source (the sanitizer build of the test-suite)
        _lib = C.CDLL(os.environ.get("DYNORACLE_LIB") or build())
        _lib.dynoracle_ingest.restype = C.c_int
        _lib.dynoracle_eval.restype = C.c_int
        _lib.dynoracle_window_totals.restype = C.c_int
        _lib.dynoracle_select_row.restype = C.c_int
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_P)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def ingest(trace: Dict[str, np.ndarray], edges: Dict[str, np.ndarray], n_window: int,
           window_s: float) -> Dict[str, np.ndarray]:
    """Raw trace -> cell-sorted in/out arrays and cell offsets."""
    lib = _load()
    t = _c(trace["t_s"], np.float64); i = _c(trace["in_tok"], np.int32)
    o = _c(trace["out_tok"], np.int32); mdl = _c(trace["model"], np.int32)
    ie = _c(edges["in_edge"], np.int32); oe = _c(edges["out_edge"], np.int32)
    n_model, bi, bo = ie.shape[0], ie.shape[1] + 1, oe.shape[1] + 1
    n = t.size
    cells = n_window * n_model * bi * bo
    ins = np.empty(n, np.int32); outs = np.empty(n, np.int32)
    off = np.empty(cells + 1, np.int64)
    rc = lib.dynoracle_ingest(_ptr(t), _ptr(i), _ptr(o), _ptr(mdl), C.c_int64(n), C.c_int32(n_model),
                              C.c_int32(bi), C.c_int32(bo), _ptr(ie), _ptr(oe), C.c_int32(n_window),
                              C.c_double(window_s), _ptr(ins), _ptr(outs), _ptr(off))
    if rc != 0:
        raise ValueError(f"dynoracle_ingest failed: {rc}")
    return {"in_tok": ins, "out_tok": outs, "cell_off": off}


def evaluate(profile: Dict[str, np.ndarray], sorted_trace: Dict[str, np.ndarray], n_window: int,
             window_s: float, configs: Dict[str, np.ndarray], slos: Dict[str, np.ndarray],
             pct=(99, 100), gpu_budget: Optional[np.ndarray] = None, idle_cost_weight: float = 0.0,
             cell_ids: Optional[np.ndarray] = None, full_sort: bool = False,
             want_space: bool = True) -> Dict[str, np.ndarray]:
    """Evaluates the listed cells (all when cell_ids is None) under every configuration."""
    lib = _load()
    tp = _c(profile["tp"], np.int32); fg = _c(profile["f_mhz"], np.float64)
    rg = _c(profile["rho"], np.float64)
    PF = _c(profile["prefill_ms_per_tok"], np.float64); TB = _c(profile["tbt_ms"], np.float64)
    PW = _c(profile["power_w"], np.float64); ML = _c(profile["max_load_tps"], np.float64)
    G = PF.shape[0]
    assert PF.shape == (G, tp.size, fg.size, rg.size) == TB.shape == PW.shape
    assert ML.shape == (G, tp.size, fg.size)
    ins = _c(sorted_trace["in_tok"], np.int32); outs = _c(sorted_trace["out_tok"], np.int32)
    off = _c(sorted_trace["cell_off"], np.int64)
    cells = n_window * G
    assert off.size == cells + 1
    cn = _c(configs["n_inst"], np.int32); ct = _c(configs["tp_index"], np.int32)
    cf = _c(configs["f_mhz"], np.float64)
    K = cn.size
    st = _c(slos["slo_ttft_ms"], np.float64); sb = _c(slos["slo_tbt_ms"], np.float64)
    assert st.size == G and sb.size == G
    bud = None if gpu_budget is None else _c(gpu_budget, np.int32)
    ids = None if cell_ids is None else _c(cell_ids, np.int64)
    ns = cells if ids is None else ids.size
    r: Dict[str, np.ndarray] = {}
    if want_space:
        r["energy_j"] = np.empty((ns, K)); r["p99_ttft_ms"] = np.empty((ns, K))
        r["p99_tbt_ms"] = np.empty((ns, K)); r["flags"] = np.empty((ns, K), np.uint8)
        r["cost"] = np.empty((ns, K))
    r["m"] = np.empty(ns, np.int64); r["tin"] = np.empty(ns, np.int64); r["tout"] = np.empty(ns, np.int64)
    r["in_p99"] = np.empty(ns, np.int32); r["sel"] = np.empty(ns, np.int32)
    r["sel_energy_j"] = np.empty(ns); r["sel_cost"] = np.empty(ns)
    rc = lib.dynoracle_eval(
        C.c_int32(G), C.c_int32(tp.size), _ptr(tp), C.c_int32(fg.size), _ptr(fg), C.c_int32(rg.size),
        _ptr(rg), _ptr(PF), _ptr(TB), _ptr(PW), _ptr(ML),
        C.c_int64(ins.size), C.c_int32(n_window), C.c_double(window_s), _ptr(ins), _ptr(outs), _ptr(off),
        C.c_int32(K), _ptr(cn), _ptr(ct), _ptr(cf),
        _ptr(st), _ptr(sb), C.c_int32(pct[0]), C.c_int32(pct[1]), _ptr(bud), C.c_double(idle_cost_weight),
        C.c_int64(ns), _ptr(ids), C.c_int32(1 if full_sort else 0),
        _ptr(r.get("energy_j")), _ptr(r.get("p99_ttft_ms")), _ptr(r.get("p99_tbt_ms")), _ptr(r.get("flags")),
        _ptr(r.get("cost")), _ptr(r["m"]), _ptr(r["tin"]), _ptr(r["tout"]), _ptr(r["in_p99"]),
        _ptr(r["sel"]), _ptr(r["sel_energy_j"]), _ptr(r["sel_cost"]))
    if rc != 0:
        raise ValueError(f"dynoracle_eval failed: {rc}")
    return r


def evaluate_parallel(profile, sorted_trace, n_window, window_s, configs, slos, pct=(99, 100), gpu_budget=None,
                      idle_cost_weight=0.0, threads: Optional[int] = None, windows_per_task: int = 0,
                      want_space: bool = False) -> Dict[str, np.ndarray]:
    """evaluate() over every cell with the windows dealt to `threads` host threads (cells are independent; each
    task is one plain call of the single-threaded oracle on a run of windows, and ctypes releases the
    interpreter lock for its duration).  Same outputs as evaluate(), in cell order, plus "threads"."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    G = np.asarray(profile["prefill_ms_per_tok"]).shape[0]
    threads = threads or min(32, os.cpu_count() or 1)
    per = windows_per_task or max(1, n_window // (threads * 8))
    tasks = [(w0, min(w0 + per, n_window)) for w0 in range(0, n_window, per)]

    def run(t):
        ids = np.arange(t[0] * G, t[1] * G, dtype=np.int64)
        return evaluate(profile, sorted_trace, n_window, window_s, configs, slos, pct, gpu_budget, idle_cost_weight,
                        cell_ids=ids, want_space=want_space)

    _load()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(run, tasks))
    r = {k: np.concatenate([p_[k] for p_ in parts]) for k in parts[0]}
    r["threads"] = threads
    return r


def evaluate_ticks(profile: Dict[str, np.ndarray], fine_trace: Dict[str, np.ndarray], n_window: int, n_tick: int,
                   tick_s: float, configs: Dict[str, np.ndarray], slos: Dict[str, np.ndarray], pct=(99, 100),
                   gpu_budget: Optional[np.ndarray] = None, idle_cost_weight: float = 0.0) -> Dict[str, np.ndarray]:
    """Tick-level evaluation; `fine_trace` is sorted by (w*n_tick + tick)*G + class."""
    lib = _load()
    lib.dynoracle_eval_ticks.restype = C.c_int
    tp = _c(profile["tp"], np.int32); fg = _c(profile["f_mhz"], np.float64)
    rg = _c(profile["rho"], np.float64)
    PF = _c(profile["prefill_ms_per_tok"], np.float64); TB = _c(profile["tbt_ms"], np.float64)
    PW = _c(profile["power_w"], np.float64); ML = _c(profile["max_load_tps"], np.float64)
    G = PF.shape[0]
    ins = _c(fine_trace["in_tok"], np.int32); outs = _c(fine_trace["out_tok"], np.int32)
    off = _c(fine_trace["cell_off"], np.int64)
    assert off.size == n_window * n_tick * G + 1
    cn = _c(configs["n_inst"], np.int32); ct = _c(configs["tp_index"], np.int32)
    cf = _c(configs["f_mhz"], np.float64)
    K = cn.size
    st = _c(slos["slo_ttft_ms"], np.float64); sb = _c(slos["slo_tbt_ms"], np.float64)
    bud = None if gpu_budget is None else _c(gpu_budget, np.int32)
    cells = n_window * G
    r = {"energy_j": np.empty((cells, K)), "p99_ttft_ms": np.empty((cells, K)), "p99_tbt_ms": np.empty((cells, K)),
         "flags": np.empty((cells, K), np.uint8), "cost": np.empty((cells, K)), "m": np.empty(cells, np.int64),
         "sel": np.empty(cells, np.int32), "sel_energy_j": np.empty(cells), "sel_cost": np.empty(cells)}
    rc = lib.dynoracle_eval_ticks(
        C.c_int32(G), C.c_int32(tp.size), _ptr(tp), C.c_int32(fg.size), _ptr(fg), C.c_int32(rg.size), _ptr(rg),
        _ptr(PF), _ptr(TB), _ptr(PW), _ptr(ML),
        C.c_int64(ins.size), C.c_int32(n_window), C.c_int32(n_tick), C.c_double(tick_s), _ptr(ins), _ptr(outs),
        _ptr(off), C.c_int32(K), _ptr(cn), _ptr(ct), _ptr(cf), _ptr(st), _ptr(sb), C.c_int32(pct[0]),
        C.c_int32(pct[1]), _ptr(bud), C.c_double(idle_cost_weight),
        _ptr(r["energy_j"]), _ptr(r["p99_ttft_ms"]), _ptr(r["p99_tbt_ms"]), _ptr(r["flags"]), _ptr(r["cost"]),
        _ptr(r["m"]), _ptr(r["sel"]), _ptr(r["sel_energy_j"]), _ptr(r["sel_cost"]))
    if rc != 0:
        raise ValueError(f"dynoracle_eval_ticks failed: {rc}")
    return r


def mixed(profile: Dict[str, np.ndarray], sorted_trace: Dict[str, np.ndarray], n_window: int, window_s: float,
          n_share: int, n_max, slos: Dict[str, np.ndarray], pct=(99, 100),
          gpu_budget: Optional[np.ndarray] = None, want_types: bool = False) -> Dict[str, np.ndarray]:
    """Mixed pools (Eq. 1 in full): least-energy assignment of instances, frequencies and load shares per cell."""
    lib = _load()
    lib.dynoracle_mixed.restype = C.c_int
    tp = _c(profile["tp"], np.int32); fg = _c(profile["f_mhz"], np.float64)
    rg = _c(profile["rho"], np.float64)
    PF = _c(profile["prefill_ms_per_tok"], np.float64); TB = _c(profile["tbt_ms"], np.float64)
    PW = _c(profile["power_w"], np.float64); ML = _c(profile["max_load_tps"], np.float64)
    G = PF.shape[0]
    ins = _c(sorted_trace["in_tok"], np.int32); outs = _c(sorted_trace["out_tok"], np.int32)
    off = _c(sorted_trace["cell_off"], np.int64)
    assert off.size == n_window * G + 1
    nm = _c(n_max, np.int32)
    assert nm.size == tp.size
    st = _c(slos["slo_ttft_ms"], np.float64); sb = _c(slos["slo_tbt_ms"], np.float64)
    bud = None if gpu_budget is None else _c(gpu_budget, np.int32)
    cells = n_window * G
    n_entry = int(nm.sum()) * n_share
    r = {"energy_j": np.empty(cells), "n_inst": np.empty((cells, tp.size), np.int32),
         "f_index": np.empty((cells, tp.size), np.int32), "share": np.empty((cells, tp.size), np.int32),
         "n_optimal": np.empty(cells, np.int64)}
    if want_types:
        r["type_energy"] = np.empty((cells, n_entry)); r["type_f"] = np.empty((cells, n_entry), np.int32)
    rc = lib.dynoracle_mixed(
        C.c_int32(G), C.c_int32(tp.size), _ptr(tp), C.c_int32(fg.size), _ptr(fg), C.c_int32(rg.size), _ptr(rg),
        _ptr(PF), _ptr(TB), _ptr(PW), _ptr(ML),
        C.c_int64(ins.size), C.c_int32(n_window), C.c_double(window_s), _ptr(ins), _ptr(outs), _ptr(off),
        C.c_int32(n_share), _ptr(nm), _ptr(st), _ptr(sb), C.c_int32(pct[0]), C.c_int32(pct[1]), _ptr(bud),
        _ptr(r["energy_j"]), _ptr(r["n_inst"]), _ptr(r["f_index"]), _ptr(r["share"]), _ptr(r["n_optimal"]),
        _ptr(r.get("type_energy")), _ptr(r.get("type_f")))
    if rc != 0:
        raise ValueError(f"dynoracle_mixed failed: {rc}")
    return r


def select_path(space_cost: np.ndarray, feasible: np.ndarray, n_window: int, n_class: int, layout, transition):
    """Least-total sequence of configurations per class with transition costs between consecutive windows.
    space_cost, feasible: [cells, K]; layout: [K]; transition: [n_layout, n_layout] (from, to).
    Returns (sel [cells], path_cost [n_class])."""
    lib = _load()
    lib.dynoracle_select_path.restype = C.c_int
    cost = _c(space_cost, np.float64); feas = _c(feasible, np.uint8)
    K = cost.shape[1]
    lay = _c(layout, np.int32); tr = _c(transition, np.float64)
    assert cost.shape == feas.shape == (n_window * n_class, K) and lay.size == K and tr.shape[0] == tr.shape[1]
    sel = np.empty(n_window * n_class, np.int32); pc = np.empty(n_class)
    rc = lib.dynoracle_select_path(C.c_int32(n_window), C.c_int32(n_class), C.c_int32(K), _ptr(cost), _ptr(feas),
                                   C.c_int32(tr.shape[0]), _ptr(lay), _ptr(tr), _ptr(sel), _ptr(pc))
    if rc != 0:
        raise ValueError(f"dynoracle_select_path failed: {rc}")
    return sel, pc


def account(configs: Dict[str, np.ndarray], tp, sel: np.ndarray, window_energy_j: np.ndarray, n_window: int, n_class: int,
            window_s: float, gpu_hour_price: float, kwh_price: float, carbon_g_per_kwh, gpus_per_server: int = 8):
    """Cost and carbon of a selection; see dynoracle_account."""
    lib = _load()
    lib.dynoracle_account.restype = C.c_int
    cn = _c(configs["n_inst"], np.int32); ct = _c(configs["tp_index"], np.int32); tpa = _c(tp, np.int32)
    s_ = _c(sel, np.int32); we = _c(window_energy_j, np.float64); ci = _c(carbon_g_per_kwh, np.float64)
    assert s_.size == n_window * n_class and we.size == n_window and ci.size == n_window
    r = {"gpus": np.empty(n_window, np.int64), "gpu_cost": np.empty(n_window), "energy_cost": np.empty(n_window),
         "carbon_g": np.empty(n_window), "totals": np.empty(5)}
    rc = lib.dynoracle_account(C.c_int32(n_window), C.c_int32(n_class), C.c_int32(cn.size), _ptr(cn), _ptr(ct), _ptr(tpa),
                               _ptr(s_), _ptr(we), C.c_double(window_s), C.c_double(gpu_hour_price), C.c_double(kwh_price),
                               _ptr(ci), C.c_int32(gpus_per_server), _ptr(r["gpus"]), _ptr(r["gpu_cost"]),
                               _ptr(r["energy_cost"]), _ptr(r["carbon_g"]), _ptr(r["totals"]))
    if rc != 0:
        raise ValueError(f"dynoracle_account failed: {rc}")
    return r


def hierarchy(profile: Dict[str, np.ndarray], coarse: Dict[str, np.ndarray], fine: Dict[str, np.ndarray], n_window: int,
              n_tick: int, tick_s: float, epoch_windows: int, tp_ref: int, f_ref: int, gpus_per_node: int,
              lay_n, lay_tp, slos: Dict[str, np.ndarray], pct=(99, 100), transition=None,
              spill: bool = False) -> Dict[str, np.ndarray]:
    """Scale-out / shard / frequency controllers, top down; see dynoracle_hierarchy.  `transition`
    ([n_layout][n_layout] joules, from -> to) makes the shard controller weigh re-sharding overheads;
    `spill` applies the fragmentation rule (adds "keep" [n_epoch][G] and "served" [n_window*G])."""
    lib = _load()
    lib.dynoracle_hierarchy.restype = C.c_int
    tp = _c(profile["tp"], np.int32); fg = _c(profile["f_mhz"], np.float64); rg = _c(profile["rho"], np.float64)
    PF = _c(profile["prefill_ms_per_tok"], np.float64); TB = _c(profile["tbt_ms"], np.float64)
    PW = _c(profile["power_w"], np.float64); ML = _c(profile["max_load_tps"], np.float64)
    G = PF.shape[0]
    ic = _c(coarse["in_tok"], np.int32); oc = _c(coarse["out_tok"], np.int32); co = _c(coarse["cell_off"], np.int64)
    if_ = _c(fine["in_tok"], np.int32); of_ = _c(fine["out_tok"], np.int32); fo = _c(fine["cell_off"], np.int64)
    assert co.size == n_window * G + 1 and fo.size == n_window * n_tick * G + 1 and ic.size == if_.size
    ln = _c(lay_n, np.int32); lt = _c(lay_tp, np.int32)
    st = _c(slos["slo_ttft_ms"], np.float64); sb = _c(slos["slo_tbt_ms"], np.float64)
    n_epoch = (n_window + epoch_windows - 1) // epoch_windows
    cells = n_window * G
    r = {"nodes": np.empty((n_epoch, G), np.int32), "layout_sel": np.empty(cells, np.int32),
         "f_sel": np.empty((n_window * n_tick, G), np.int32), "energy_j": np.empty(cells),
         "violations": np.empty(cells, np.int32), "keep": np.empty((n_epoch, G)), "served": np.empty(cells)}
    tr = None
    if transition is not None:
        tr = _c(transition, np.float64)
        assert tr.shape == (ln.size, ln.size)
        r["path_cost"] = np.empty(G)
    rc = lib.dynoracle_hierarchy(
        C.c_int32(G), C.c_int32(tp.size), _ptr(tp), C.c_int32(fg.size), _ptr(fg), C.c_int32(rg.size), _ptr(rg),
        _ptr(PF), _ptr(TB), _ptr(PW), _ptr(ML), C.c_int64(ic.size), C.c_int32(n_window), C.c_int32(n_tick),
        C.c_double(tick_s), _ptr(ic), _ptr(oc), _ptr(co), _ptr(if_), _ptr(of_), _ptr(fo), C.c_int32(epoch_windows),
        C.c_int32(tp_ref), C.c_int32(f_ref), C.c_int32(gpus_per_node), C.c_int32(ln.size), _ptr(ln), _ptr(lt), _ptr(st),
        _ptr(sb), C.c_int32(pct[0]), C.c_int32(pct[1]), None if tr is None else _ptr(tr), C.c_int32(1 if spill else 0),
        _ptr(r["nodes"]), _ptr(r["layout_sel"]), _ptr(r["f_sel"]), _ptr(r["energy_j"]), _ptr(r["violations"]),
        None if tr is None else _ptr(r["path_cost"]), _ptr(r["keep"]), _ptr(r["served"]))
    if rc != 0:
        raise ValueError(f"dynoracle_hierarchy failed: {rc}")
    return r


def window_totals(sel: np.ndarray, sel_energy_j: np.ndarray, n_window: int, n_class: int):
    lib = _load()
    s = _c(sel, np.int32); e = _c(sel_energy_j, np.float64)
    assert s.size == n_window * n_class == e.size
    we = np.empty(n_window); wi = np.empty(n_window, np.int32)
    rc = lib.dynoracle_window_totals(C.c_int32(n_window), C.c_int32(n_class), _ptr(s), _ptr(e), _ptr(we),
                                     _ptr(wi))
    if rc != 0:
        raise ValueError(f"dynoracle_window_totals failed: {rc}")
    return we, wi


def select_row(cost: np.ndarray, feasible: np.ndarray) -> int:
    lib = _load()
    c = _c(cost, np.float64); f = _c(feasible, np.uint8)
    assert c.size == f.size
    return int(lib.dynoracle_select_row(C.c_int32(c.size), _ptr(c), _ptr(f)))
