"""A second, independent statement of the evaluator in NumPy/SciPy, for tiny inputs.

Used only to pin the C++ oracle: it is written against library routines (np.interp,
scipy's RegularGridInterpolator, np.sort, np.searchsorted, stable argsort) and Python
integers/Fractions, not against the oracle's formulas, and shares nothing with it.
"""
from fractions import Fraction
import math

import numpy as np
from scipy.interpolate import RegularGridInterpolator


def np_ingest(trace, edges, n_window, window_s):
    t = np.asarray(trace["t_s"]); x = np.asarray(trace["in_tok"]); y = np.asarray(trace["out_tok"])
    mdl = np.asarray(trace["model"])
    ie, oe = np.asarray(edges["in_edge"]), np.asarray(edges["out_edge"])
    n_model, bi, bo = ie.shape[0], ie.shape[1] + 1, oe.shape[1] + 1
    G = n_model * bi * bo
    cell = np.empty(t.size, np.int64)
    for r in range(t.size):
        w = int(math.floor(Fraction(float(t[r])) / Fraction(float(window_s))))  # exact quotient
        a = int(np.searchsorted(ie[mdl[r]], x[r], side="right"))
        b = int(np.searchsorted(oe[mdl[r]], y[r], side="right"))
        cell[r] = w * G + (mdl[r] * bi + a) * bo + b
    order = np.argsort(cell, kind="stable")
    off = np.zeros(n_window * G + 1, np.int64)
    np.add.at(off, cell + 1, 1)
    return {"in_tok": x[order].astype(np.int32), "out_tok": y[order].astype(np.int32),
            "cell_off": np.cumsum(off)}


def np_eval(profile, st, n_window, window_s, configs, slos, pct=(99, 100), gpu_budget=None,
            idle_cost_weight=0.0):
    tp = profile["tp"]; fg = profile["f_mhz"]; rg = profile["rho"]
    PF, TB, PW, ML = (profile[k] for k in ("prefill_ms_per_tok", "tbt_ms", "power_w", "max_load_tps"))
    G = PF.shape[0]
    K = configs["n_inst"].size
    cells = n_window * G
    off = st["cell_off"]
    out = {k: np.zeros((cells, K)) for k in ("energy_j", "p99_ttft_ms", "p99_tbt_ms", "cost", "rho")}
    out["flags"] = np.zeros((cells, K), np.uint8)
    out["sel"] = np.full(cells, -1, np.int32)
    out["in_p99"] = np.zeros(cells, np.int32)
    out["m"] = np.diff(off)

    def look(X, g, ti, f, r):
        if fg.size == 1:
            return float(np.interp(r, rg, X[g, ti, 0]))
        hit = np.nonzero(fg == f)[0]
        if hit.size:                                    # profiled frequency: the paper's 1-D case
            return float(np.interp(r, rg, X[g, ti, hit[0]]))
        return float(RegularGridInterpolator((fg, rg), X[g, ti])((f, r)))

    for c in range(cells):
        g = c % G
        x = st["in_tok"][off[c]:off[c + 1]].astype(np.int64)
        y = st["out_tok"][off[c]:off[c + 1]].astype(np.int64)
        m = x.size
        load = float(Fraction(int(x.sum() + y.sum())) / Fraction(float(window_s)))
        rank = int(math.ceil(Fraction(pct[0] * m, pct[1])))
        if m:
            out["in_p99"][c] = np.sort(x)[rank - 1]
        best, best_cost = -1, math.inf
        for k in range(K):
            n = int(configs["n_inst"][k]); ti = int(configs["tp_index"][k]); f = float(configs["f_mhz"][k])
            cap = float(np.interp(f, fg, ML[g, ti])) if fg.size > 1 else float(ML[g, ti, 0])
            rho = load / (n * cap)
            over = rho > rg[-1]
            r = min(rho, rg[-1])
            pf, tb, pw = look(PF, g, ti, f, r), look(TB, g, ti, f, r), look(PW, g, ti, f, r)
            pw0 = look(PW, g, ti, f, 0.0)
            ttft = float(np.sort(x * pf)[rank - 1]) if m else 0.0
            tbt = tb if m else 0.0
            e = n * pw * window_s
            cost = e + idle_cost_weight * n * pw0 * window_s
            fl = 0
            if over: fl |= 2
            if ttft > slos["slo_ttft_ms"][g]: fl |= 4
            if tbt > slos["slo_tbt_ms"][g]: fl |= 8
            if gpu_budget is not None and gpu_budget[g] > 0 and n * int(tp[ti]) > gpu_budget[g]: fl |= 16
            if m == 0: fl |= 32
            if not fl & 30: fl |= 1
            out["energy_j"][c, k] = e; out["p99_ttft_ms"][c, k] = ttft; out["p99_tbt_ms"][c, k] = tbt
            out["cost"][c, k] = cost; out["flags"][c, k] = fl; out["rho"][c, k] = rho
            if fl & 1 and cost < best_cost:
                best, best_cost = k, cost
        out["sel"][c] = best
    return out


def np_eval_ticks(profile, fine, n_window, n_tick, tick_s, configs, slos, pct=(99, 100), gpu_budget=None,
                  idle_cost_weight=0.0):
    """Tick-level variant: every request is served under the load of its own tick (sub-window)."""
    tp = profile["tp"]; fg = profile["f_mhz"]; rg = profile["rho"]
    PF, TB, PW, ML = (profile[k] for k in ("prefill_ms_per_tok", "tbt_ms", "power_w", "max_load_tps"))
    G = PF.shape[0]
    K = configs["n_inst"].size
    off = fine["cell_off"]
    cells = n_window * G
    out = {k: np.zeros((cells, K)) for k in ("energy_j", "p99_ttft_ms", "p99_tbt_ms", "cost")}
    out["flags"] = np.zeros((cells, K), np.uint8)
    out["sel"] = np.full(cells, -1, np.int32)

    def look(X, g, ti, f, r):
        if fg.size == 1:
            return float(np.interp(r, rg, X[g, ti, 0]))
        hit = np.nonzero(fg == f)[0]
        if hit.size:
            return float(np.interp(r, rg, X[g, ti, hit[0]]))
        return float(RegularGridInterpolator((fg, rg), X[g, ti])((f, r)))

    for w in range(n_window):
        for g in range(G):
            c = w * G + g
            segs = []
            for q in range(n_tick):
                f = (w * n_tick + q) * G + g
                segs.append((fine["in_tok"][off[f]:off[f + 1]].astype(np.int64),
                             fine["out_tok"][off[f]:off[f + 1]].astype(np.int64)))
            m = sum(x.size for x, _ in segs)
            rank = int(math.ceil(Fraction(pct[0] * m, pct[1])))
            best, best_cost = -1, math.inf
            for k in range(K):
                n = int(configs["n_inst"][k]); ti = int(configs["tp_index"][k]); f = float(configs["f_mhz"][k])
                cap = float(np.interp(f, fg, ML[g, ti])) if fg.size > 1 else float(ML[g, ti, 0])
                ttft, tbt, e, over = [], [], 0.0, False
                for x, y in segs:
                    load = float(Fraction(int(x.sum() + y.sum())) / Fraction(float(tick_s)))
                    rho = load / (n * cap)
                    over = over or rho > rg[-1]
                    r = min(rho, rg[-1])
                    ttft.extend((x * look(PF, g, ti, f, r)).tolist())
                    tbt.extend([look(TB, g, ti, f, r)] * x.size)
                    e += n * look(PW, g, ti, f, r) * tick_s
                p1 = sorted(ttft)[rank - 1] if m else 0.0
                p2 = sorted(tbt)[rank - 1] if m else 0.0
                cost = e + idle_cost_weight * n * look(PW, g, ti, f, 0.0) * (n_tick * tick_s)
                fl = 0
                if over: fl |= 2
                if p1 > slos["slo_ttft_ms"][g]: fl |= 4
                if p2 > slos["slo_tbt_ms"][g]: fl |= 8
                if gpu_budget is not None and gpu_budget[g] > 0 and n * int(tp[ti]) > gpu_budget[g]: fl |= 16
                if m == 0: fl |= 32
                if not fl & 30: fl |= 1
                out["energy_j"][c, k] = e; out["p99_ttft_ms"][c, k] = p1; out["p99_tbt_ms"][c, k] = p2
                out["cost"][c, k] = cost; out["flags"][c, k] = fl
                if fl & 1 and cost < best_cost:
                    best, best_cost = k, cost
            out["sel"][c] = best
    return out


def np_mixed(profile, st, n_window, window_s, n_share, n_max, slos, pct=(99, 100), gpu_budget=None):
    """Eq. 1 by brute force: every (instances, frequency, shares) of every type at once, nothing factored."""
    import itertools
    tp = profile["tp"]; fg = profile["f_mhz"]; rg = profile["rho"]
    PF, TB, PW, ML = (profile[k] for k in ("prefill_ms_per_tok", "tbt_ms", "power_w", "max_load_tps"))
    G = PF.shape[0]
    off = st["cell_off"]
    cells = n_window * G
    energy = np.full(cells, np.inf)
    pick = [None] * cells
    n_opt = np.zeros(cells, np.int64)
    options = []
    for i in range(tp.size):
        o = [None]
        o += [(n, f, a) for n in range(1, int(n_max[i]) + 1) for f in range(fg.size) for a in range(1, n_share + 1)]
        options.append(o)
    for c in range(cells):
        g = c % G
        x = st["in_tok"][off[c]:off[c + 1]].astype(np.int64)
        y = st["out_tok"][off[c]:off[c + 1]].astype(np.int64)
        m = x.size
        load = float(Fraction(int(x.sum() + y.sum())) / Fraction(float(window_s)))
        rank = int(math.ceil(Fraction(pct[0] * m, pct[1])))
        # per type option: (energy, admissible)
        val = []
        for i in range(tp.size):
            v = {}
            for o in options[i][1:]:
                n, f, a = o
                rho = load * a / n_share / (n * ML[g, i, f])
                r = min(rho, rg[-1])
                pf, tb, pw = (float(np.interp(r, rg, X[g, i, f])) for X in (PF, TB, PW))
                ttft = float(np.sort(x * pf)[rank - 1]) if m else 0.0
                ok = rho <= rg[-1] and ttft <= slos["slo_ttft_ms"][g] and (tb if m else 0.0) <= slos["slo_tbt_ms"][g]
                v[o] = (n * pw * window_s, ok)
            val.append(v)
        best = []
        for combo in itertools.product(*options):
            used = [(i, o) for i, o in enumerate(combo) if o is not None]
            if sum(o[2] for _, o in used) != n_share:
                continue
            if gpu_budget is not None and gpu_budget[g] > 0 and sum(o[0] * int(tp[i]) for i, o in used) > gpu_budget[g]:
                continue
            if not all(val[i][o][1] for i, o in used):
                continue
            e = 0.0
            for i, o in used:
                e += val[i][o][0]
            best.append((e, combo))
        if best:
            emin = min(e for e, _ in best)
            energy[c] = emin
            # distinct (instances, shares) assignments reaching the minimum (the frequency is a dependent choice)
            keys = {tuple((o[0], o[2]) if o else (0, 0) for o in cb) for e, cb in best if e == emin}
            n_opt[c] = len(keys)
            pick[c] = sorted(keys)
    return {"energy_j": energy, "assignments": pick, "n_optimal": n_opt}


def np_hierarchy(profile, tr, edges, n_window, n_tick, tick_s, epoch_windows, tp_ref, f_ref, gpus_per_node, lay_n, lay_tp,
                 slos, pct=(99, 100), spill=False):
    """Scale-out / shard / frequency controllers from the raw trace, NumPy arithmetic.  With `spill` a pool below the
    last class that would not fill its last node gets one node less and passes the share of its arriving load that the
    remaining nodes cannot carry on to the next class."""
    tp = profile["tp"]; fg = profile["f_mhz"]; rg = profile["rho"]
    PF, TB, PW, ML = (profile[k] for k in ("prefill_ms_per_tok", "tbt_ms", "power_w", "max_load_tps"))
    G = PF.shape[0]
    W = n_tick * tick_s
    coarse = np_ingest(tr, edges, n_window, W)
    fine = np_ingest(tr, edges, n_window * n_tick, tick_s)

    def run(st, c):
        o = st["cell_off"]
        return st["in_tok"][o[c]:o[c + 1]].astype(np.int64), st["out_tok"][o[c]:o[c + 1]].astype(np.int64)

    def pct_of(v):
        if v.size == 0:
            return 0.0
        return float(np.sort(v)[int(math.ceil(Fraction(pct[0] * v.size, pct[1]))) - 1])

    def admissible(g, ti, f, n, x, load):
        rho = load / (n * ML[g, ti, f])
        r = min(rho, rg[-1])
        pf, tb, pw = (float(np.interp(r, rg, X[g, ti, f])) for X in (PF, TB, PW))
        ok = rho <= rg[-1] and pct_of(x * pf) <= slos["slo_ttft_ms"][g] and (tb if x.size else 0.0) <= slos["slo_tbt_ms"][g]
        return ok, pw

    n_epoch = -(-n_window // epoch_windows)
    nodes = np.zeros((n_epoch, G), np.int32)
    keep = np.ones((n_epoch, G))
    own_c = np.array([[float(sum(v.sum() for v in run(coarse, w * G + g))) / W for g in range(G)] for w in range(n_window)])
    own_f = np.array([[float(sum(v.sum() for v in run(fine, t * G + g))) / tick_s for g in range(G)]
                      for t in range(n_window * n_tick)])
    srv_c = np.zeros_like(own_c); srv_f = np.zeros_like(own_f)
    for e in range(n_epoch):
        ws = slice(e * epoch_windows, min(n_window, (e + 1) * epoch_windows))
        ts = slice(ws.start * n_tick, ws.stop * n_tick)
        pass_c = np.zeros(ws.stop - ws.start); pass_f = np.zeros(ts.stop - ts.start)
        for g in range(G):
            arr_c = own_c[ws, g] + pass_c; arr_f = own_f[ts, g] + pass_f
            peak = max(0.0, arr_c.max())
            cap = max(1, gpus_per_node // int(tp[tp_ref])) * ML[g, tp_ref, f_ref] * rg[-1]
            full = math.floor(peak / cap)
            if spill and g < G - 1 and 1 <= full < peak / cap:
                nodes[e, g] = full
                keep[e, g] = full * cap / peak * (1.0 - 2.0 ** -40)
            else:
                nodes[e, g] = max(1, math.ceil(peak / cap))
            srv_c[ws, g] = keep[e, g] * arr_c; srv_f[ts, g] = keep[e, g] * arr_f
            pass_c = arr_c - srv_c[ws, g]; pass_f = arr_f - srv_f[ts, g]
    lay = np.full(n_window * G, -1, np.int32)
    fsel = np.full((n_window * n_tick, G), -1, np.int32)
    energy = np.full(n_window * G, np.inf)
    viol = np.zeros(n_window * G, np.int32)
    for w in range(n_window):
        for g in range(G):
            c = w * G + g
            x, y = run(coarse, c)
            best, be = -1, np.inf
            for l in range(len(lay_n)):
                if lay_n[l] * int(tp[lay_tp[l]]) > nodes[w // epoch_windows, g] * gpus_per_node:
                    continue
                ok, pw = admissible(g, lay_tp[l], f_ref, lay_n[l], x, srv_c[w, g])
                if ok and lay_n[l] * pw * W < be:
                    best, be = l, lay_n[l] * pw * W
            lay[c] = best
            if best < 0:
                continue
            e = 0.0
            for q in range(n_tick):
                xf, yf = run(fine, (w * n_tick + q) * G + g)
                cand = [(pw, f) for f in range(fg.size) for ok, pw in [admissible(g, lay_tp[best], f, lay_n[best], xf, srv_f[w * n_tick + q, g])] if ok]
                if cand:
                    pw, f = min(cand)
                else:
                    _, pw = admissible(g, lay_tp[best], f_ref, lay_n[best], xf, srv_f[w * n_tick + q, g])
                    f = f_ref
                    viol[c] += 1
                fsel[w * n_tick + q, g] = f
                e += lay_n[best] * pw * tick_s
            energy[c] = e
    return {"nodes": nodes, "layout_sel": lay, "f_sel": fsel, "energy_j": energy, "violations": viol, "keep": keep,
            "served": srv_c.reshape(-1)}
