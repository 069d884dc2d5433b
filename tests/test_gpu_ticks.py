"""Tick-level evaluation (load followed inside a window) on a real MI355X against the CPU oracle."""
import numpy as np
import pytest

import oracle
from workloads import SPECS, make

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KEYS = ("energy_j", "p99_ttft_ms", "p99_tbt_ms", "flags", "sel", "sel_energy_j", "sel_cost")


@pytest.fixture(scope="module")
def dyn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2408_00741_amd as d
    return d


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_ticks(dyn, w, n_tick, gpu_budget=None, trace=None, pct=None):
    """Sorts the trace by tick on the GPU, then evaluates.  Returns (results, fine trace on the host)."""
    tr = trace or w["trace"]
    tick_s = w["window_s"] / n_tick
    ins, outs, off, iws = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]),
                                               _dev(tr["model"]), w["edges"], w["n_window"] * n_tick, tick_s)
    assert dyn.dyn_workspace_status(iws) == 0
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], pct or w["pct"], gpu_budget, w["idle_cost_weight"])
    space, sel, ws = dyn.dyn_eval_select_ticks(prof, ins, outs, off, w["n_window"], n_tick, tick_s, plan)
    status = dyn.dyn_workspace_status(ws)
    torch.cuda.synchronize()
    r = {k: v.cpu().numpy() for k, v in space.items()}
    r.update({k: v.cpu().numpy() for k, v in sel.items()})
    r["status"] = status
    fine = {"in_tok": ins.cpu().numpy(), "out_tok": outs.cpu().numpy(), "cell_off": off.cpu().numpy()}
    prof.free()
    return r, fine


def ora_ticks(w, fine, n_tick, gpu_budget=None, pct=None):
    return oracle.evaluate_ticks(w["profile"], fine, w["n_window"], n_tick, w["window_s"] / n_tick, w["configs"],
                                 w["slos"], pct or w["pct"], gpu_budget, w["idle_cost_weight"])


def assert_same(w, g, o, skip_cells=None):
    keep = np.ones(o["sel"].size, bool)
    if skip_cells is not None:
        keep[skip_cells] = False
    for k in KEYS:
        np.testing.assert_array_equal(g[k][keep], o[k][keep], err_msg=k)
    if skip_cells is None:
        we, wi = oracle.window_totals(o["sel"], o["sel_energy_j"], w["n_window"], w["n_class"])
        np.testing.assert_array_equal(g["window_energy_j"], we)
        np.testing.assert_array_equal(g["window_infeasible"], wi)


CASES = {
    "cfg0-T12": (SPECS[0], 12),
    "cfg0-T16": (SPECS[0], 16),
    "cfg0-T7": (SPECS[0], 7),
    "cfg0-T60": (SPECS[0], 60),
    "cfg1-60k-T12": (SPECS[1].scaled(60_000, 48), 12),
    "cfg1-bigcells-T12": (SPECS[1].scaled(150_000, 2), 12),         # cells of 3*10^4 requests: percentiles 300 deep
    "cfg2-300k-T12": (SPECS[2].scaled(300_000, 40), 12),
    "cfg3-100k-T4": (SPECS[3].scaled(100_001, 9), 4),
    "cfg3-100k-T60": (SPECS[3].scaled(100_001, 9), 60),             # 5-minute windows in 5-second ticks
    "cfg3-200k-T12": (SPECS[3].scaled(200_000, 3), 12),             # percentiles 17 .. 64 and beyond 64 deep
    "cfg4-250k-T6": (SPECS[4].scaled(250_000, 24), 6),
    "cfg4-250k-T64": (SPECS[4].scaled(250_000, 24), 64),
}


@pytest.mark.parametrize("name", list(CASES))
def test_ticks_match_oracle(dyn, name):
    spec, T = CASES[name]
    w = make(spec)
    if spec.n_req >= 150_000:         # the oracle sorts every request under every configuration: every third one will do
        w["configs"] = {k: v[::3].copy() for k, v in w["configs"].items()}
    g, fine = gpu_ticks(dyn, w, T)
    # the fine trace itself is the oracle's (stable order)
    of = oracle.ingest(w["trace"], w["edges"], w["n_window"] * T, w["window_s"] / T)
    for k in ("in_tok", "out_tok", "cell_off"):
        np.testing.assert_array_equal(fine[k], of[k], err_msg=k)
    o = ora_ticks(w, of, T)
    assert g["status"] == 0
    assert_same(w, g, o)
    assert (o["flags"] & 1).any() and (o["flags"] & 6).any()
    j = o["m"] - np.ceil(w["pct"][0] * o["m"] / w["pct"][1]) + 1
    if "bigcells" in name:
        assert j.max() > 64
    if "200k" in name:
        assert ((j > 16) & (j <= 64)).any() and (j > 64).any()


@pytest.mark.parametrize("idx", [0, 1])
def test_one_tick_equals_window_level_entry_point(dyn, idx):
    """One tick per window: every output equals dyn_eval_select's, also for cells of 10^4 requests in one tick."""
    w = make(SPECS[idx] if idx == 0 else SPECS[1].scaled(300_000, 3))
    tr = w["trace"]
    ins, outs, off, _ = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]),
                                             _dev(tr["model"]), w["edges"], w["n_window"], w["window_s"])
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    a_space, a_sel, _ = dyn.dyn_eval_select(prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    b_space, b_sel, ws = dyn.dyn_eval_select_ticks(prof, ins, outs, off, w["n_window"], 1, w["window_s"], plan)
    assert dyn.dyn_workspace_status(ws) == 0
    torch.cuda.synchronize()
    if idx:
        assert int(np.diff(off.cpu().numpy()).max()) > 8192       # a tick larger than the deep-cell kernel sorts whole
    for k in a_space:
        np.testing.assert_array_equal(a_space[k].cpu().numpy(), b_space[k].cpu().numpy(), err_msg=k)
    for k in a_sel:
        np.testing.assert_array_equal(a_sel[k].cpu().numpy(), b_sel[k].cpu().numpy(), err_msg=k)
    prof.free()


def _random_case(seed, n_req, NW, T, tick, in_hi=600, crowd=None):
    rng = np.random.default_rng(700 + seed)
    n_f, n_rho, G = int(rng.integers(1, 4)), int(rng.integers(2, 7)), 2
    fg = np.sort(rng.uniform(500, 2000, n_f))
    rg = np.concatenate([[0.0], np.sort(rng.uniform(0.05, 0.95, n_rho - 1))])
    shape = (G, 2, n_f, n_rho)
    prof = {"tp": np.asarray([2, 4], np.int32), "f_mhz": fg, "rho": rg,
            "prefill_ms_per_tok": rng.uniform(0.05, 0.3, shape), "tbt_ms": np.sort(rng.uniform(10, 150, shape), axis=-1),
            "power_w": np.sort(rng.uniform(100, 3000, shape), axis=-1), "max_load_tps": rng.uniform(100, 900, shape[:3])}
    fcand = list(fg) + ([float(rng.uniform(fg[0], fg[-1]))] if n_f > 1 else [])
    K = 70
    cfg = {"n_inst": rng.integers(1, 9, K).astype(np.int32), "tp_index": rng.integers(0, 2, K).astype(np.int32),
           "f_mhz": rng.choice(fcand, K)}
    t = rng.uniform(0, NW * T * tick, n_req)
    if crowd is not None:
        t[: n_req // 2] = rng.uniform(crowd * tick, (crowd + 1) * tick, n_req // 2)   # half of the trace in one tick
    tr = {"t_s": t, "in_tok": rng.integers(0, in_hi, n_req).astype(np.int32),
          "out_tok": rng.integers(1, 300, n_req).astype(np.int32), "model": np.zeros(n_req, np.int32)}
    w = {"profile": prof, "configs": cfg, "trace": tr, "n_window": NW, "window_s": T * tick, "n_class": G,
         "edges": {"in_edge": np.asarray([[in_hi // 3]], np.int32), "out_edge": np.zeros((1, 0), np.int32)},
         "slos": {"slo_ttft_ms": rng.uniform(20, 120, G), "slo_tbt_ms": rng.uniform(40, 140, G)},
         "pct": (99, 100), "idle_cost_weight": 0.1}
    return w


@pytest.mark.parametrize("seed", range(6))
def test_random_profiles_with_budget_and_idle_cost(dyn, seed):
    w = _random_case(seed, 4000, 5, 4 + seed, 5.0, crowd=3 if seed % 2 else None)
    bud = np.asarray([0, 12], np.int32)
    g, fine = gpu_ticks(dyn, w, w_ticks(w, 5.0), bud)
    o = ora_ticks(w, fine, w_ticks(w, 5.0), bud)
    assert g["status"] == 0
    assert_same(w, g, o)
    assert (o["flags"] & 16).any()


def w_ticks(w, tick):
    return int(round(w["window_s"] / tick))


@pytest.mark.parametrize("pct", [(50, 100), (9, 10), (1, 1), (1, 100)])
def test_other_percentiles(dyn, pct):
    """Median, P90, maximum and minimum: j = m - rank + 1 up to the whole cell."""
    w = _random_case(11, 360, 6, 5, 5.0)     # about 30 requests per cell
    g, fine = gpu_ticks(dyn, w, 5, pct=pct)
    o = ora_ticks(w, fine, 5, pct=pct)
    assert g["status"] == 0
    assert_same(w, g, o)


def test_many_equal_lengths_and_zero_lengths(dyn):
    w = _random_case(3, 3000, 4, 8, 5.0, in_hi=3)    # input lengths 0, 1, 2 only: ties everywhere
    g, fine = gpu_ticks(dyn, w, 8)
    o = ora_ticks(w, fine, 8)
    assert g["status"] == 0
    assert_same(w, g, o)


def _one_class(w):
    w["edges"] = {"in_edge": np.zeros((1, 0), np.int32), "out_edge": np.zeros((1, 0), np.int32)}
    for k in ("prefill_ms_per_tok", "tbt_ms", "power_w", "max_load_tps"):
        w["profile"][k] = w["profile"][k][:1]
    w["slos"] = {k: v[:1] for k, v in w["slos"].items()}
    w["n_class"] = 1
    return w


@pytest.mark.parametrize("n_req,NW,T,crowd", [(12_000, 2, 8, None), (40_000, 2, 12, None), (40_000, 2, 5, 3),
                                              (30_000, 1, 33, 7), (9_000, 3, 64, None)])
def test_deep_percentiles_with_load_dependent_prefill(dyn, n_req, NW, T, crowd):
    """Random tables (the prefill time changes from tick to tick) and cells of thousands of requests: percentiles
    17 .. 64 deep (lists from the cell kernel) and hundreds deep (lists from the deep-cell kernel), both found by
    bisecting the bracket; with `crowd` half of the trace sits in one tick."""
    w = _random_case(20 + T, n_req, NW, T, 5.0, in_hi=8000, crowd=crowd)
    g, fine = gpu_ticks(dyn, w, T)
    o = ora_ticks(w, fine, T)
    assert g["status"] == 0
    assert_same(w, g, o)
    j = o["m"] - np.ceil(99 * o["m"] / 100) + 1
    assert j.max() > 16


@pytest.mark.parametrize("kind", ["flat", "zero", "narrow", "wide"])
@pytest.mark.parametrize("pct", [(99, 100), (9, 10)])
def test_walk_lists_pruned_by_the_prefill_spread(dyn, kind, pct):
    """The walk drops list entries below x_j times (least / largest prefill time of the block's table rows).  Flat
    rows (everything below x_j goes), rows with a zero (nothing may go), rows that differ in the 7th digit (the bound
    falls between neighbouring lengths) and rows a factor 3 apart, on lengths crowded around the percentile: many equal
    to x_j, many one below or above it."""
    w = _random_case(40, 5000, 4, 6, 5.0)
    rng = np.random.default_rng(41)
    pf = w["profile"]["prefill_ms_per_tok"]
    base = rng.uniform(0.05, 0.3, pf.shape[:3] + (1,))
    if kind == "flat":
        pf[...] = base
    elif kind == "zero":
        pf[...] = base
        pf[..., 0] = 0.0
    elif kind == "narrow":
        pf[...] = base * (1.0 + rng.uniform(-3e-7, 3e-7, pf.shape))
    else:
        pf[...] = base * rng.uniform(1.0, 3.0, pf.shape)
    n = w["trace"]["in_tok"].size
    w["trace"]["in_tok"] = (1000 + rng.integers(-2, 3, n) * (rng.uniform(0, 1, n) < 0.9)
                            + rng.integers(-400, 400, n) * (rng.uniform(0, 1, n) < 0.1)).astype(np.int32)
    w["edges"] = {"in_edge": np.asarray([[1000]], np.int32), "out_edge": np.zeros((1, 0), np.int32)}
    g, fine = gpu_ticks(dyn, w, 6, pct=pct)
    o = ora_ticks(w, fine, 6, pct=pct)
    assert g["status"] == 0
    assert_same(w, g, o)


@pytest.mark.parametrize("kind", ["few-values", "narrow-range", "wide-tokens", "crowded-tick", "big-cells", "top-of-16-bits"])
@pytest.mark.parametrize("pct", [(99, 100), (1, 2), (1, 1)])
def test_cells_settled_by_their_ties(dyn, kind, pct):
    """Flat prefill tables (the percentile belongs to a request of length x_j, found from the ticks' counts of such
    requests) with: lengths from five values (hundreds of ties: at the median the rank among them is out of reach of
    the walk's four ticks from both ends and all ticks are ranked; at the 99th percentile the four smallest per-tick
    counts cover it), lengths from a range of 270 values at about six requests per value (ranks within four of the top
    and of the bottom), one token count of 2^16 and more in some cells (those build per-tick lists), half of the trace in one
    tick (too uneven for one wave's registers), and cells of 10^4 requests (a block per cell)."""
    big = kind == "big-cells"
    w = _random_case(50, 60_000 if big else 13_000, 3 if big else 4, 12, 5.0, crowd=3 if kind == "crowded-tick" else None)
    rng = np.random.default_rng(51)
    pf = w["profile"]["prefill_ms_per_tok"]
    pf[...] = rng.uniform(0.05, 0.3, pf.shape[:3] + (1,))
    n = w["trace"]["in_tok"].size
    if kind == "few-values":
        w["trace"]["in_tok"] = rng.choice(np.asarray([900, 950, 1000, 1050, 1100], np.int32), n)
    else:
        w["trace"]["in_tok"] = rng.integers(1000, 1270, n).astype(np.int32)
    if kind == "top-of-16-bits":         # x_j = 65535 is the packed registers' padding value: such a cell builds lists
        w["trace"]["in_tok"] = rng.integers(65_530, 65_536, n).astype(np.int32)
        w["edges"] = {"in_edge": np.asarray([[65_533]], np.int32), "out_edge": np.zeros((1, 0), np.int32)}
    if kind == "wide-tokens":
        w["trace"]["out_tok"][rng.integers(0, n, 4)] = 70_000
        w["trace"]["in_tok"][rng.integers(0, n, 2)] = 65_536
    if kind != "top-of-16-bits":
        w["edges"] = {"in_edge": np.asarray([[1100]], np.int32), "out_edge": np.zeros((1, 0), np.int32)}
    g, fine = gpu_ticks(dyn, w, 12, pct=pct)
    o = ora_ticks(w, fine, 12, pct=pct)
    assert g["status"] == 0
    assert_same(w, g, o)


@pytest.mark.parametrize("pct", [(9, 10), (1, 2), (1, 100)])
def test_sparse_ticks_take_the_general_route(dyn, pct):
    """Many ticks with one or two requests each and a percentile deeper than any four ticks hold: the TBT percentile
    needs all ticks in descending TBT order."""
    w = _random_case(31, 700, 2, 64, 5.0)
    g, fine = gpu_ticks(dyn, w, 64, pct=pct)
    o = ora_ticks(w, fine, 64, pct=pct)
    assert g["status"] == 0
    assert_same(w, g, o)
    cnt = np.diff(fine["cell_off"]).reshape(2, 64, 2)
    j = o["m"] - np.ceil(pct[0] * o["m"] / pct[1]) + 1
    four_smallest = np.sort(np.where(cnt > 0, cnt, 10 ** 9), axis=1)[:, :4, :].sum(axis=1).reshape(-1)
    assert (four_smallest < j).any()


def test_ranks_around_the_depth_of_the_lists(dyn):
    """One cell whose median is exactly DYN_TICK_DEPTH deep (m = 16383: the deepest that gets per-tick lists), one
    request more (whole ticks sorted), and cells three times as deep with half of the trace in one tick (sorted in
    pieces), at the median and at the first percentile (j = 99 % of the cell)."""
    for extra in (0, 1):
        w = _one_class(_random_case(5, 2 * dyn.DYN_TICK_DEPTH - 1 + extra, 1, 8, 5.0, in_hi=5000))
        g, fine = gpu_ticks(dyn, w, 8, pct=(1, 2))
        assert g["status"] == 0
        assert_same(w, g, ora_ticks(w, fine, 8, pct=(1, 2)))
    for pct, crowd, n_req, T in (((1, 2), 3, 50_000, 8), ((1, 100), None, 50_000, 8), ((99, 100), 5, 50_000, 8),
                                ((1, 2), 1, 90_000, 4)):          # the last: a tick of 2 x 22 000 requests, sorted in three pieces
        w = _random_case(6, n_req, 1, T, 5.0, in_hi=3000, crowd=crowd)
        g, fine = gpu_ticks(dyn, w, T, pct=pct)
        o = ora_ticks(w, fine, T, pct=pct)
        assert g["status"] == 0
        assert_same(w, g, o)
        j = o["m"] - np.ceil(pct[0] * o["m"] / pct[1]) + 1
        assert pct == (99, 100) or j.max() > dyn.DYN_TICK_DEPTH


def test_empty_trace_and_empty_ticks(dyn):
    w = _random_case(7, 60, 3, 6, 5.0)
    w["trace"]["t_s"][:] = np.random.default_rng(1).uniform(31.0, 34.0, 60)   # everything in one tick of window 1
    g, fine = gpu_ticks(dyn, w, 6)
    o = ora_ticks(w, fine, 6)
    assert g["status"] == 0
    assert_same(w, g, o)
    assert (o["flags"] & 32).any()
    none = {k: v[:0] for k, v in w["trace"].items()}
    g, fine = gpu_ticks(dyn, w, 6, trace=none)
    o = ora_ticks(w, fine, 6)
    assert_same(w, g, o)
    assert np.all(o["flags"] & 32)


def test_argument_errors(dyn):
    w = _random_case(0, 100, 2, 4, 5.0)
    tr = w["trace"]
    ins, outs, off, _ = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]),
                                             _dev(tr["model"]), w["edges"], 8, 5.0)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"])
    ws = torch.empty(dyn.dyn_eval_ticks_workspace(100, 2, 4, 2, 70), dtype=torch.uint8, device="cuda")
    with pytest.raises(dyn.DynError) as e:      # workspace of the wrong size
        dyn.dyn_eval_select_ticks(prof, ins, outs, off, 2, 4, 5.0, plan, workspace=ws[:1024])
    assert e.value.status == -6
    with pytest.raises(dyn.DynError) as e:      # more ticks than the kernels are built for
        dyn.dyn_eval_select_ticks(prof, ins, outs, torch.zeros(2 * 65 * 2 + 1, dtype=torch.int64, device="cuda"), 2, 65,
                                  5.0, plan, workspace=ws)
    assert e.value.status == -2
    with pytest.raises(dyn.DynError) as e:
        dyn.dyn_eval_select_ticks(prof, ins, outs, off, 2, 4, 0.0, plan, workspace=ws)
    assert e.value.status == -3
    # and the same buffers still work afterwards
    space, sel, _ = dyn.dyn_eval_select_ticks(prof, ins, outs, off, 2, 4, 5.0, plan, workspace=ws)
    torch.cuda.synchronize()
    assert np.isfinite(space["energy_j"].cpu().numpy()).all()
    prof.free()


@pytest.mark.parametrize("idx,n_run", [(2, 6), (3, 2)])
def test_full_size_traces_sampled_windows(dyn, idx, n_run):
    """The one-day and the one-week workload at full size (10^7 requests, 36000 cells x 576 configurations; 5*10^7
    requests, 50400 cells x 1152 configurations, cells of up to 7000 requests), 12 ticks per window, in the launch
    configuration the benchmark's --ticks mode times.  The oracle evaluates three runs of windows (start, the
    evening peak with the deepest percentiles, end), each as a trace of its own; the rest is checked through
    properties that hold at any size."""
    w = make(SPECS[idx])
    T = 12
    NW, G, K = w["n_window"], w["n_class"], w["configs"]["n_inst"].size
    g, fine = gpu_ticks(dyn, w, T)
    assert g["status"] == 0
    off = fine["cell_off"]
    assert off[0] == 0 and off[-1] == w["trace"]["t_s"].size and (np.diff(off) >= 0).all()
    m = np.diff(off).reshape(NW, T, G).sum(axis=1)
    peak = int(np.argmax(m.sum(axis=1)))
    for wa in (0, max(0, min(NW - n_run, peak - n_run // 2)), NW - n_run):
        wb = wa + n_run
        lo, hi = wa * T * G, wb * T * G
        sub = {"in_tok": fine["in_tok"][off[lo]:off[hi]], "out_tok": fine["out_tok"][off[lo]:off[hi]],
               "cell_off": off[lo:hi + 1] - off[lo]}
        o = oracle.evaluate_ticks(w["profile"], sub, wb - wa, T, w["window_s"] / T, w["configs"], w["slos"], w["pct"],
                                  None, w["idle_cost_weight"])
        for k in KEYS:
            np.testing.assert_array_equal(g[k][wa * G:wb * G], o[k], err_msg=f"{k} windows {wa}..{wb}")
        we, wi = oracle.window_totals(o["sel"], o["sel_energy_j"], wb - wa, G)
        np.testing.assert_array_equal(g["window_energy_j"][wa:wb], we)
        np.testing.assert_array_equal(g["window_infeasible"][wa:wb], wi)
    j = m - np.ceil(99 * m / 100) + 1
    assert j.max() > (64 if idx == 3 else 16), "the workload is meant to reach percentiles beyond the register list"
    feas = (g["flags"] & 1).astype(bool)
    sel = g["sel"]
    has = sel >= 0
    assert (feas.any(axis=1) == has).all()
    masked = np.where(feas, g["energy_j"], np.inf)              # idle_cost_weight is 0 for these workloads
    assert w["idle_cost_weight"] == 0.0
    np.testing.assert_array_equal(masked.argmin(axis=1)[has], sel[has])
    np.testing.assert_array_equal(masked.min(axis=1)[has], g["sel_energy_j"][has])
    assert ((g["flags"] & dyn.DYN_F_EMPTY) != 0).all(axis=1).tolist() == (m.reshape(-1) == 0).tolist()
    # a window's energy under tick-level load: never below the least energy any configuration has at zero load
    assert np.isfinite(g["energy_j"]).all() and (g["energy_j"] > 0).all()
    assert np.isfinite(g["p99_ttft_ms"]).all()
