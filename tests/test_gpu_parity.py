"""Parity of the HIP library (through its C ABI) against the CPU oracle, on a real MI355X."""
import numpy as np
import pytest

import oracle
from workloads import SPECS, make

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

RTOL = 1e-9          # tolerance stated for energies and percentiles; results are expected bit-equal


@pytest.fixture(scope="module")
def dyn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2408_00741_amd as d
    return d


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def gpu_ingest(dyn, w):
    tr = w["trace"]
    ins, outs, off, ws = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]),
                                              _dev(tr["model"]), w["edges"], w["n_window"], w["window_s"])
    return ins, outs, off, ws


def gpu_eval(dyn, w, ins, outs, off, gpu_budget=None, prof=None, plan=None):
    own = prof is None
    prof = prof or dyn.dyn_profile_load(w["profile"])
    plan = plan or dyn.Plan(w["configs"], w["slos"], w["pct"], gpu_budget, w["idle_cost_weight"])
    space, ws = dyn.dyn_eval_space(prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    sel = dyn.dyn_select_config(prof, space, w["n_window"], w["window_s"], plan)
    tin, tout, p99 = dyn.dyn_cell_stats(ws, w["n_window"], w["n_class"])
    status = dyn.dyn_workspace_status(ws)
    torch.cuda.synchronize()
    r = {k: v.cpu().numpy() for k, v in space.items()}
    r.update({k: v.cpu().numpy() for k, v in sel.items()})
    r.update(tin=tin.cpu().numpy(), tout=tout.cpu().numpy(), in_p99=p99.cpu().numpy(), status=status)
    # the fused entry point must give the same bits as the two calls above
    space2, sel2, ws2 = dyn.dyn_eval_select(prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    assert dyn.dyn_workspace_status(ws2) == status
    torch.cuda.synchronize()
    for k, v in space2.items():
        np.testing.assert_array_equal(v.cpu().numpy(), r[k], err_msg=f"fused {k}")
    for k, v in sel2.items():
        np.testing.assert_array_equal(v.cpu().numpy(), r[k], err_msg=f"fused {k}")
    if own:
        prof.free()
    return r


def ora_eval(w, st, gpu_budget=None, cell_ids=None):
    return oracle.evaluate(w["profile"], st, w["n_window"], w["window_s"], w["configs"], w["slos"], w["pct"],
                           gpu_budget, w["idle_cost_weight"], cell_ids=cell_ids)


def assert_parity(w, g, o, cell_ids=None, check_windows=True):
    """g: GPU results over all cells; o: oracle results over `cell_ids` (all cells when None)."""
    idx = np.arange(g["sel"].size) if cell_ids is None else np.asarray(cell_ids)
    G = w["n_class"]
    # integer intermediates: bit-exact
    np.testing.assert_array_equal(g["tin"][idx], o["tin"])
    np.testing.assert_array_equal(g["tout"][idx], o["tout"])
    np.testing.assert_array_equal(g["in_p99"][idx], o["in_p99"])
    # floating point: within 1e-9 relative (absolute 0 where the oracle is 0)
    for k in ("energy_j", "p99_ttft_ms", "p99_tbt_ms"):
        a, b = g[k][idx], o[k]
        assert np.all(np.abs(a - b) <= RTOL * np.abs(b)), k
    # flags: equal, except where a value sits within 1e-9 of its threshold (none expected)
    diff = g["flags"][idx] != o["flags"]
    n_amb = 0
    if diff.any():
        c, k = np.nonzero(diff)
        gg = idx[c] % G
        st, sb = w["slos"]["slo_ttft_ms"][gg], w["slos"]["slo_tbt_ms"][gg]
        rg = w["profile"]["rho"]
        prof, cfg = w["profile"], w["configs"]
        fidx = np.searchsorted(prof["f_mhz"], cfg["f_mhz"][k])
        load = (o["tin"][c] + o["tout"][c]) / w["window_s"]
        rho = load / (cfg["n_inst"][k] * prof["max_load_tps"][gg, cfg["tp_index"][k], np.minimum(fidx, prof["f_mhz"].size - 1)])
        amb = (np.abs(o["p99_ttft_ms"][c, k] - st) <= RTOL * st) | (np.abs(o["p99_tbt_ms"][c, k] - sb) <= RTOL * sb) | \
              (np.abs(rho - rg[-1]) <= RTOL * rg[-1])
        assert amb.all(), f"{(~amb).sum()} flag mismatches away from any threshold"
        n_amb = int(amb.sum())
    # selection: bit-exact, except ties within 1e-9 relative among oracle-feasible candidates
    gs, os_ = g["sel"][idx], o["sel"]
    bad = np.nonzero(gs != os_)[0]
    for i in bad:
        assert n_amb or (gs[i] >= 0 and os_[i] >= 0), "selection differs"
        if gs[i] >= 0 and os_[i] >= 0 and (o["flags"][i, gs[i]] & 1):
            assert abs(o["cost"][i, gs[i]] - o["cost"][i, os_[i]]) <= RTOL * abs(o["cost"][i, os_[i]])
        else:
            assert n_amb, "selection differs with no ambiguous entry to explain it"
    ok = gs == os_
    fin = ok & (os_ >= 0)
    assert np.all(np.abs(g["sel_energy_j"][idx][fin] - o["sel_energy_j"][fin]) <= RTOL * o["sel_energy_j"][fin])
    assert np.all(np.abs(g["sel_cost"][idx][fin] - o["sel_cost"][fin]) <= RTOL * np.abs(o["sel_cost"][fin]))
    none = ok & (os_ < 0)
    assert np.all(np.isinf(g["sel_energy_j"][idx][none])) and np.all(np.isinf(g["sel_cost"][idx][none]))
    if check_windows and cell_ids is None:
        we, wi = oracle.window_totals(o["sel"], o["sel_energy_j"], w["n_window"], G)
        if not bad.size:
            assert np.all(np.abs(g["window_energy_j"] - we) <= RTOL * np.abs(we))
            np.testing.assert_array_equal(g["window_infeasible"], wi)
    exact = all(np.array_equal(g[k][idx], o[k]) for k in ("energy_j", "p99_ttft_ms", "p99_tbt_ms", "flags"))
    return {"bit_exact": exact, "ambiguous": n_amb, "sel_mismatch": int(bad.size)}


# ------------------------------------------------------------------------------ ingestion
INGEST_CASES = {
    "cfg0-full": SPECS[0],
    "cfg1-40k": SPECS[1].scaled(40_000, 7),
    "cfg2-300k": SPECS[2].scaled(300_000, 40),
    "cfg3-100k": SPECS[3].scaled(100_001, 9),
    "cfg4-250k": SPECS[4].scaled(250_000, 12),
}


@pytest.mark.parametrize("name", list(INGEST_CASES))
@pytest.mark.parametrize("shuffle", [False, True])
def test_ingest_matches_oracle(dyn, name, shuffle):
    w = make(INGEST_CASES[name])
    if shuffle:      # arrival order is not required to be time order
        perm = np.random.default_rng(5).permutation(w["trace"]["t_s"].size)
        w["trace"] = {k: v[perm] for k, v in w["trace"].items()}
    st = oracle.ingest(w["trace"], w["edges"], w["n_window"], w["window_s"])
    ins, outs, off, ws = gpu_ingest(dyn, w)
    assert dyn.dyn_workspace_status(ws) == 0
    np.testing.assert_array_equal(off.cpu().numpy(), st["cell_off"])
    np.testing.assert_array_equal(ins.cpu().numpy(), st["in_tok"])
    np.testing.assert_array_equal(outs.cpu().numpy(), st["out_tok"])


def test_ingest_edge_cases(dyn):
    edges = {"in_edge": np.asarray([[256, 1024]], np.int32), "out_edge": np.asarray([[100, 350]], np.int32)}
    # Table IV thresholds, values on and around every edge, a window boundary, one request per class
    x = np.asarray([255, 256, 257, 1023, 1024, 1025, 8192, 1, 1], np.int32)
    y = np.asarray([349, 350, 351, 99, 100, 101, 8192, 1, 1], np.int32)
    t = np.asarray([0.0, 59.999, 60.0, 60.0, 119.9, 0.5, 179.99, 120.0, 0.25])
    tr = {"t_s": t, "in_tok": x, "out_tok": y, "model": np.zeros(9, np.int32)}
    st = oracle.ingest(tr, edges, 3, 60.0)
    ins, outs, off, ws = dyn.dyn_trace_ingest(_dev(t), _dev(x), _dev(y), None, edges, 3, 60.0)
    assert dyn.dyn_workspace_status(ws) == 0
    np.testing.assert_array_equal(off.cpu().numpy(), st["cell_off"])
    np.testing.assert_array_equal(ins.cpu().numpy(), st["in_tok"])
    np.testing.assert_array_equal(outs.cpu().numpy(), st["out_tok"])
    # empty trace
    e = torch.empty(0, dtype=torch.float64, device="cuda"); ei = torch.empty(0, dtype=torch.int32, device="cuda")
    ins, outs, off, ws = dyn.dyn_trace_ingest(e, ei, ei.clone(), None, edges, 3, 60.0)
    assert off.cpu().numpy().tolist() == [0] * 28 and ins.numel() == 0
    # one class, one window (a single cell): order must be preserved exactly
    one = {"in_edge": np.zeros((1, 0), np.int32), "out_edge": np.zeros((1, 0), np.int32)}
    n = 20_000
    tag = np.arange(n, dtype=np.int32)
    ins, outs, off, ws = dyn.dyn_trace_ingest(_dev(np.linspace(0, 59, n)), _dev(tag), _dev(tag[::-1].copy()), None,
                                              one, 1, 60.0)
    np.testing.assert_array_equal(ins.cpu().numpy(), tag)
    assert off.cpu().numpy().tolist() == [0, n]
    # timestamps outside the windows and a bad model index are reported, never dereferenced out of range
    bad_t = np.asarray([-1.0, 10.0, 1e9, float("nan")])
    ins, outs, off, ws = dyn.dyn_trace_ingest(_dev(bad_t), _dev(np.ones(4, np.int32)), _dev(np.ones(4, np.int32)),
                                              _dev(np.asarray([0, 0, 0, 7], np.int32)), edges, 3, 60.0)
    assert dyn.dyn_workspace_status(ws) & dyn.DYN_WS_BAD_REQUEST
    assert off.cpu().numpy()[-1] == 4


@pytest.mark.parametrize("case", ["sorted", "one-swap", "reversed-windows", "sorted-many-classes", "sorted-empty-windows"])
def test_ingest_routes(dyn, case):
    """A trace in window order is moved window by window, any other one by the general sort; more classes than
    the window route keeps counters for always take the sort.  Same result either way."""
    rng = np.random.default_rng(21)
    n, NW, W = 60_000, 7, 10.0
    t = np.sort(rng.uniform(0, NW * W, n))
    x = rng.integers(1, 8193, n).astype(np.int32); y = rng.integers(1, 8193, n).astype(np.int32)
    edges = {"in_edge": np.asarray([[64, 512, 4096]], np.int32), "out_edge": np.asarray([[100, 1000]], np.int32)}
    if case == "one-swap":                 # a single request out of window order, near the end
        t[-10], t[-30000] = t[-30000], t[-10]
    elif case == "reversed-windows":
        t = t[::-1].copy()
    elif case == "sorted-many-classes":    # 40 x 30 = 1200 classes
        edges = {"in_edge": np.arange(100, 4000, 100, dtype=np.int32)[None, :39], "out_edge": np.arange(50, 1500, 50, dtype=np.int32)[None, :29]}
    elif case == "sorted-empty-windows":   # nothing in windows 0, 3 and the last two
        t = np.sort(np.concatenate([rng.uniform(W, 3 * W, n // 2), rng.uniform(4 * W, 5 * W, n - n // 2)]))
    tr = {"t_s": t, "in_tok": x, "out_tok": y, "model": np.zeros(n, np.int32)}
    st = oracle.ingest(tr, edges, NW, W)
    ins, outs, off, ws = dyn.dyn_trace_ingest(_dev(t), _dev(x), _dev(y), None, edges, NW, W)
    assert dyn.dyn_workspace_status(ws) == 0
    np.testing.assert_array_equal(off.cpu().numpy(), st["cell_off"])
    np.testing.assert_array_equal(ins.cpu().numpy(), st["in_tok"])
    np.testing.assert_array_equal(outs.cpu().numpy(), st["out_tok"])


# ------------------------------------------------------------------- evaluation + selection
EVAL_CASES = {
    "cfg0-full": (SPECS[0], None),
    "cfg1-60k": (SPECS[1].scaled(60_000, 6), None),
    "cfg1-bigcells": (SPECS[1].scaled(150_000, 2), None),          # cells of ~10^4 requests: streamed path
    "cfg2-200k": (SPECS[2].scaled(200_000, 29), None),
    "cfg3-150k": (SPECS[3].scaled(150_000, 5), None),
    "cfg4-120k": (SPECS[4].scaled(120_000, 3), None),
    "cfg2-budget": (SPECS[2].scaled(50_000, 7), "budget"),
}


@pytest.mark.parametrize("name", list(EVAL_CASES))
def test_eval_and_select_match_oracle(dyn, name):
    spec, extra = EVAL_CASES[name]
    w = make(spec)
    bud = None
    if extra == "budget":
        bud = (np.arange(w["n_class"]) % 4 * 8).astype(np.int32)        # 0 (unlimited), 8, 16, 24 GPUs
    st = oracle.ingest(w["trace"], w["edges"], w["n_window"], w["window_s"])
    ins, outs, off, _ = gpu_ingest(dyn, w)
    g = gpu_eval(dyn, w, ins, outs, off, bud)
    assert g["status"] == 0
    o = ora_eval(w, st, bud)
    rep = assert_parity(w, g, o)
    print(name, rep)
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0
    feas = (o["flags"] & 1).astype(bool)
    assert feas.any() and not feas.all()


def _profile(tp, fg, rg, PF, TB, PW, ML):
    return {"tp": np.asarray(tp, np.int32), "f_mhz": np.asarray(fg, float), "rho": np.asarray(rg, float),
            "prefill_ms_per_tok": np.asarray(PF, float), "tbt_ms": np.asarray(TB, float),
            "power_w": np.asarray(PW, float), "max_load_tps": np.asarray(ML, float)}


def _worked():
    PF = np.empty((1, 2, 2, 3)); TB = np.empty((1, 2, 2, 3)); PW = np.empty((1, 2, 2, 3))
    PF[0, 0, 0] = 0.4; PF[0, 0, 1] = 0.2; PF[0, 1, 0] = 0.2; PF[0, 1, 1] = 0.1
    TB[0, 0, 0] = [40, 80, 160]; TB[0, 0, 1] = [20, 40, 80]; TB[0, 1, 0] = [20, 40, 80]; TB[0, 1, 1] = [10, 20, 40]
    PW[0, 0, 0] = [200, 275, 312.5]; PW[0, 0, 1] = [200, 800, 1100]
    PW[0, 1, 0] = [400, 550, 625]; PW[0, 1, 1] = [400, 1600, 2200]
    prof = _profile([2, 4], [1000, 2000], [0, 0.5, 0.75], PF, TB, PW, [[[20.0, 40.0], [40.0, 80.0]]])
    cfg = {"n_inst": np.asarray([1, 1, 1, 2, 1, 1], np.int32), "tp_index": np.asarray([0, 0, 0, 0, 1, 1], np.int32),
           "f_mhz": np.asarray([1000.0, 1500, 2000, 2000, 1000, 2000])}
    return prof, cfg


def _single(dyn, prof, cfg, x, y, slo_ttft, slo_tbt, wlen, lam=0.0, pct=(99, 100), budget=None, n_window=1, off=None):
    G = np.asarray(prof["prefill_ms_per_tok"]).shape[0]
    w = {"profile": prof, "configs": cfg, "slos": {"slo_ttft_ms": np.full(G, float(slo_ttft)) if np.isscalar(slo_ttft) else slo_ttft,
                                                   "slo_tbt_ms": np.full(G, float(slo_tbt)) if np.isscalar(slo_tbt) else slo_tbt},
         "pct": pct, "idle_cost_weight": lam, "n_window": n_window, "window_s": wlen, "n_class": G}
    x = np.asarray(x, np.int32); y = np.asarray(y, np.int32)
    off = np.asarray([0, x.size], np.int64) if off is None else np.asarray(off, np.int64)
    st = {"in_tok": x, "out_tok": y, "cell_off": off}
    g = gpu_eval(dyn, w, _dev(x), _dev(y), _dev(off), budget)
    return w, st, g


def test_worked_example_on_gpu(dyn, golden_dir):
    import os
    rows = np.asarray([[float(v) for v in l.split()] for l in open(os.path.join(golden_dir, "worked_example.txt"))
                       if l.strip() and not l.startswith("#")])
    prof, cfg = _worked()
    w, st, g = _single(dyn, prof, cfg, [100, 200, 300, 400], [50, 100, 150, 200], 100, 50, 100.0, lam=0.1)
    np.testing.assert_allclose(g["p99_ttft_ms"][0], rows[:, 5], rtol=1e-13)
    np.testing.assert_array_equal(g["p99_tbt_ms"][0], rows[:, 6])
    np.testing.assert_array_equal(g["energy_j"][0], rows[:, 8])
    np.testing.assert_array_equal(g["flags"][0] & 1, rows[:, 10].astype(np.uint8))
    assert g["sel"][0] == 4 and g["sel_energy_j"][0] == 51250.0 and g["sel_cost"][0] == 55250.0
    assert g["in_p99"][0] == 400 and g["tin"][0] == 1000 and g["tout"][0] == 500
    assert_parity(w, g, ora_eval(w, st))
    for (a, b, lam, want) in ((100, 30, 0.0, 3), (50, 50, 0.0, 5), (30, 50, 0.0, -1)):
        w, st, g = _single(dyn, prof, cfg, [100, 200, 300, 400], [50, 100, 150, 200], a, b, 100.0, lam=lam)
        assert g["sel"][0] == want
        assert_parity(w, g, ora_eval(w, st))
    w, st, g = _single(dyn, prof, cfg, [100, 200, 300, 500], [50, 100, 150, 200], 100, 50, 100.0)
    assert g["flags"][0, 0] & dyn.DYN_F_OVERLOAD
    w, st, g = _single(dyn, prof, cfg, [], [], 100, 50, 100.0)
    np.testing.assert_array_equal(g["energy_j"][0], [20000, 20000, 20000, 40000, 40000, 40000])
    assert g["sel"][0] == 0 and (g["flags"][0] == 33).all()
    # GPU budget of two GPUs per pool
    w, st, g = _single(dyn, prof, cfg, [100, 200, 300, 400], [50, 100, 150, 200], 100, 50, 100.0,
                       budget=np.asarray([2], np.int32))
    assert g["sel"][0] == 2
    assert_parity(w, g, ora_eval(w, st, np.asarray([2], np.int32)))


@pytest.mark.parametrize("m", [1, 2, 63, 64, 65, 99, 100, 101, 128, 129, 200, 511, 513, 1024, 1025, 2047, 2048,
                               2049, 3072, 3073, 4095, 4096, 4097, 6144, 6145, 6401, 8191, 8192, 8193, 12_801, 70_001])
def test_rank_select_cell_sizes(dyn, m):
    """Every register tier (plain and packed), the tier boundaries and the streamed path; distinct and duplicate
    values; 16-bit values incl. 0 and 65535 (the packed tiers' padding value) and a single 65536 among them (the
    cell then leaves the packed tier for the streamed path)."""
    prof, cfg = _worked()
    rng = np.random.default_rng(m)
    for kind in ("perm", "dups", "wide", "u16", "top16", "over"):
        if kind == "perm":
            x = rng.permutation(np.arange(1, m + 1))
        elif kind == "dups":
            x = rng.integers(1, 40, m)
        elif kind == "u16":
            x = rng.integers(0, 65536, m)
            x[rng.integers(0, m, 3)] = 65535
            x[rng.integers(0, m)] = 0
        elif kind == "top16":                          # the percentile itself is 65535 or just below it
            x = rng.integers(65_530, 65_536, m)
        elif kind == "over":
            x = rng.integers(60000, 65536, m)
            x[rng.integers(0, m)] = 65536
        else:
            x = rng.integers(0, 2 ** 30, m)            # exercises the 16-bit split sums and 30-bit selection
        y = rng.integers(1, 8193, m) if kind != "over" else rng.integers(65000, 65536, m)
        for pct in ((99, 100), (1, 2), (1, 1), (1, 100)):
            w, st, g = _single(dyn, prof, cfg, x, y, 1e12, 1e12, 1e6, pct=pct)
            rank = -(-pct[0] * m // pct[1])
            assert g["in_p99"][0] == np.sort(x)[rank - 1], (kind, pct)
            assert g["tin"][0] == int(x.astype(np.int64).sum()) and g["tout"][0] == int(y.astype(np.int64).sum())
            assert g["status"] == 0
        assert_parity(w, g, ora_eval(w, st))


def test_ragged_and_empty_cells(dyn):
    """Many cells of sizes 0..300 in one launch, with empty cells first, last and in runs."""
    prof, cfg = _worked()
    rng = np.random.default_rng(11)
    sizes = np.concatenate([[0, 0, 1, 0, 64, 65, 0], rng.integers(0, 300, 500), [2049, 0, 0]])
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = rng.integers(1, 8193, n); y = rng.integers(1, 8193, n)
    w, st, g = _single(dyn, prof, cfg, x, y, 100, 50, 1000.0, n_window=sizes.size, off=off, lam=0.1)
    o = ora_eval(w, st)
    rep = assert_parity(w, g, o)
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0
    assert ((g["flags"] & dyn.DYN_F_EMPTY) != 0).all(axis=1).tolist() == (sizes == 0).tolist()


def test_mixed_small_and_large_cells(dyn):
    """Cells from empty to several thousand requests side by side: staged runs that end at a large
    cell, cells between the register tiers and the staging capacity, cells handled by a whole block."""
    prof, cfg = _worked()
    rng = np.random.default_rng(12)
    for hi, n_cells in ((6000, 70), (1200, 150), (40, 333)):
        sizes = rng.integers(0, hi, n_cells)
        sizes[rng.integers(0, n_cells, 5)] = 0
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        n = int(off[-1])
        x = rng.integers(1, 8193, n); y = rng.integers(1, 8193, n)
        w, st, g = _single(dyn, prof, cfg, x, y, 100, 50, 1000.0, n_window=sizes.size, off=off, lam=0.1)
        assert g["status"] == 0
        rep = assert_parity(w, g, ora_eval(w, st))
        assert rep["bit_exact"] and rep["sel_mismatch"] == 0


@pytest.mark.parametrize("pct", [(99, 100), (1, 2)])
def test_blocks_mixing_packed_streamed_and_handed_over_cells(dyn, pct):
    """Blocks of four consecutive cells in which a wave's own cell (plain or packed registers), cells beyond 8192
    requests (streamed by the block) and packed-size cells that hold a token count of 2^16 or more, or a negative one
    (handed over to the block after the waves' own work), sit side by side in every combination."""
    prof, cfg = _worked()
    rng = np.random.default_rng(77 + pct[0])
    kinds = rng.integers(0, 5, 96)
    sizes = np.select([kinds == 0, kinds == 1, kinds == 2, kinds == 3], [rng.integers(0, 2049, 96), rng.integers(2049, 8193, 96),
                      rng.integers(8193, 12000, 96), rng.integers(2049, 8193, 96)], rng.integers(2049, 8193, 96))
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = rng.integers(1, 8193, n); y = rng.integers(1, 8193, n)
    neg = []
    for c in np.nonzero(kinds == 3)[0]:                       # a large input or output count somewhere in the cell
        i = int(rng.integers(off[c], off[c + 1]))
        if c % 2:
            x[i] = 65536 + int(rng.integers(0, 1000))
        else:
            y[i] = 1 << 20
    for c in np.nonzero(kinds == 4)[0][:3]:                   # a negative count: status bit, sums still signed
        y[int(rng.integers(off[c], off[c + 1]))] = -5
        neg.append(c)
    w, st, g = _single(dyn, prof, cfg, x, y, 100, 50, 1000.0, n_window=sizes.size, off=off, lam=0.1, pct=pct)
    assert g["status"] == (dyn.DYN_WS_BAD_REQUEST if neg else 0)
    for c in range(sizes.size):
        seg = x[off[c]:off[c + 1]]
        assert g["tin"][c] == int(seg.astype(np.int64).sum())
        assert g["tout"][c] == int(y[off[c]:off[c + 1]].astype(np.int64).sum())
        if seg.size:
            assert g["in_p99"][c] == np.sort(seg)[-(-pct[0] * seg.size // pct[1]) - 1], (c, kinds[c], seg.size)


@pytest.mark.parametrize("pct", [(99, 100), (1, 2), (1, 1), (1, 100), (9, 10)])
def test_many_small_cells_with_outliers(dyn, pct):
    """A tick-like cut (a few dozen requests per cell on average, several cells per wave) with everything
    that leaves the common path mixed in: cells whose nearest rank is not among the two largest inputs,
    runs of cells too long to stage, cells for one wave alone and for a whole block, token counts of 2^20
    and more, empty stretches, and a last group that is not full."""
    prof, cfg = _worked()
    rng = np.random.default_rng(13 + pct[0])
    sizes = rng.integers(0, 60, 3001)
    sizes[rng.integers(0, sizes.size, 300)] = 0
    sizes[rng.integers(0, sizes.size, 40)] = rng.integers(100, 1000, 40)
    sizes[rng.integers(0, sizes.size, 8)] = rng.integers(1025, 2049, 8)
    sizes[[17, 1500, 2999]] = [2049, 5000, 3000]
    sizes[100:140] = 0
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    assert n // 48 <= sizes.size
    x = rng.integers(1, 8193, n); y = rng.integers(1, 8193, n)
    for c in (5, 640, 1501, 2500, 2999):                   # wide values: sums beyond 32 bits per lane
        x[off[c]:off[c + 1]] = rng.integers(2 ** 20, 2 ** 30, sizes[c])
        y[off[c]:off[c + 1]] = rng.integers(0, 2 ** 30, sizes[c])
    w, st, g = _single(dyn, prof, cfg, x, y, 100, 50, 1000.0, n_window=sizes.size, off=off, lam=0.1, pct=pct)
    assert g["status"] == 0
    xs = x.astype(np.int64); ys = y.astype(np.int64)
    for c in range(sizes.size):
        seg = xs[off[c]:off[c + 1]]
        assert g["tin"][c] == seg.sum() and g["tout"][c] == ys[off[c]:off[c + 1]].sum(), c
        if seg.size:
            assert g["in_p99"][c] == np.sort(seg)[-(-pct[0] * seg.size // pct[1]) - 1], (c, seg.size)
    rep = assert_parity(w, g, ora_eval(w, st))
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0


def test_small_cells_bad_offsets_and_negative_tokens_are_reported_per_cell(dyn):
    prof, cfg = _worked()
    rng = np.random.default_rng(14)
    sizes = rng.integers(0, 40, 200)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = rng.integers(1, 8193, n); y = rng.integers(1, 8193, n)
    good = _single(dyn, prof, cfg, x, y, 100, 50, 1000.0, n_window=sizes.size, off=off)[2]
    bad_off = off.copy(); bad_off[70] = off[90]            # cells 69 and 70 now have offsets out of order
    g = _single(dyn, prof, cfg, x, y, 100, 50, 1000.0, n_window=sizes.size, off=bad_off)[2]
    assert g["status"] & dyn.DYN_WS_BAD_OFFSETS
    keep = np.ones(sizes.size, bool); keep[[69, 70]] = False
    np.testing.assert_array_equal(g["tin"][keep], good["tin"][keep])
    np.testing.assert_array_equal(g["in_p99"][keep], good["in_p99"][keep])
    x2 = x.copy(); x2[off[33]] = -5
    g = _single(dyn, prof, cfg, x2, y, 100, 50, 1000.0, n_window=sizes.size, off=off)[2]
    assert g["status"] & dyn.DYN_WS_BAD_REQUEST
    keep = np.ones(sizes.size, bool); keep[33] = False
    np.testing.assert_array_equal(g["tin"][keep], good["tin"][keep])
    np.testing.assert_array_equal(g["in_p99"][keep], good["in_p99"][keep])
    # a negative output length inside a cell that the whole block takes (more than 2048 requests)
    big = rng.integers(1, 8193, 5000); yb = rng.integers(1, 8193, 5000); yb[4321] = -7
    g = _single(dyn, prof, cfg, big, yb, 100, 50, 1000.0)[2]
    assert g["status"] & dyn.DYN_WS_BAD_REQUEST
    assert g["tin"][0] == int(big.sum()) and g["tout"][0] == int(yb.sum())


def test_off_grid_frequencies_single_frequency_and_odd_k(dyn):
    rng = np.random.default_rng(21)
    G, n_tp = 3, 2
    for n_f, n_rho, K in ((4, 5, 37), (1, 2, 1), (3, 9, 300), (2, 64, 65)):
        fg = np.sort(rng.uniform(500, 2000, n_f)); rg = np.concatenate([[0.0], np.sort(rng.uniform(0.05, 0.95, n_rho - 1))])
        shape = (G, n_tp, n_f, n_rho)
        prof = _profile([2, 4], fg, rg, rng.uniform(0.05, 0.3, shape), np.sort(rng.uniform(10, 150, shape), axis=-1),
                        np.sort(rng.uniform(100, 3000, shape), axis=-1), rng.uniform(20, 400, shape[:3]))
        f = np.where(rng.random(K) < 0.5, rng.choice(fg, K), rng.uniform(fg[0], fg[-1], K))
        cfg = {"n_inst": rng.integers(1, 9, K).astype(np.int32), "tp_index": rng.integers(0, n_tp, K).astype(np.int32),
               "f_mhz": f}
        NW = 4
        sizes = rng.integers(0, 400, NW * G)
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        x = rng.integers(1, 600, off[-1]); y = rng.integers(1, 300, off[-1])
        slo_t = rng.uniform(20, 120, G); slo_b = rng.uniform(40, 140, G)
        w, st, g = _single(dyn, prof, cfg, x, y, slo_t, slo_b, 30.0, lam=0.1, n_window=NW, off=off,
                           budget=np.asarray([0, 8, 16], np.int32))
        o = ora_eval(w, st, np.asarray([0, 8, 16], np.int32))
        rep = assert_parity(w, g, o)
        assert rep["bit_exact"] and rep["sel_mismatch"] == 0, (n_f, n_rho, K, rep)


def test_table_rows_beyond_lds_fall_back_to_global_reads(dyn):
    """A long load grid with every candidate on its own pair of rows exceeds the LDS budget."""
    rng = np.random.default_rng(31)
    G, n_tp, n_f, n_rho, K = 2, 2, 40, 200, 64
    fg = np.linspace(500, 2000, n_f); rg = np.linspace(0, 0.9, n_rho)
    shape = (G, n_tp, n_f, n_rho)
    prof = _profile([1, 8], fg, rg, rng.uniform(0.05, 0.3, shape), np.sort(rng.uniform(10, 150, shape), axis=-1),
                    np.sort(rng.uniform(100, 3000, shape), axis=-1), rng.uniform(20, 400, shape[:3]))
    cfg = {"n_inst": rng.integers(1, 5, K).astype(np.int32), "tp_index": (np.arange(K) % 2).astype(np.int32),
           "f_mhz": rng.uniform(fg[0], fg[-1], K)}
    sizes = rng.integers(1, 200, 3 * G)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    x = rng.integers(1, 600, off[-1]); y = rng.integers(1, 300, off[-1])
    w, st, g = _single(dyn, prof, cfg, x, y, 60.0, 90.0, 30.0, n_window=3, off=off)
    rep = assert_parity(w, g, ora_eval(w, st))
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0


def test_largest_candidate_list(dyn):
    """65536 candidates, the capacity of a profile handle's candidate table (one more is refused)."""
    rng = np.random.default_rng(41)
    G, n_tp, n_f, n_rho, K = 2, 3, 6, 12, 65536
    fg = np.linspace(600, 2000, n_f); rg = np.concatenate([[0.0], np.sort(rng.uniform(0.05, 0.95, n_rho - 1))])
    shape = (G, n_tp, n_f, n_rho)
    prof = _profile([2, 4, 8], fg, rg, rng.uniform(0.05, 0.3, shape), np.sort(rng.uniform(10, 150, shape), axis=-1),
                    np.sort(rng.uniform(100, 3000, shape), axis=-1), rng.uniform(20, 400, shape[:3]))
    f = np.where(rng.random(K) < 0.7, rng.choice(fg, K), rng.uniform(fg[0], fg[-1], K))
    cfg = {"n_inst": rng.integers(1, 200, K).astype(np.int32), "tp_index": rng.integers(0, n_tp, K).astype(np.int32),
           "f_mhz": f}
    sizes = np.asarray([130, 0, 77, 1])
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    x = rng.integers(1, 600, off[-1]); y = rng.integers(1, 300, off[-1])
    w, st, g = _single(dyn, prof, cfg, x, y, np.asarray([80.0, 50.0]), np.asarray([90.0, 70.0]), 30.0, lam=0.02, n_window=2,
                       off=off, budget=np.asarray([0, 400], np.int32))
    rep = assert_parity(w, g, ora_eval(w, st, np.asarray([0, 400], np.int32)))
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0
    cfg1 = {k: np.concatenate([v, v[:1]]) for k, v in cfg.items()}
    with pytest.raises(dyn.DynError) as e:
        _single(dyn, prof, cfg1, x, y, np.asarray([80.0, 50.0]), np.asarray([90.0, 70.0]), 30.0, n_window=2, off=off)
    assert e.value.status == -2


def test_device_side_checks_raise_status_not_faults(dyn):
    prof, cfg = _worked()
    x = np.arange(1, 11); y = np.ones(10)
    # offsets that run backwards and past the end of the trace: the cells are skipped and reported
    w, st, g = _single(dyn, prof, cfg, x, y, 100, 50, 100.0, n_window=3, off=[0, 7, 3, 10_000])
    assert g["status"] & dyn.DYN_WS_BAD_OFFSETS
    assert g["tin"][0] == 28
    # a negative token count is reported
    w, st, g = _single(dyn, prof, cfg, [5, -3, 7], [1, 1, 1], 100, 50, 100.0)
    assert g["status"] & dyn.DYN_WS_BAD_REQUEST


def test_argument_errors(dyn):
    prof_d, cfg = _worked()
    prof = dyn.dyn_profile_load(prof_d)
    x = _dev(np.arange(1, 5, dtype=np.int32)); off = _dev(np.asarray([0, 4], np.int64))
    slos = {"slo_ttft_ms": np.asarray([100.0]), "slo_tbt_ms": np.asarray([50.0])}

    def status(fn):
        with pytest.raises(dyn.DynError) as e:
            fn()
        assert dyn.dyn_last_error()
        return e.value.status

    bad = dict(cfg); bad["f_mhz"] = cfg["f_mhz"].copy(); bad["f_mhz"][0] = 999.0
    assert status(lambda: dyn.dyn_eval_space(prof, x, x, off, 1, 100.0, dyn.Plan(bad, slos))) == -3
    bad = dict(cfg); bad["n_inst"] = cfg["n_inst"].copy(); bad["n_inst"][1] = 0
    assert status(lambda: dyn.dyn_eval_space(prof, x, x, off, 1, 100.0, dyn.Plan(bad, slos))) == -3
    bad = dict(cfg); bad["tp_index"] = cfg["tp_index"].copy(); bad["tp_index"][1] = 2
    assert status(lambda: dyn.dyn_eval_space(prof, x, x, off, 1, 100.0, dyn.Plan(bad, slos))) == -3
    assert status(lambda: dyn.dyn_eval_space(prof, x, x, off, 1, 0.0, dyn.Plan(cfg, slos))) == -3
    assert status(lambda: dyn.dyn_eval_space(prof, x, x, off, 1, 100.0, dyn.Plan(cfg, slos, pct=(101, 100)))) == -3
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    assert status(lambda: dyn.dyn_eval_space(prof, x, x, off, 1, 100.0, dyn.Plan(cfg, slos), workspace=small)) == -6
    # a valid call still works afterwards
    space, ws = dyn.dyn_eval_space(prof, x, x, off, 1, 100.0, dyn.Plan(cfg, slos))
    torch.cuda.synchronize()
    prof.free()


def test_plan_changes_between_calls_are_picked_up(dyn):
    """The profile handle caches the candidate list and SLOs; changing them must take effect."""
    w = make(SPECS[0].scaled(2000, 1))
    st = oracle.ingest(w["trace"], w["edges"], 1, w["window_s"])
    ins, outs, off, _ = gpu_ingest(dyn, w)
    prof = dyn.dyn_profile_load(w["profile"])
    for it in range(3):
        w2 = dict(w)
        w2["slos"] = {"slo_ttft_ms": w["slos"]["slo_ttft_ms"] * (1 + it), "slo_tbt_ms": w["slos"]["slo_tbt_ms"] * (1 + 0.5 * it)}
        keep = np.arange(w["configs"]["n_inst"].size)[it:]
        w2["configs"] = {k: v[keep] for k, v in w["configs"].items()}
        g = gpu_eval(dyn, w2, ins, outs, off, prof=prof)
        rep = assert_parity(w2, g, ora_eval(w2, st))
        assert rep["bit_exact"] and rep["sel_mismatch"] == 0
    prof.free()


def test_calls_in_flight_on_two_streams_give_the_same_bits(dyn):
    """Steps on alternating streams with outputs and workspace of their own (one profile handle, one plan): every
    step's results equal those of a step that ran alone."""
    w = make(SPECS[2].scaled(400_000, 60))
    ins, outs, off, _ = gpu_ingest(dyn, w)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    args = (prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    ref_space, ref_sel, ref_ws = dyn.dyn_eval_select(*args)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sets = [dyn.dyn_eval_select(*args) for _ in streams]     # allocates the output sets; results overwritten below
    torch.cuda.synchronize()
    for s_ in sets:
        for d in s_[:2]:
            for v in d.values():
                v.fill_(-1 if v.dtype != torch.uint8 else 255)
    torch.cuda.synchronize()
    for i in range(12):
        sp, se, ws = sets[i % 2]
        dyn.dyn_eval_select(*args, out=sp, sel=se, workspace=ws, stream=streams[i % 2])
    torch.cuda.synchronize()
    for sp, se, ws in sets:
        assert dyn.dyn_workspace_status(ws) == dyn.dyn_workspace_status(ref_ws) == 0
        for k in ref_space:
            assert torch.equal(sp[k], ref_space[k]), k
        for k in ref_sel:
            assert torch.equal(se[k], ref_sel[k]), k
    prof.free()


def test_tuned_block_shape_changes_no_result(dyn):
    """dyn_eval_tune picks how many windows a block of the evaluation kernel walks; every output stays bit-equal, the
    choice sticks to the candidate list and is dropped when the list changes."""
    w = make(SPECS[2].scaled(600_000, 90))
    st = oracle.ingest(w["trace"], w["edges"], w["n_window"], w["window_s"])
    ins, outs, off, _ = gpu_ingest(dyn, w)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    args = (prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    space0, sel0, ws = dyn.dyn_eval_select(*args)
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in {**space0, **sel0}.items()}
    chosen = dyn.dyn_eval_tune(*args, out=space0, sel=sel0, workspace=ws)
    assert 1 <= chosen <= 32
    torch.cuda.synchronize()
    for k, v in {**space0, **sel0}.items():
        assert torch.equal(v, ref[k]), k
    space1, sel1, _ = dyn.dyn_eval_select(*args)
    space2, _ = dyn.dyn_eval_space(*args)
    torch.cuda.synchronize()
    for k, v in {**space1, **sel1}.items():
        assert torch.equal(v, ref[k]), k
    for k, v in space2.items():
        assert torch.equal(v, ref[k]), k
    o = ora_eval(w, st)
    np.testing.assert_array_equal(sel1["sel"].cpu().numpy(), o["sel"])
    np.testing.assert_array_equal(space1["energy_j"].cpu().numpy(), o["energy_j"])
    # another candidate list: the rule's shape again, same results as the oracle's
    w2 = dict(w); w2["configs"] = {k: v[5:].copy() for k, v in w["configs"].items()}
    g = gpu_eval(dyn, w2, ins, outs, off, prof=prof)
    rep = assert_parity(w2, g, ora_eval(w2, st))
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0
    prof.free()


# ------------------------------------------------------------- full size, every cell
def _excused(w, o_row, k_gpu, k_ora, g):
    """The stated tolerance for a differing selection: both candidates feasible for the oracle and their oracle costs
    within 1e-9 relative, or an oracle value of one of them within 1e-9 of a threshold (SLO, last load point)."""
    if k_gpu < 0 or k_ora < 0:
        ks = [k for k in (k_gpu, k_ora) if k >= 0]
    else:
        if (o_row["flags"][k_gpu] & 1) and abs(o_row["cost"][k_gpu] - o_row["cost"][k_ora]) <= RTOL * abs(o_row["cost"][k_ora]):
            return True
        ks = [k_gpu, k_ora]
    st, sb = w["slos"]["slo_ttft_ms"][g], w["slos"]["slo_tbt_ms"][g]
    return any(abs(o_row["p99_ttft_ms"][k] - st) <= RTOL * st or abs(o_row["p99_tbt_ms"][k] - sb) <= RTOL * sb for k in ks)


def compare_every_cell(w, st, g_sel, g_stats, o):
    """g_sel: sel / sel_energy_j / sel_cost / window_* of the GPU (NumPy); g_stats: (tin, tout, in_p99); o: the
    oracle over every cell.  Returns the counts the benchmark also prints."""
    G, NW = w["n_class"], w["n_window"]
    np.testing.assert_array_equal(g_stats[0], o["tin"])
    np.testing.assert_array_equal(g_stats[1], o["tout"])
    np.testing.assert_array_equal(g_stats[2], o["in_p99"])
    bad = np.nonzero(g_sel["sel"] != o["sel"])[0]
    excused = 0
    if bad.size:
        ob = oracle.evaluate(w["profile"], st, NW, w["window_s"], w["configs"], w["slos"], w["pct"], None,
                             w["idle_cost_weight"], cell_ids=bad.astype(np.int64))
        for i, c in enumerate(bad):
            row = {k: ob[k][i] for k in ("flags", "cost", "p99_ttft_ms", "p99_tbt_ms")}
            assert _excused(w, row, int(g_sel["sel"][c]), int(o["sel"][c]), int(c % G)), f"cell {c}: selection differs"
            excused += 1
    same = g_sel["sel"] == o["sel"]
    fin = same & (o["sel"] >= 0)
    for k in ("sel_energy_j", "sel_cost"):
        a, b = g_sel[k][fin], o[k][fin]
        assert np.all(np.abs(a - b) <= RTOL * np.abs(b)), k
        assert np.all(np.isinf(g_sel[k][same & (o["sel"] < 0)]))
    we, wi = oracle.window_totals(o["sel"], o["sel_energy_j"], NW, G)
    clean = np.ones(NW, bool)
    clean[np.unique(bad // G)] = False
    assert np.all(np.abs(g_sel["window_energy_j"][clean] - we[clean]) <= RTOL * np.abs(we[clean]))
    np.testing.assert_array_equal(g_sel["window_infeasible"][clean], wi[clean])
    bit_equal = bool(np.array_equal(g_sel["sel_energy_j"][same], o["sel_energy_j"][same]) and
                     np.array_equal(g_sel["sel_cost"][same], o["sel_cost"][same]) and
                     np.array_equal(g_sel["window_energy_j"][clean], we[clean]))
    return {"cells": int(o["sel"].size), "sel_mismatch": int(bad.size), "excused": excused, "bit_equal": bit_equal}


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_full_size_every_cell_against_the_oracle(dyn, idx):
    """The named workloads at full size (one hour, one day, one week, one week with four models) in the launch
    configuration the benchmark times.  The oracle ingests the raw trace itself and evaluates EVERY cell (its windows
    dealt to the host's cores); compared: the sorted trace and offsets bit for bit, per cell the token sums, the
    P99 input length, the selected configuration, its energy and cost, per window the totals.  On a sample of cells
    the whole evaluated space is compared element by element as well."""
    w = make(SPECS[idx])
    tr = w["trace"]
    G, NW, K = w["n_class"], w["n_window"], w["configs"]["n_inst"].size
    cells = G * NW
    st = oracle.ingest(tr, w["edges"], NW, w["window_s"])               # the oracle's own ingestion of the raw trace
    ins, outs, off, ws_i = gpu_ingest(dyn, w)
    assert dyn.dyn_workspace_status(ws_i) == 0
    del ws_i
    assert torch.equal(off.cpu(), torch.from_numpy(st["cell_off"]))
    assert torch.equal(ins.cpu(), torch.from_numpy(st["in_tok"]))
    assert torch.equal(outs.cpu(), torch.from_numpy(st["out_tok"]))
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    space, sel, ws = dyn.dyn_eval_select(prof, ins, outs, off, NW, w["window_s"], plan)
    assert dyn.dyn_workspace_status(ws) == 0
    tin, tout, p99 = dyn.dyn_cell_stats(ws, NW, G)
    torch.cuda.synchronize()
    o = oracle.evaluate_parallel(w["profile"], st, NW, w["window_s"], w["configs"], w["slos"], w["pct"], None,
                                 w["idle_cost_weight"])
    g_sel = {k: v.cpu().numpy() for k, v in sel.items()}
    rep = compare_every_cell(w, st, g_sel, (tin.cpu().numpy(), tout.cpu().numpy(), p99.cpu().numpy()), o)
    print(f"workload {idx} every cell:", rep, "oracle threads", o["threads"])
    assert rep["sel_mismatch"] == 0 and rep["bit_equal"]
    # the evaluated space element by element on a sample: largest cell, empty cells, cells the whole block takes, random
    m = np.diff(st["cell_off"])
    rng = np.random.default_rng(idx)
    ids = np.unique(np.concatenate([[0, cells - 1, int(np.argmax(m))], np.nonzero(m == 0)[0][:4], np.nonzero(m == 1)[0][:3],
                                    np.nonzero(m > 2048)[0][:3], rng.integers(0, cells, 40)])).astype(np.int64)
    os_ = ora_eval(w, st, cell_ids=ids)
    idt = torch.from_numpy(ids).cuda()
    g_ = {k: v.index_select(0, idt).cpu().numpy() for k, v in space.items()}
    g_.update({k: sel[k].index_select(0, idt).cpu().numpy() for k in ("sel", "sel_energy_j", "sel_cost")})
    g_.update(tin=tin.index_select(0, idt).cpu().numpy(), tout=tout.index_select(0, idt).cpu().numpy(),
              in_p99=p99.index_select(0, idt).cpu().numpy())
    rep = assert_parity(w, g_, os_, check_windows=False)
    assert rep["bit_exact"] and rep["sel_mismatch"] == 0
    # the selection is the argmin of the evaluated space (over every cell, on the device)
    s_ = sel["sel"].long()
    has = s_ >= 0
    rows = torch.nonzero(has).squeeze(1)
    assert bool(((space["flags"][rows, s_[rows]] & 1) == 1).all())                  # infeasible is never selected
    assert bool((space["energy_j"][rows, s_[rows]] == sel["sel_energy_j"][rows]).all())
    assert bool(((space["flags"] & 1).any(dim=1) == has).all())
    assert bool((((space["flags"] & 32) != 0).all(dim=1) == torch.from_numpy(m == 0).cuda()).all())
    if idx <= 2:        # the two-call route (dyn_eval_space, dyn_select_config) gives the same bits at this size too
        space2 = {k: torch.empty_like(v) for k, v in space.items()}
        dyn.dyn_eval_space(prof, ins, outs, off, NW, w["window_s"], plan, out=space2, workspace=ws)
        sel2 = dyn.dyn_select_config(prof, space2, NW, w["window_s"], plan)
        for k in space:
            assert torch.equal(space2[k], space[k]), k
        for k in sel:
            assert torch.equal(sel2[k], sel[k]), k
    prof.free()
