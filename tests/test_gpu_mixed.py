"""Mixed pools (Eq. 1 with several instance types per pool) on a real MI355X against the CPU oracle."""
import numpy as np
import pytest

import oracle
from workloads import SPECS, make

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dyn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2408_00741_amd as d
    return d


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_mixed(dyn, w, n_share, n_max, gpu_budget=None, pct=None, st=None):
    if st is None:
        tr = w["trace"]
        ins, outs, off, iws = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]),
                                                   _dev(tr["model"]), w["edges"], w["n_window"], w["window_s"])
        assert dyn.dyn_workspace_status(iws) == 0
    else:
        ins, outs, off = _dev(st["in_tok"]), _dev(st["out_tok"]), _dev(st["cell_off"])
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.MixedPlan(n_share, n_max, w["slos"], pct or w["pct"], gpu_budget)
    out, ws = dyn.dyn_eval_select_mixed(prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    status = dyn.dyn_workspace_status(ws)
    torch.cuda.synchronize()
    r = {k: v.cpu().numpy() for k, v in out.items()}
    r["status"] = status
    sorted_trace = {"in_tok": ins.cpu().numpy(), "out_tok": outs.cpu().numpy(), "cell_off": off.cpu().numpy()}
    prof.free()
    return r, sorted_trace


def check(w, g, o, n_share, n_max, gpu_budget):
    """Energies bit-equal; the assignment equal where the optimum is unique, else a valid optimal one: its
    entries of the oracle's per-type table add up (in type order, from zero) to the same energy, within the
    budget, with all shares assigned."""
    assert g["status"] == 0
    np.testing.assert_array_equal(g["energy_j"], o["energy_j"])
    fin = np.isfinite(o["energy_j"])
    uniq = fin & (o["n_optimal"] == 1)
    for k in ("n_inst", "f_index", "share"):
        np.testing.assert_array_equal(g[k][uniq], o[k][uniq], err_msg=k)
        np.testing.assert_array_equal(g[k][~fin], o[k][~fin], err_msg=k)       # 0 / -1 / 0 where nothing is feasible
    tp = w["profile"]["tp"]
    n_max = np.asarray(n_max)
    offs = np.concatenate([[0], np.cumsum(n_max * n_share)])
    G = w["n_class"]
    for c in np.nonzero(fin & ~uniq)[0]:
        e = 0.0
        for i in range(tp.size):
            n, a = int(g["n_inst"][c, i]), int(g["share"][c, i])
            assert (n > 0) == (a > 0) and 0 <= n <= n_max[i]
            if n:
                ent = offs[i] + (n - 1) * n_share + a - 1
                e += o["type_energy"][c, ent]
                assert g["f_index"][c, i] == o["type_f"][c, ent]
            else:
                assert g["f_index"][c, i] == -1
        assert e == o["energy_j"][c]
        assert g["share"][c].sum() == n_share
        if gpu_budget is not None and gpu_budget[c % G] > 0:
            assert (g["n_inst"][c] * tp).sum() <= gpu_budget[c % G]
    we, wi = oracle.window_totals(np.where(fin, 0, -1).astype(np.int32), o["energy_j"], w["n_window"], G)
    np.testing.assert_array_equal(g["window_energy_j"], we)
    np.testing.assert_array_equal(g["window_infeasible"], wi)
    return int(uniq.sum()), int((fin & ~uniq).sum()), int((~fin).sum())


CASES = {
    # name: (spec, shares, instances per type, budget per class or None)
    "cfg0-S4": (SPECS[0], 4, 4, 24),
    "cfg1-6k-S8": (SPECS[1].scaled(6000, 6), 8, 5, None),
    "cfg2-30k-S8": (SPECS[2].scaled(30_000, 4), 8, 6, 32),
    "cfg3-20k-S3": (SPECS[3].scaled(20_000, 3), 3, 8, 40),
    "cfg4-25k-S5": (SPECS[4].scaled(25_000, 2), 5, 4, None),
}


@pytest.mark.parametrize("name", list(CASES))
def test_mixed_matches_oracle(dyn, name):
    spec, S, nm, bud = CASES[name]
    w = make(spec)
    T = w["profile"]["tp"].size
    n_max = [nm] * T
    budget = None if bud is None else np.full(w["n_class"], bud, np.int32)
    g, st = gpu_mixed(dyn, w, S, n_max, budget)
    o = oracle.mixed(w["profile"], st, w["n_window"], w["window_s"], S, n_max, w["slos"], w["pct"], budget,
                     want_types=True)
    rep = check(w, g, o, S, n_max, budget)
    print(name, "unique / tied / infeasible cells:", rep)
    assert rep[0] > 0
    assert (o["n_inst"] > 0).sum(axis=1).max() >= 1


def test_many_instances_of_one_type(dyn):
    """240 instances allowed for the smallest type: the per-type capacities no longer fit in LDS beside the table rows
    (64 load points per row: 18 KB of rows + 46 KB of capacities) and the per-type energies come from the kernel that
    forms them per lane; a budget keeps the assignment small."""
    w = make(SPECS[2].scaled(6000, 4))
    T = w["profile"]["tp"].size
    S = 2
    n_max = [240] + [2] * (T - 1)
    budget = np.full(w["n_class"], 24, np.int32)
    g, st = gpu_mixed(dyn, w, S, n_max, budget)
    o = oracle.mixed(w["profile"], st, w["n_window"], w["window_s"], S, n_max, w["slos"], w["pct"], budget, want_types=True)
    rep = check(w, g, o, S, n_max, budget)
    print("unique / tied / infeasible cells:", rep)
    assert rep[0] > 0


def _random_case(seed):
    rng = np.random.default_rng(1100 + seed)
    n_tp, n_f, n_rho, G = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(2, 9)), 3
    fg = np.sort(rng.uniform(500, 2000, n_f))
    rg = np.concatenate([[0.0], np.sort(rng.uniform(0.05, 0.95, n_rho - 1))])
    shape = (G, n_tp, n_f, n_rho)
    prof = {"tp": np.asarray([1, 2, 4, 8][:n_tp], np.int32) * int(rng.integers(1, 3)), "f_mhz": fg, "rho": rg,
            "prefill_ms_per_tok": rng.uniform(0.05, 0.3, shape), "tbt_ms": np.sort(rng.uniform(10, 150, shape), axis=-1),
            "power_w": np.sort(rng.uniform(100, 3000, shape), axis=-1), "max_load_tps": rng.uniform(50, 400, shape[:3])}
    NW, W, R = 4, 20.0, 900
    tr = {"t_s": rng.uniform(0, NW * W, R), "in_tok": rng.integers(0, 600, R).astype(np.int32),
          "out_tok": rng.integers(1, 300, R).astype(np.int32), "model": np.zeros(R, np.int32)}
    tr["t_s"][tr["t_s"] > 3 * W] = 5.0                    # the last window is empty
    w = {"profile": prof, "trace": tr, "n_window": NW, "window_s": W, "n_class": G,
         "edges": {"in_edge": np.asarray([[150, 350]], np.int32), "out_edge": np.zeros((1, 0), np.int32)},
         "slos": {"slo_ttft_ms": rng.uniform(30, 150, G), "slo_tbt_ms": rng.uniform(40, 140, G)}, "pct": (99, 100)}
    n_max = rng.integers(0, 7, n_tp)
    n_max[int(rng.integers(0, n_tp))] = max(1, int(n_max.max()))
    S = int(rng.integers(1, 9))
    bud = rng.choice([0, 6, 16, 40], G).astype(np.int32)
    return w, S, n_max.tolist(), bud


@pytest.mark.parametrize("seed", range(8))
def test_random_profiles_types_and_budgets(dyn, seed):
    w, S, n_max, bud = _random_case(seed)
    g, st = gpu_mixed(dyn, w, S, n_max, bud)
    o = oracle.mixed(w["profile"], st, w["n_window"], w["window_s"], S, n_max, w["slos"], w["pct"], bud, want_types=True)
    rep = check(w, g, o, S, n_max, bud)
    print("seed", seed, "tp", w["profile"]["tp"], "S", S, "n_max", n_max, "->", rep)


def test_one_share_equals_window_level_selection(dyn):
    """With one share the whole load goes to one type: the result is dyn_eval_select's over the candidates
    (instances, TP, profiled frequency) under the same budget."""
    w = make(SPECS[1].scaled(20_000, 5))
    prof_h = w["profile"]
    T, nm = prof_h["tp"].size, 6
    cfg = {"n_inst": [], "tp_index": [], "f_mhz": []}
    for ti in range(T):
        for n in range(1, nm + 1):
            for f in prof_h["f_mhz"]:
                cfg["n_inst"].append(n); cfg["tp_index"].append(ti); cfg["f_mhz"].append(f)
    cfg = {k: np.asarray(v, np.int32 if k != "f_mhz" else np.float64) for k, v in cfg.items()}
    bud = np.full(w["n_class"], 16, np.int32)
    g, st = gpu_mixed(dyn, w, 1, [nm] * T, bud)
    prof = dyn.dyn_profile_load(prof_h)
    plan = dyn.Plan(cfg, w["slos"], w["pct"], bud, 0.0)
    _, sel, _ = dyn.dyn_eval_select(prof, _dev(st["in_tok"]), _dev(st["out_tok"]), _dev(st["cell_off"]), w["n_window"],
                                    w["window_s"], plan)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(g["energy_j"], sel["sel_energy_j"].cpu().numpy())
    np.testing.assert_array_equal(g["window_energy_j"], sel["window_energy_j"].cpu().numpy())
    np.testing.assert_array_equal(g["window_infeasible"], sel["window_infeasible"].cpu().numpy())
    prof.free()


def test_argument_errors(dyn):
    w = make(SPECS[0])
    st = oracle.ingest(w["trace"], w["edges"], w["n_window"], w["window_s"])
    ins, outs, off = _dev(st["in_tok"]), _dev(st["out_tok"]), _dev(st["cell_off"])
    prof = dyn.dyn_profile_load(w["profile"])
    T = w["profile"]["tp"].size
    for S, nm, status in ((0, [2] * T, -2), (17, [2] * T, -2), (4, [0] * T, -2), (4, [300] + [1] * (T - 1), -3),
                          (16, [255] * T, -2)):            # the last one: state too large for LDS without a budget
        plan = dyn.MixedPlan(S, nm, w["slos"])
        assert dyn.dyn_mixed_workspace(prof, w["n_window"], plan) == 0 or status == -2 and S == 16
        ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
        with pytest.raises(dyn.DynError) as e:
            dyn.dyn_eval_select_mixed(prof, ins, outs, off, w["n_window"], w["window_s"], plan, workspace=ws)
        assert e.value.status == status, (S, nm, dyn.dyn_last_error())
    plan = dyn.MixedPlan(4, [2] * T, w["slos"])
    with pytest.raises(dyn.DynError) as e:
        dyn.dyn_eval_select_mixed(prof, ins, outs, off, w["n_window"], w["window_s"], plan,
                                  workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -6
    out, _ = dyn.dyn_eval_select_mixed(prof, ins, outs, off, w["n_window"], w["window_s"], plan)
    torch.cuda.synchronize()
    assert np.isfinite(out["energy_j"].cpu().numpy()).any()
    prof.free()


def test_full_size_day_trace_sampled_windows(dyn):
    """The one-day workload at full size (36000 cells) in the configuration the benchmark's --mixed mode times:
    8 shares, a budget of 32 GPUs per class, up to 32/TP instances per type.  The oracle evaluates three runs of
    windows; the rest is checked through properties that hold at any size."""
    w = make(SPECS[2])
    S, gpus = 8, 32
    tp = w["profile"]["tp"]
    n_max = [gpus // int(t) for t in tp]
    NW, G = w["n_window"], w["n_class"]
    bud = np.full(G, gpus, np.int32)
    g, st = gpu_mixed(dyn, w, S, n_max, bud)
    assert g["status"] == 0
    off = st["cell_off"]
    m = np.diff(off).reshape(NW, G)
    peak = int(np.argmax(m.sum(axis=1)))
    seen_mix = 0
    for wa in (0, max(0, min(NW - 4, peak - 2)), NW - 4):
        wb = wa + 4
        lo, hi = wa * G, wb * G
        sub = {"in_tok": st["in_tok"][off[lo]:off[hi]], "out_tok": st["out_tok"][off[lo]:off[hi]],
               "cell_off": off[lo:hi + 1] - off[lo]}
        w4 = dict(w, n_window=wb - wa)
        o = oracle.mixed(w["profile"], sub, wb - wa, w["window_s"], S, n_max, w["slos"], w["pct"], bud, want_types=True)
        gs = {k: (v[lo:hi] if k not in ("window_energy_j", "window_infeasible", "status") else v) for k, v in g.items()}
        gs["window_energy_j"], gs["window_infeasible"] = g["window_energy_j"][wa:wb], g["window_infeasible"][wa:wb]
        check(w4, gs, o, S, n_max, bud)
        seen_mix += int(((o["n_inst"] > 0).sum(axis=1) > 1).sum())
    print("cells with more than one type among the sampled windows:", seen_mix)
    fin = np.isfinite(g["energy_j"])
    used = g["n_inst"] > 0
    assert (g["share"][fin].sum(axis=1) == S).all() and ((g["share"] > 0) == used).all() and ((g["f_index"] >= 0) == used).all()
    assert ((g["n_inst"] * tp[None, :]).sum(axis=1) <= gpus).all()
    assert (g["n_inst"][~fin] == 0).all()
    we = np.where(fin, g["energy_j"], 0.0).reshape(NW, G)
    assert np.all(np.abs(g["window_energy_j"] - we.sum(axis=1)) <= 1e-12 * we.sum(axis=1))
    np.testing.assert_array_equal(g["window_infeasible"], (~fin).reshape(NW, G).sum(axis=1))
    # the mix never costs more than the window-level selection over single-type candidates within the same budget
    cfg = {"n_inst": [], "tp_index": [], "f_mhz": []}
    for ti in range(tp.size):
        for n in range(1, n_max[ti] + 1):
            for f in w["profile"]["f_mhz"]:
                cfg["n_inst"].append(n); cfg["tp_index"].append(ti); cfg["f_mhz"].append(f)
    cfg = {k: np.asarray(v, np.int32 if k != "f_mhz" else np.float64) for k, v in cfg.items()}
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(cfg, w["slos"], w["pct"], bud, 0.0)
    _, sel, _ = dyn.dyn_eval_select(prof, _dev(st["in_tok"]), _dev(st["out_tok"]), _dev(off), NW, w["window_s"], plan)
    torch.cuda.synchronize()
    single = sel["sel_energy_j"].cpu().numpy()
    assert (g["energy_j"] <= single).all()
    print("cells where the mix beats every single type: %d of %d; feasible only as a mix: %d" %
          (int((g["energy_j"] < single).sum()), fin.sum(), int((fin & ~np.isfinite(single)).sum())))
    prof.free()


@pytest.mark.parametrize("seed", range(4))
def test_tiny_pools_against_the_unfactored_product(dyn, seed):
    """The GPU against a search that factors nothing (Eq. 1 with several types per pool): every (instances,
    frequency, shares) of every type in one product, NumPy arithmetic, no code shared with the oracle.  The
    sums are formed in another order there, hence the relative tolerance of a few ulps on the energy; the
    assignment must be one of the product's optimal ones."""
    from tests import npcheck
    rng = np.random.default_rng(900 + seed)
    n_tp, n_f, n_rho, G = 2 + seed % 2, 1 + seed % 3, 3, 2
    fg = np.sort(rng.uniform(500, 2000, n_f))
    rg = np.concatenate([[0.0], np.sort(rng.uniform(0.1, 0.95, n_rho - 1))])
    shape = (G, n_tp, n_f, n_rho)
    prof = {"tp": np.asarray([2, 4, 8][:n_tp], np.int32), "f_mhz": fg, "rho": rg,
            "prefill_ms_per_tok": rng.uniform(0.05, 0.3, shape), "tbt_ms": np.sort(rng.uniform(10, 150, shape), axis=-1),
            "power_w": np.sort(rng.uniform(100, 3000, shape), axis=-1), "max_load_tps": rng.uniform(200, 900, shape[:3])}
    R, NW, W = 60, 2, 10.0
    tr = {"t_s": rng.uniform(0, NW * W, R), "in_tok": rng.integers(1, 400, R).astype(np.int32),
          "out_tok": rng.integers(1, 200, R).astype(np.int32), "model": np.zeros(R, np.int32)}
    tr["t_s"][tr["t_s"] > 15.0] = 1.0
    edges = {"in_edge": np.asarray([[150]], np.int32), "out_edge": np.zeros((1, 0), np.int32)}
    slo = {"slo_ttft_ms": rng.uniform(40, 120, G), "slo_tbt_ms": rng.uniform(60, 140, G)}
    bud = np.asarray([0, 10], np.int32)
    n_max = [2, 2, 1][:n_tp]
    S = 3
    w = {"trace": tr, "edges": edges, "n_window": NW, "window_s": W, "profile": prof, "slos": slo, "pct": (99, 100),
         "n_class": G}
    g, _ = gpu_mixed(dyn, w, S, n_max, bud)
    assert g["status"] == 0
    b = npcheck.np_mixed(prof, npcheck.np_ingest(tr, edges, NW, W), NW, W, S, n_max, slo, (99, 100), bud)
    fin = np.isfinite(b["energy_j"])
    assert (np.isfinite(g["energy_j"]) == fin).all() and fin.any()
    np.testing.assert_allclose(g["energy_j"][fin], b["energy_j"][fin], rtol=1e-12)
    for c in np.nonzero(fin)[0]:
        assert tuple(zip(g["n_inst"][c].tolist(), g["share"][c].tolist())) in b["assignments"][c]
