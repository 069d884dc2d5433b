"""Selection with transition overheads between consecutive windows on a real MI355X against the CPU oracle."""
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


def total_of(cost, feas, sel, lay, tr, NW, G, g):
    """Total of the sequence(s) `sel` describes for class g, in the definition's order of additions; also checks
    that every choice is feasible and that -1 appears exactly where nothing is feasible."""
    total, run = 0.0, None
    prev = -1
    for w in range(NW):
        c = w * G + g
        k = int(sel[c])
        if not feas[c].any():
            assert k == -1
            if run is not None:
                total += run
                run = None
            prev = -1
            continue
        assert k >= 0 and feas[c, k]
        run = cost[c, k] if run is None else (run + tr[lay[prev], lay[k]]) + cost[c, k]
        prev = k
    if run is not None:
        total += run
    return total


def run_path(dyn, prof, plan, energy, flags, NW, W, lay, tr):
    space = {"energy_j": _dev(energy), "flags": _dev(flags)}
    out, ws = dyn.dyn_select_path(prof, space, NW, W, plan, lay, tr)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def check(g, o_sel, o_pc, cost, feas, energy, lay, tr, NW, G):
    np.testing.assert_array_equal(g["path_cost"], o_pc)
    same = 0
    for cls in range(G):
        assert total_of(cost, feas, g["sel"], lay, tr, NW, G, cls) == o_pc[cls]
        same += int(np.array_equal(g["sel"][cls::G], o_sel[cls::G]))
    has = g["sel"] >= 0
    np.testing.assert_array_equal(g["sel_energy_j"][has], energy[np.nonzero(has)[0], g["sel"][has]])
    assert np.isinf(g["sel_energy_j"][~has]).all()
    we, wi = oracle.window_totals(g["sel"], g["sel_energy_j"], NW, G)
    np.testing.assert_array_equal(g["window_energy_j"], we)
    np.testing.assert_array_equal(g["window_infeasible"], wi)
    return same


def _layouts(cfg):
    """Layout = (TP degree, instances): frequency changes are free."""
    key = cfg["tp_index"].astype(np.int64) * 1000 + cfg["n_inst"]
    uniq, lay = np.unique(key, return_inverse=True)
    return lay.astype(np.int32), uniq


CASES = {
    "cfg1-6k": (SPECS[1].scaled(6000, 24), 0.0),
    "cfg2-40k": (SPECS[2].scaled(40_000, 30), 0.0),
    "cfg3-30k-idle": (SPECS[3].scaled(30_000, 12), 0.05),
}


@pytest.mark.parametrize("name", list(CASES))
def test_path_matches_oracle_on_evaluated_spaces(dyn, name):
    spec, lam = CASES[name]
    w = make(spec)
    cfg = w["configs"]
    if cfg["n_inst"].size > 600:                     # keep the per-class state (layouts^2) within LDS
        keep = cfg["n_inst"] <= 16
        cfg = {k: v[keep] for k, v in cfg.items()}
    NW, G, W = w["n_window"], w["n_class"], w["window_s"]
    st = oracle.ingest(w["trace"], w["edges"], NW, W)
    o = oracle.evaluate(w["profile"], st, NW, W, cfg, w["slos"], w["pct"], None, lam)
    feas = (o["flags"] & 1).astype(np.uint8)
    lay, uniq = _layouts(cfg)
    NL = uniq.size
    gpus = (uniq // 1000 + 1) * 2 * (uniq % 1000)          # rough size of a layout
    rng = np.random.default_rng(7)
    scale = np.median(o["sel_cost"][np.isfinite(o["sel_cost"])]) * 0.02
    tr = scale * np.abs(gpus[:, None] - gpus[None, :]) * rng.uniform(0.5, 1.5, (NL, NL))
    tr[np.diag_indices(NL)] = 0.0
    o_sel, o_pc = oracle.select_path(o["cost"], feas, NW, G, lay, tr)
    assert (o_sel != o["sel"]).any(), "the transition costs are meant to change some choices"

    ins, outs, off = _dev(st["in_tok"]), _dev(st["out_tok"]), _dev(st["cell_off"])
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(cfg, w["slos"], w["pct"], None, lam)
    space, _ = dyn.dyn_eval_space(prof, ins, outs, off, NW, W, plan)
    out, _ = dyn.dyn_select_path(prof, space, NW, W, plan, lay, tr)
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in out.items()}
    same = check(g, o_sel, o_pc, o["cost"], feas, o["energy_j"], lay, tr, NW, G)
    print(name, "classes with the oracle's exact sequence:", same, "of", G, "; layouts", NL)
    # without overheads the result is the per-window selection
    out0, _ = dyn.dyn_select_path(prof, space, NW, W, plan, lay, np.zeros((NL, NL)))
    sel0 = dyn.dyn_select_config(prof, space, NW, W, plan)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out0["sel"].cpu().numpy(), sel0["sel"].cpu().numpy())
    np.testing.assert_array_equal(out0["window_energy_j"].cpu().numpy(), sel0["window_energy_j"].cpu().numpy())
    prof.free()


@pytest.mark.parametrize("seed", range(8))
def test_random_spaces_with_gaps(dyn, seed):
    """Arbitrary evaluated spaces fed through the ABI: windows without any feasible candidate, many exact ties
    (costs on a coarse grid), one layout, one candidate."""
    rng = np.random.default_rng(1500 + seed)
    w = make(SPECS[0])
    G = w["n_class"]
    NW = int(rng.integers(1, 200))
    K = int(rng.choice([1, 2, 7, 64, 257, 700]))
    NL = int(rng.integers(1, min(K, 40) + 1))
    cfg = {"n_inst": rng.integers(1, 5, K).astype(np.int32), "tp_index": rng.integers(0, w["profile"]["tp"].size, K).astype(np.int32),
           "f_mhz": rng.choice(w["profile"]["f_mhz"], K)}
    coarse = seed % 2 == 0
    energy = np.round(rng.uniform(1, 50, (NW * G, K)), 0 if coarse else 6)
    flags = np.where(rng.uniform(0, 1, (NW * G, K)) < 0.6, 1, 4).astype(np.uint8)
    for _ in range(NW // 10 + 1):                      # gaps
        flags[int(rng.integers(0, NW)) * G + int(rng.integers(0, G))] = 8
    lay = rng.integers(0, NL, K).astype(np.int32)
    tr = np.round(rng.uniform(0, 6, (NL, NL)), 0 if coarse else 6)
    tr[np.diag_indices(NL)] = 0.0
    feas = (flags & 1).astype(np.uint8)
    o_sel, o_pc = oracle.select_path(energy, feas, NW, G, lay, tr)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(cfg, w["slos"], w["pct"], None, 0.0)
    g = run_path(dyn, prof, plan, energy, flags, NW, 60.0, lay, tr)
    same = check(g, o_sel, o_pc, energy, feas, energy, lay, tr, NW, G)
    print("seed", seed, "NW", NW, "K", K, "layouts", NL, "exact sequences:", same, "of", G)
    prof.free()


def test_full_size_day_trace(dyn):
    """The one-day workload at full size (1440 windows x 25 classes x 576 candidates, 48 layouts): every class's
    total and sequence against the oracle for three classes, the definition's total for all."""
    w = make(SPECS[2])
    cfg = w["configs"]
    NW, G, W, K = w["n_window"], w["n_class"], w["window_s"], cfg["n_inst"].size
    tr_ = w["trace"]
    ins, outs, off, _ = dyn.dyn_trace_ingest(_dev(tr_["t_s"]), _dev(tr_["in_tok"]), _dev(tr_["out_tok"]), _dev(tr_["model"]),
                                             w["edges"], NW, W)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(cfg, w["slos"], w["pct"], None, 0.0)
    space, _ = dyn.dyn_eval_space(prof, ins, outs, off, NW, W, plan)
    lay, uniq = _layouts(cfg)
    NL = uniq.size
    gpus = (uniq // 1000 + 1) * 2 * (uniq % 1000)
    sel0 = dyn.dyn_select_config(prof, space, NW, W, plan)
    torch.cuda.synchronize()
    e0 = sel0["sel_energy_j"].cpu().numpy()
    scale = np.median(e0[np.isfinite(e0)]) * 0.01
    tr = scale * np.abs(gpus[:, None] - gpus[None, :]).astype(float)
    out, _ = dyn.dyn_select_path(prof, space, NW, W, plan, lay, tr)
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in out.items()}
    energy = space["energy_j"].cpu().numpy()
    feas = (space["flags"].cpu().numpy() & 1).astype(np.uint8)
    for cls in range(G):                               # the definition's total of the returned sequence
        assert total_of(energy, feas, g["sel"], lay, tr, NW, G, cls) == g["path_cost"][cls]
    cls3 = [0, 11, G - 1]
    sub_e = np.ascontiguousarray(energy.reshape(NW, G, K)[:, cls3].reshape(NW * 3, K))
    sub_f = np.ascontiguousarray(feas.reshape(NW, G, K)[:, cls3].reshape(NW * 3, K))
    o_sel, o_pc = oracle.select_path(sub_e, sub_f, NW, 3, lay, tr)
    np.testing.assert_array_equal(g["path_cost"][cls3], o_pc)
    same = sum(int(np.array_equal(g["sel"][c::G], o_sel[i::3])) for i, c in enumerate(cls3))
    changes0 = int((np.diff(lay[sel0["sel"].cpu().numpy().reshape(NW, G)], axis=0) != 0).sum())
    changes1 = int((np.diff(lay[g["sel"].reshape(NW, G)], axis=0) != 0).sum())
    print("exact sequences", same, "of 3; layout changes without / with overheads:", changes0, changes1)
    assert changes1 < changes0
    # the sequence costs no more than the per-window choices charged with the same overheads, and no less than them uncharged
    for cls in range(G):
        per_window = total_of(energy, feas, sel0["sel"].cpu().numpy(), lay, tr, NW, G, cls)
        assert g["path_cost"][cls] <= per_window
        assert g["path_cost"][cls] >= e0.reshape(NW, G)[:, cls].sum() * (1 - 1e-12)
    prof.free()


@pytest.mark.parametrize("NL,K", [(64, 64), (64, 3000), (66, 300), (17, 33), (33, 500), (49, 49)])
def test_layout_counts_around_the_route_boundaries(dyn, NL, K):
    """Up to 64 layouts one wave walks a class (register tiers of 16, 32, 48 and 64 layouts, any number of
    candidates); beyond that a block does, with the candidates in registers and the overheads in LDS."""
    rng = np.random.default_rng(NL * 1000 + K)
    w = make(SPECS[0])
    G = w["n_class"]
    NW = 70
    cfg = {"n_inst": rng.integers(1, 5, K).astype(np.int32), "tp_index": rng.integers(0, w["profile"]["tp"].size, K).astype(np.int32),
           "f_mhz": rng.choice(w["profile"]["f_mhz"], K)}
    energy = np.round(rng.uniform(1, 50, (NW * G, K)), 3)
    flags = np.where(rng.uniform(0, 1, (NW * G, K)) < 0.5, 1, 4).astype(np.uint8)
    flags[(NW // 2) * G:(NW // 2) * G + G] = 8                 # one window without candidates, for every class
    lay = rng.permutation(np.arange(K) % NL).astype(np.int32)   # every layout is used
    tr = np.round(rng.uniform(0, 6, (NL, NL)), 3)
    tr[np.diag_indices(NL)] = 0.0
    feas = (flags & 1).astype(np.uint8)
    o_sel, o_pc = oracle.select_path(energy, feas, NW, G, lay, tr)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(cfg, w["slos"], w["pct"], None, 0.0)
    g = run_path(dyn, prof, plan, energy, flags, NW, 60.0, lay, tr)
    same = check(g, o_sel, o_pc, energy, feas, energy, lay, tr, NW, G)
    print("layouts", NL, "K", K, "exact sequences:", same, "of", G)
    assert same == G
    prof.free()


@pytest.mark.parametrize("NW", [1, 2, 16, 17, 63, 64, 65, 128, 129, 1089, 1200])
def test_window_counts_around_the_trace_back_runs(dyn, NW):
    """The walk visits global memory 16 windows at a time and the trace-back follows runs of 64 windows, chaining the
    runs' records 16 at a time: window counts on both sides of every one of those boundaries, with gaps in the sequences
    and ties (costs on a coarse grid)."""
    rng = np.random.default_rng(7000 + NW)
    w = make(SPECS[0])
    G = w["n_class"]
    K, NL = 24, 7
    cfg = {"n_inst": rng.integers(1, 5, K).astype(np.int32), "tp_index": rng.integers(0, w["profile"]["tp"].size, K).astype(np.int32),
           "f_mhz": rng.choice(w["profile"]["f_mhz"], K)}
    energy = np.round(rng.uniform(1, 50, (NW * G, K)), 1)
    flags = np.where(rng.uniform(0, 1, (NW * G, K)) < 0.5, 1, 4).astype(np.uint8)
    for _ in range(NW // 40 + 1):
        flags[int(rng.integers(0, NW)) * G + int(rng.integers(0, G))] = 8
    if NW > 64:
        flags[63 * G:65 * G] = 8                           # a gap on both sides of the first run boundary, every class
    lay = rng.permutation(np.arange(K) % NL).astype(np.int32)
    tr = np.round(rng.uniform(0, 6, (NL, NL)), 1)
    tr[np.diag_indices(NL)] = 0.0
    feas = (flags & 1).astype(np.uint8)
    o_sel, o_pc = oracle.select_path(energy, feas, NW, G, lay, tr)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(cfg, w["slos"], w["pct"], None, 0.0)
    g = run_path(dyn, prof, plan, energy, flags, NW, 60.0, lay, tr)
    check(g, o_sel, o_pc, energy, feas, energy, lay, tr, NW, G)
    prof.free()


def test_argument_errors(dyn):
    w = make(SPECS[0])
    K = w["configs"]["n_inst"].size
    G = w["n_class"]
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"])
    space = {"energy_j": torch.ones((2 * G, K), dtype=torch.float64, device="cuda"),
             "flags": torch.ones((2 * G, K), dtype=torch.uint8, device="cuda")}
    lay = np.zeros(K, np.int32)
    for bad_lay, bad_tr, status in ((np.full(K, 3, np.int32), np.zeros((2, 2)), -3), (lay, np.asarray([[0.0, -1.0], [0.0, 0.0]]), -3),
                                    (lay, np.asarray([[0.0, np.nan], [0.0, 0.0]]), -4), (lay, np.zeros((90, 90)), -2)):
        with pytest.raises(dyn.DynError) as e:
            dyn.dyn_select_path(prof, space, 2, 60.0, plan, bad_lay, bad_tr)
        assert e.value.status == status, dyn.dyn_last_error()
    with pytest.raises(dyn.DynError) as e:
        dyn.dyn_select_path(prof, space, 2, 60.0, plan, lay, np.zeros((1, 1)),
                            workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -6
    out, _ = dyn.dyn_select_path(prof, space, 2, 60.0, plan, lay, np.zeros((1, 1)))
    torch.cuda.synchronize()
    assert (out["sel"].cpu().numpy() == 0).all() and (out["path_cost"].cpu().numpy() == 2.0).all()
    prof.free()


@pytest.mark.parametrize("seed", range(6))
def test_tiny_spaces_against_every_sequence(dyn, seed):
    """The GPU against the definition written out (reconfiguration overheads between consecutive windows, Section
    IV-C): every sequence of feasible candidates over each run of windows is priced with itertools, sums in window
    order; the GPU's total must equal the smallest one and its sequence must be one of those that reach it."""
    import itertools
    rng = np.random.default_rng(1300 + seed)
    w = make(SPECS[0])
    G = w["n_class"]
    NW, K, NL = int(rng.integers(2, 6)), int(rng.integers(2, 5)), int(rng.integers(1, 4))
    energy = rng.uniform(1, 10, (NW * G, K))
    flags = np.where(rng.uniform(0, 1, (NW * G, K)) < 0.7, 1, 4).astype(np.uint8)
    if seed % 2:
        flags[(NW // 2) * G + 1] = 4                         # class 1 has a window without any feasible candidate
    feas = (flags & 1).astype(bool)
    lay = rng.integers(0, NL, K).astype(np.int32)
    tr = rng.uniform(0, 4, (NL, NL)); tr[np.diag_indices(NL)] = 0.0
    cfg = {"n_inst": rng.integers(1, 5, K).astype(np.int32),
           "tp_index": rng.integers(0, w["profile"]["tp"].size, K).astype(np.int32),
           "f_mhz": rng.choice(w["profile"]["f_mhz"], K)}
    prof = dyn.dyn_profile_load(w["profile"])
    r = run_path(dyn, prof, dyn.Plan(cfg, w["slos"], w["pct"], None, 0.0), energy, flags, NW, 60.0, lay, tr)
    prof.free()
    sel, pc = r["sel"], r["path_cost"]
    for g in range(G):
        ok = [feas[x * G + g].any() for x in range(NW)]
        total, x = 0.0, 0
        while x < NW:
            if not ok[x]:
                assert sel[x * G + g] == -1
                x += 1
                continue
            e = x
            while e < NW and ok[e]:
                e += 1
            best, best_seq = np.inf, []
            for seq in itertools.product(range(K), repeat=e - x):
                if not all(feas[(x + i) * G + g, k] for i, k in enumerate(seq)):
                    continue
                v = energy[x * G + g, seq[0]]
                for i in range(1, len(seq)):
                    v = (v + tr[lay[seq[i - 1]], lay[seq[i]]]) + energy[(x + i) * G + g, seq[i]]
                if v < best:
                    best, best_seq = v, [seq]
                elif v == best:
                    best_seq.append(seq)
            total += best
            assert tuple(int(sel[(x + i) * G + g]) for i in range(e - x)) in best_seq
            x = e
        assert pc[g] == total
