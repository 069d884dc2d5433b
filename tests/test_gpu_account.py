"""Cost and carbon of a selection on a real MI355X against the CPU oracle."""
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


@pytest.mark.parametrize("idx,n_req,n_win", [(1, 50_000, 37), (2, 200_000, 130), (4, 150_000, 21)])
def test_account_matches_oracle(dyn, idx, n_req, n_win):
    w = make(SPECS[idx].scaled(n_req, n_win))
    tr = w["trace"]
    NW, G, W = w["n_window"], w["n_class"], w["window_s"]
    ins, outs, off, _ = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]), _dev(tr["model"]),
                                             w["edges"], NW, W)
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    _, sel, _ = dyn.dyn_eval_select(prof, ins, outs, off, NW, W, plan)
    rng = np.random.default_rng(idx)
    ci = rng.uniform(80.0, 700.0, NW)                      # synthetic grid carbon intensity, g/kWh
    out, ws = dyn.dyn_account(prof, sel["sel"], sel["window_energy_j"], plan, NW, W, 11.06, 0.0832, _dev(ci), 8)
    assert dyn.dyn_workspace_status(ws) == 0
    torch.cuda.synchronize()
    o = oracle.account(w["configs"], w["profile"]["tp"], sel["sel"].cpu().numpy(), sel["window_energy_j"].cpu().numpy(), NW, G, W,
                       11.06, 0.0832, ci, 8)
    for k in ("gpus", "gpu_cost", "energy_cost", "carbon_g", "totals"):
        np.testing.assert_array_equal(out[k].cpu().numpy(), o[k], err_msg=k)
    assert o["totals"][0] > 0 and o["totals"][3] > 0
    # a selection entry the candidate list does not have is reported and counts as no selection
    bad = sel["sel"].clone()
    bad[3] = 10 ** 6
    out2, ws2 = dyn.dyn_account(prof, bad, sel["window_energy_j"], plan, NW, W, 11.06, 0.0832, _dev(ci), 8)
    assert dyn.dyn_workspace_status(ws2) == dyn.DYN_WS_BAD_REQUEST
    with pytest.raises(dyn.DynError) as e:
        dyn.dyn_account(prof, sel["sel"], sel["window_energy_j"], plan, NW, W, float("nan"), 0.1, _dev(ci), 8)
    assert e.value.status == -4
    with pytest.raises(dyn.DynError) as e:
        dyn.dyn_account(prof, sel["sel"], sel["window_energy_j"], plan, NW, W, 1.0, 0.1, _dev(ci), 0)
    assert e.value.status == -2
    prof.free()
