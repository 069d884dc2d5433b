"""The entry points enqueue on the caller's stream and return: no call waits for the device in the steady state
(same candidate list, objective and small host tables as the call before)."""
import numpy as np
import pytest

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


def _busy(ms=40.0):
    """Keeps the current stream busy for a while: a host call that waited for the stream would outlast it."""
    x = torch.empty(1 << 28, dtype=torch.float32, device="cuda")        # 1 GiB fills, a few hundred microseconds each
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(); x.fill_(1.0); e1.record()
    torch.cuda.synchronize()
    n = max(4, int(ms / max(e0.elapsed_time(e1), 1e-3)))
    return x, n


def test_ten_calls_of_every_entry_point_return_before_the_device_is_done(dyn):
    w = make(SPECS[2].scaled(400_000, 60))
    tr = w["trace"]
    NW, G, T = w["n_window"], w["n_class"], 6
    dev = [_dev(tr[k]) for k in ("t_s", "in_tok", "out_tok", "model")]
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    K = plan.K
    # reference results, and warm-up of every cache of the profile handle
    ins, outs, off, ws_i = dyn.dyn_trace_ingest(*dev, w["edges"], NW, w["window_s"])
    fin = dyn.dyn_trace_ingest(*dev, w["edges"], NW * T, w["window_s"] / T)[:3]
    space, sel, ws = dyn.dyn_eval_select(prof, ins, outs, off, NW, w["window_s"], plan)
    cfgs = w["configs"]
    uniq, lay = np.unique(cfgs["tp_index"].astype(np.int64) * 100000 + cfgs["n_inst"], return_inverse=True)
    lay = lay.astype(np.int32)
    gpus = w["profile"]["tp"][uniq // 100000].astype(np.int64) * (uniq % 100000)
    trans = 1000.0 * np.abs(gpus[:, None] - gpus[None, :]).astype(np.float64)
    psel, ws_p = dyn.dyn_select_path(prof, space, NW, w["window_s"], plan, lay, trans)
    lay_n, lay_tp = (uniq % 100000).astype(np.int32), (uniq // 100000).astype(np.int32)
    hargs = (NW, T, w["window_s"] / T, 6, int(w["profile"]["tp"].size) - 1, int(w["profile"]["f_mhz"].size) - 1, 8, lay_n, lay_tp,
             w["slos"], w["pct"])
    hout, ws_h = dyn.dyn_hierarchy(prof, (ins, outs, off), fin, *hargs, transition_j=trans)
    tsp, tse, ws_t = dyn.dyn_eval_select_ticks(prof, *fin, NW, T, w["window_s"] / T, plan)
    torch.cuda.synchronize()
    ref = {"ingest": [t.clone() for t in (ins, outs, off)], "sel": {k: v.clone() for k, v in sel.items()},
           "psel": {k: v.clone() for k, v in psel.items()}, "hout": {k: v.clone() for k, v in hout.items()},
           "tse": {k: v.clone() for k, v in tse.items()}}

    filler, n_fill = _busy()
    done = torch.cuda.Event()
    for _ in range(n_fill):
        filler.fill_(2.0)
    for _ in range(10):
        i2 = dyn.dyn_trace_ingest(*dev, w["edges"], NW, w["window_s"], workspace=ws_i)
        dyn.dyn_eval_select(prof, ins, outs, off, NW, w["window_s"], plan, out=space, sel=sel, workspace=ws)
        dyn.dyn_select_path(prof, space, NW, w["window_s"], plan, lay, trans, out=psel, workspace=ws_p)
        dyn.dyn_hierarchy(prof, (ins, outs, off), fin, *hargs, out=hout, workspace=ws_h, transition_j=trans)
        dyn.dyn_eval_select_ticks(prof, *fin, NW, T, w["window_s"] / T, plan, out=tsp, sel=tse, workspace=ws_t)
    done.record()
    returned_early = not done.query()        # the host is back while the device still has work queued
    torch.cuda.synchronize()
    assert returned_early, "an entry point waited for the stream"
    for a, b in zip(i2[:3], ref["ingest"]):
        assert torch.equal(a, b)
    for got, want in ((sel, ref["sel"]), (psel, ref["psel"]), (hout, ref["hout"]), (tse, ref["tse"])):
        for k in want:
            assert torch.equal(got[k], want[k]), k
    assert dyn.dyn_workspace_status(ws_i) == 0 and dyn.dyn_workspace_status(ws) == 0 and dyn.dyn_workspace_status(ws_t) == 0
    prof.free()


def test_ingest_picks_its_route_on_the_device(dyn):
    """A trace in window order and the same trace shuffled through one workspace, one after the other, without a
    host synchronisation in between: each call takes its own route and both give the stable order by cell."""
    w = make(SPECS[1].scaled(120_000, 11))
    tr = w["trace"]
    perm = np.random.default_rng(3).permutation(tr["t_s"].size)
    a = [_dev(tr[k]) for k in ("t_s", "in_tok", "out_tok", "model")]
    b = [_dev(tr[k][perm]) for k in ("t_s", "in_tok", "out_tok", "model")]
    ws = torch.empty(dyn.dyn_trace_ingest_workspace(tr["t_s"].size, 11, w["n_class"]), dtype=torch.uint8, device="cuda")
    ra = dyn.dyn_trace_ingest(*a, w["edges"], 11, w["window_s"], workspace=ws)
    rb = dyn.dyn_trace_ingest(*b, w["edges"], 11, w["window_s"], workspace=ws)
    rc = dyn.dyn_trace_ingest(*a, w["edges"], 11, w["window_s"], workspace=ws)
    torch.cuda.synchronize()
    import oracle
    sa = oracle.ingest(tr, w["edges"], 11, w["window_s"])
    sb = oracle.ingest({k: v[perm] for k, v in tr.items()}, w["edges"], 11, w["window_s"])
    for r, s_ in ((ra, sa), (rb, sb), (rc, sa)):
        np.testing.assert_array_equal(r[2].cpu().numpy(), s_["cell_off"])
        np.testing.assert_array_equal(r[0].cpu().numpy(), s_["in_tok"])
        np.testing.assert_array_equal(r[1].cpu().numpy(), s_["out_tok"])
