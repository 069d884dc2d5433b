"""The allocation-free variant of dyn_eval_select (fixed workspace inside the library) against dyn_eval_select
itself, through the C ABI, on two calls in a row, the second with a smaller input."""
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


def _case(dyn, spec):
    w = make(spec)
    tr = w["trace"]
    ins, outs, off, _ = dyn.dyn_trace_ingest(_dev(tr["t_s"]), _dev(tr["in_tok"]), _dev(tr["out_tok"]), _dev(tr["model"]),
                                             w["edges"], w["n_window"], w["window_s"])
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    return w, ins, outs, off, prof, plan


def _blank_like(d):
    return {k: torch.full_like(v, 255 if v.dtype == torch.uint8 else -3) for k, v in d.items()}


def test_static_workspace_matches_the_caller_workspace_entry_point(dyn):
    # first call: 60 windows x 25 classes x 576 configurations with an off-size tail; second call: a smaller
    # trace with other classes, configurations and window length, on the same fixed array
    cases = [_case(dyn, SPECS[2].scaled(500_000, 61)), _case(dyn, SPECS[1].scaled(30_000, 5))]
    refs = []
    for w, ins, outs, off, prof, plan in cases:
        space, sel, ws = dyn.dyn_eval_select(prof, ins, outs, off, w["n_window"], w["window_s"], plan)
        assert dyn.dyn_workspace_status(ws) == 0
        refs.append((space, sel))
    torch.cuda.synchronize()
    status = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    for rep in range(2):                                   # the pair of calls twice: large, small, large, small
        for (w, ins, outs, off, prof, plan), (space, sel) in zip(cases, refs):
            out2, sel2 = _blank_like(space), _blank_like(sel)
            free0 = torch.cuda.mem_get_info()[0]
            dyn.dyn_eval_select_static(prof, ins, outs, off, w["n_window"], w["window_s"], plan, out2, sel2, status=status)
            torch.cuda.synchronize()
            if rep:                                        # (the first launches load the library's code objects)
                assert torch.cuda.mem_get_info()[0] == free0    # nothing was allocated on the device
            assert int(status.item()) == 0
            for k in space:
                assert torch.equal(out2[k], space[k]), (rep, k)
            for k in sel:
                assert torch.equal(sel2[k], sel[k]), (rep, k)
    # a negative token count shows up in the status word of the call that saw it, and not in the next one
    w, ins, outs, off, prof, plan = cases[1]
    bad = ins.clone(); bad[7] = -5
    out2, sel2 = _blank_like(refs[1][0]), _blank_like(refs[1][1])
    dyn.dyn_eval_select_static(prof, bad, outs, off, w["n_window"], w["window_s"], plan, out2, sel2, status=status)
    assert int(status.item()) & dyn.DYN_WS_BAD_REQUEST
    dyn.dyn_eval_select_static(prof, ins, outs, off, w["n_window"], w["window_s"], plan, out2, sel2, status=status)
    assert int(status.item()) == 0
    for k in refs[1][0]:
        assert torch.equal(out2[k], refs[1][0][k]), k
    for c in cases:
        c[4].free()


def test_static_workspace_refuses_what_does_not_fit(dyn):
    w = make(SPECS[3].scaled(1000, 2016), with_trace=False)          # 50400 cells x 1152 configurations: 33 MB
    prof = dyn.dyn_profile_load(w["profile"])
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])
    G, K, NW = w["n_class"], plan.K, 2016
    assert dyn.dyn_eval_space_workspace(NW, G, K) > dyn.DYN_STATIC_WORKSPACE_BYTES
    off = torch.zeros(NW * G + 1, dtype=torch.int64, device="cuda")
    x = torch.zeros(0, dtype=torch.int32, device="cuda")
    # the size check comes before anything touches the outputs
    with pytest.raises(dyn.DynError) as e:
        import ctypes as C
        from paper_2408_00741_amd import binding as b
        tv = b._TraceView(0, NW, 300.0, None, None, off.data_ptr())
        sp = b._Space(1, 1, 1, 1)          # never dereferenced: the call fails on the size
        se = b._Selection(1, 1, 1, 1, 1)
        b._check(b._lib.dyn_eval_select_static(prof.handle, C.byref(tv), plan.cfg, K, C.byref(plan.obj), C.byref(sp),
                                               C.byref(se), None, None), "dyn_eval_select_static")
    assert e.value.status == -6 and "fixed" in str(e.value)
    prof.free()
