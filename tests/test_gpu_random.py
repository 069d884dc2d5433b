"""Randomly drawn small workloads through the C ABI against the CPU oracle: shapes, token ranges and percentiles that the
named cases do not spell out one by one (every draw is seeded; a failure prints the draw)."""
import numpy as np
import pytest

import oracle
from tests.test_gpu_parity import assert_parity, gpu_eval, gpu_ingest, ora_eval
from tests.test_gpu_ticks import _random_case, assert_same, gpu_ticks, ora_ticks

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

PCTS = [(99, 100), (1, 2), (9, 10), (1, 1), (1, 100), (999, 1000), (95, 100)]
IN_HI = [3, 50, 600, 8000, 65535, 65536, 65537, 70000, 200000]
PER_BLOCK = 25


@pytest.fixture(scope="module")
def dyn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2408_00741_amd as d
    return d


def _reshape_lengths(w, rng, in_hi):
    """Input lengths: as drawn (uniform), from five values, from a range of 40, or from the six below `in_hi`."""
    n = w["trace"]["in_tok"].size
    dist = str(rng.choice(["uniform", "few", "narrow", "top"]))
    if dist == "few":
        w["trace"]["in_tok"] = rng.choice(rng.integers(0, in_hi, 5), n).astype(np.int32)
    elif dist == "narrow":
        base = int(rng.integers(0, max(1, in_hi - 40)))
        w["trace"]["in_tok"] = rng.integers(base, base + 40, n).astype(np.int32)
    elif dist == "top":
        w["trace"]["in_tok"] = rng.integers(max(0, in_hi - 6), in_hi, n).astype(np.int32)
    return dist


@pytest.mark.parametrize("block", range(6))
def test_random_draws_window_level(dyn, block):
    """1 .. 8 windows of 20 .. 120 000 requests in two classes (cells from empty to tens of thousands of requests: every
    route of the aggregation), token counts up to 2^16 and beyond, traces in and out of window order."""
    for seed in range(block * PER_BLOCK, (block + 1) * PER_BLOCK):
        rng = np.random.default_rng(19000 + seed)
        NW = int(rng.integers(1, 9))
        n_req = int(np.exp(rng.uniform(np.log(20), np.log(120000))))
        in_hi = int(rng.choice(IN_HI + [2_000_000]))
        crowd = int(rng.integers(0, NW)) if rng.random() < 0.3 else None
        w = _random_case(seed, n_req, NW, 1, 60.0, in_hi=in_hi, crowd=crowd)
        dist = _reshape_lengths(w, rng, in_hi)
        r = rng.random()
        if r < 0.25:
            w["trace"]["out_tok"][rng.integers(0, n_req, 3)] = 70_000 if r < 0.15 else 1_500_000
        if rng.random() < 0.2:
            w["trace"]["t_s"] = np.sort(w["trace"]["t_s"])          # already in window order
        w["pct"] = PCTS[int(rng.integers(0, len(PCTS)))]
        bud = np.asarray([0, 12], np.int32) if rng.random() < 0.3 else None
        tag = f"seed {seed}: NW {NW} n {n_req} in_hi {in_hi} crowd {crowd} lengths {dist} pct {w['pct']} budget {bud is not None}"
        st = oracle.ingest(w["trace"], w["edges"], w["n_window"], w["window_s"])
        ins, outs, off, iws = gpu_ingest(dyn, w)
        assert dyn.dyn_workspace_status(iws) == 0, tag
        for k, v in (("in_tok", ins), ("out_tok", outs), ("cell_off", off)):
            np.testing.assert_array_equal(v.cpu().numpy(), st[k], err_msg=f"{tag}: {k}")
        g = gpu_eval(dyn, w, ins, outs, off, bud)
        assert g["status"] == 0, tag
        rep = assert_parity(w, g, ora_eval(w, st, bud))
        assert rep["bit_exact"] and rep["sel_mismatch"] == 0, (tag, rep)


@pytest.mark.parametrize("block", range(8))
def test_random_draws_tick_level(dyn, block):
    """1 .. 6 windows of 1 .. 64 ticks, 50 .. 40 000 requests; prefill tables random, flat, flat up to the 3rd .. 8th digit,
    or with a zero; half of the trace in one tick in a third of the draws (some cells then lie deeper than the per-tick
    lists reach, j > 8192, and are searched over their requests)."""
    for seed in range(block * PER_BLOCK, (block + 1) * PER_BLOCK):
        rng = np.random.default_rng(9000 + seed)
        NW = int(rng.integers(1, 7))
        T = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 31, 60, 64]))
        n_req = int(np.exp(rng.uniform(np.log(50), np.log(40000))))
        in_hi = int(rng.choice(IN_HI))
        crowd = int(rng.integers(0, NW * T)) if rng.random() < 0.3 else None
        w = _random_case(seed, n_req, NW, T, 5.0, in_hi=in_hi, crowd=crowd)
        pf = w["profile"]["prefill_ms_per_tok"]
        mode = str(rng.choice(["random", "flat", "nearflat", "zero"], p=[0.35, 0.4, 0.2, 0.05]))
        if mode == "flat":
            pf[...] = rng.uniform(0.05, 0.3, pf.shape[:3] + (1,))
        elif mode == "nearflat":
            pf[...] = rng.uniform(0.05, 0.3, pf.shape[:3] + (1,)) * (1 + rng.uniform(0, 10.0 ** -rng.integers(3, 9), pf.shape))
        elif mode == "zero":
            pf[..., 0] = 0.0
        dist = _reshape_lengths(w, rng, in_hi)
        if rng.random() < 0.15:
            w["trace"]["out_tok"][rng.integers(0, n_req, 3)] = 70_000
        pct = PCTS[int(rng.integers(0, len(PCTS)))]
        bud = np.asarray([0, 12], np.int32) if rng.random() < 0.3 else None
        tag = (f"seed {seed}: NW {NW} T {T} n {n_req} in_hi {in_hi} crowd {crowd} prefill {mode} lengths {dist} pct {pct} "
               f"budget {bud is not None}")
        g, fine = gpu_ticks(dyn, w, T, bud, pct=pct)
        o = ora_ticks(w, fine, T, bud, pct=pct)
        assert g["status"] == 0, tag
        try:
            assert_same(w, g, o)
        except AssertionError as e:
            raise AssertionError(f"{tag}\n{e}") from None


@pytest.mark.parametrize("block", range(6))
def test_random_draws_with_many_ties(dyn, block):
    """Tick-level draws with flat (or nearly flat) prefill tables and input lengths from a handful of values: every
    percentile falls among many equal lengths, whose rank the evaluation finds from the ticks' counts of them, with its
    list of four ticks from either end or by ranking all ticks."""
    for seed in range(block * PER_BLOCK, (block + 1) * PER_BLOCK):
        rng = np.random.default_rng(29000 + seed)
        NW = int(rng.integers(1, 7))
        T = int(rng.choice([2, 3, 5, 7, 8, 12, 16, 31, 64]))
        n_req = int(np.exp(rng.uniform(np.log(200), np.log(40000))))
        in_hi = int(rng.choice([3, 7, 20, 50, 600, 8000]))
        crowd = int(rng.integers(0, NW * T)) if rng.random() < 0.3 else None
        w = _random_case(seed, n_req, NW, T, 5.0, in_hi=in_hi, crowd=crowd)
        pf = w["profile"]["prefill_ms_per_tok"]
        pf[...] = rng.uniform(0.05, 0.3, pf.shape[:3] + (1,))
        if rng.random() < 0.2:
            pf *= 1 + rng.uniform(0, 10.0 ** -rng.integers(3, 9), pf.shape)
        n = w["trace"]["in_tok"].size
        kind = str(rng.choice(["few", "narrow", "top"]))
        if kind == "few":
            w["trace"]["in_tok"] = rng.choice(rng.integers(0, in_hi, 5), n).astype(np.int32)
        elif kind == "narrow":
            base = int(rng.integers(0, max(1, in_hi - 40)))
            w["trace"]["in_tok"] = rng.integers(base, base + 40, n).astype(np.int32)
        else:
            w["trace"]["in_tok"] = rng.integers(max(0, in_hi - 6), in_hi, n).astype(np.int32)
        pct = PCTS[int(rng.integers(0, len(PCTS)))]
        tag = f"seed {seed}: NW {NW} T {T} n {n_req} in_hi {in_hi} crowd {crowd} lengths {kind} pct {pct}"
        g, fine = gpu_ticks(dyn, w, T, pct=pct)
        o = ora_ticks(w, fine, T, pct=pct)
        assert g["status"] == 0, tag
        try:
            assert_same(w, g, o)
        except AssertionError as e:
            raise AssertionError(f"{tag}\n{e}") from None
