"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, sizes its workspaces sanely and rejects bad profile tables before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dyn():
    import paper_2408_00741_amd as d
    return d


def _declared():
    text = open(os.path.join(ROOT, "include", "dyn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dyn_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(dyn):
    names = _declared()
    assert {"dyn_profile_load", "dyn_eval_space", "dyn_select_config", "dyn_trace_ingest", "dyn_profile_free",
            "dyn_cell_stats", "dyn_workspace_status", "dyn_last_error", "dyn_eval_space_workspace",
            "dyn_trace_ingest_workspace", "dyn_eval_select", "dyn_timing_enable", "dyn_timing_read",
            "dyn_timing_reset", "dyn_eval_select_ticks", "dyn_eval_ticks_workspace", "dyn_eval_select_mixed",
            "dyn_mixed_workspace", "dyn_select_path", "dyn_select_path_workspace", "dyn_account", "dyn_account_workspace",
            "dyn_hierarchy", "dyn_hierarchy_workspace"} <= set(names)
    lib = C.CDLL(dyn.lib_path())
    for n in names:
        assert hasattr(lib, n), n
    for n in names:                      # and the Python binding carries the same names
        assert hasattr(dyn, n), n


def test_workspace_sizes(dyn):
    a = dyn.dyn_eval_space_workspace(1440, 25, 576)
    assert a % 256 == 0 and a >= 36000 * 28
    assert dyn.dyn_eval_space_workspace(2016, 100, 2048) > a
    assert dyn.dyn_eval_space_workspace(0, 25, 576) == 0
    b = dyn.dyn_trace_ingest_workspace(10_000_000, 1440, 25)
    assert b % 256 == 0 and b >= 4 * 4 * 10_000_000
    assert dyn.dyn_trace_ingest_workspace(0, 1, 1) > 0
    c = dyn.dyn_eval_ticks_workspace(10_000_000, 1440, 12, 25, 576)
    assert c % 256 == 0 and c >= 4 * 10_000_000 + 36000 * 12 * 53
    assert dyn.dyn_eval_ticks_workspace(10_000_000, 1440, 65, 25, 576) == 0      # beyond DYN_TICK_LIMIT
    assert dyn.dyn_eval_ticks_workspace(10_000_000, 1440, 0, 25, 576) == 0
    h = dyn.dyn_hierarchy_workspace(1440, 12, 25, 48)
    assert h % 256 == 0 and h >= 36000 * 13 * 53            # both aggregations: 53 bytes per window and per tick cell
    assert dyn.dyn_hierarchy_workspace(1440, 12, 25, 0) == 0 and dyn.dyn_hierarchy_workspace(1440, 0, 25, 48) == 0


def _prof():
    rng = np.random.default_rng(0)
    shape = (2, 2, 3, 4)
    return {"tp": np.asarray([2, 4], np.int32), "f_mhz": np.asarray([800.0, 1200.0, 1980.0]),
            "rho": np.asarray([0.0, 0.3, 0.6, 0.95]), "prefill_ms_per_tok": rng.uniform(0.1, 0.2, shape),
            "tbt_ms": rng.uniform(10, 20, shape), "power_w": rng.uniform(100, 200, shape),
            "max_load_tps": rng.uniform(100, 200, shape[:3])}


@pytest.mark.parametrize("mutate,status", [
    (lambda p: p.update(rho=np.asarray([0.1, 0.3, 0.6, 0.95])), -3),                 # rho[0] != 0
    (lambda p: p.update(rho=np.asarray([0.0, 0.6, 0.6, 0.95])), -5),                 # not increasing
    (lambda p: p.update(f_mhz=np.asarray([800.0, 700.0, 1980.0])), -5),
    (lambda p: p.update(tp=np.asarray([4, 2], np.int32)), -5),
    (lambda p: p["tbt_ms"].__setitem__((0, 0, 0, 0), np.nan), -4),
    (lambda p: p["power_w"].__setitem__((1, 1, 2, 3), -1.0), -4),
    (lambda p: p["prefill_ms_per_tok"].__setitem__((1, 0, 0, 0), np.inf), -4),
    (lambda p: p["max_load_tps"].__setitem__((0, 0, 0), 0.0), -4),
])
def test_profile_load_rejects_bad_tables_on_the_host(dyn, mutate, status):
    p = _prof()
    mutate(p)
    with pytest.raises(dyn.DynError) as e:
        dyn.dyn_profile_load(p, stream=_NullStream())
    assert e.value.status == status and dyn.dyn_last_error()


class _NullStream:
    cuda_stream = 0


def test_binding_refuses_host_tensors(dyn):
    import torch
    with pytest.raises(ValueError):
        dyn.binding._dp(torch.zeros(4, dtype=torch.int32), torch.int32, "x")
