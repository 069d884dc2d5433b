"""The seeded generators give the same bytes everywhere: checksums of workloads 0-2 against the recorded ones
(tests/golden/input_checksums.txt, written by tests/golden/make_input_checksums.py; workloads 3-4 take minutes to
generate here and are compared by bench.py --checksums on the machine that runs it)."""
import os

import pytest

from workloads import SPECS, checksum, make

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "input_checksums.txt")


def recorded():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        i, name, value = line.split()
        out[(int(i), name)] = value
    return out


def test_every_workload_is_recorded():
    rec = recorded()
    for i in range(len(SPECS)):
        names = {n for (j, n) in rec if j == i}
        assert {"trace.t_s", "trace.in_tok", "trace.out_tok", "trace.model", "profile.power_w", "configs.n_inst",
                "slos.slo_ttft_ms"} <= names


@pytest.mark.parametrize("i", [0, 1, 2])
def test_generated_arrays_match_the_recorded_checksums(i):
    rec = recorded()
    w = make(SPECS[i])
    n = 0
    for group in ("trace", "profile", "configs", "slos"):
        for k, v in w[group].items():
            assert f"{checksum(v):016x}" == rec[(i, f"{group}.{k}")], (i, group, k)
            n += 1
    assert n == sum(1 for (j, _) in rec if j == i)
