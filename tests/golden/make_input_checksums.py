"""Writes tests/golden/input_checksums.txt: order-sensitive 64-bit checksums of every array the seeded generators
produce for the five benchmark workloads (stand-ins for the paper's 1-hour, 1-day and 1-week traces, Section III).
Calls only the generators; run from the repository root:  python tests/golden/make_input_checksums.py"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from workloads import SPECS, checksum, make  # noqa: E402


def lines_of(i):
    w = make(SPECS[i])
    out = []
    for group in ("trace", "profile", "configs", "slos"):
        for k, v in w[group].items():
            out.append(f"{i} {group}.{k} {checksum(v):016x}")
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "input_checksums.txt")
    with open(path, "w") as f:
        f.write("# workload  array  checksum (workloads.checksum); written by make_input_checksums.py\n")
        for i in range(len(SPECS)):
            f.write("\n".join(lines_of(i)) + "\n")
    print("wrote", path)
