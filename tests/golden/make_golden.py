"""Writes the stored expected values under tests/golden/.  Calls only the seeded
input generators and the CPU oracle (never the GPU path).

    python tests/golden/make_golden.py

cfg0_oracle.txt   one line per (scenario, candidate) pair of configuration 0, scenarios 0, 10, 20:
                  "k c makespan flag bubble_0 .. bubble_{S-1}", as simulated by the
                  oracle.  It guards the oracle and the generator against drift;
                  the oracle itself is pinned by tests/test_oracle_pins.py.
workload_sha256.txt  SHA-256 of the generated inputs of the five configurations.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import oracle  # noqa: E402
from paper_2504_19232_amd import workloads  # noqa: E402


def main():
    wl = workloads.config(0)
    r = oracle.eval_workload(wl, threads=1)
    with open(os.path.join(HERE, "cfg0_oracle.txt"), "w") as f:
        f.write(f"# oracle outputs for workloads.config(0), inputs sha256 {wl.sha256()}\n")
        for k in (0, 10, 20):
            for c in range(wl.n_cand):
                b = " ".join(str(int(r["bubble"][s, k, c])) for s in range(wl.S))
                f.write(f"{k} {c} {int(r['makespan'][k, c])} {int(r['flag'][k, c])} {b}\n")
    with open(os.path.join(HERE, "workload_sha256.txt"), "w") as f:
        for i in range(5):
            wl = workloads.config(i)
            f.write(f"{i} {wl.name} {wl.sha256()}\n")


if __name__ == "__main__":
    main()
