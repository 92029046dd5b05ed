"""Writes tests/golden/plan_sizes.txt from the oracle planner alone (never from the HIP
library).  The paper prints no worked numeric example of Algorithm 1, so these values are
regression pins of the oracle; its independent pins are the brute-force and closed-form
tests in tests/test_oracle_plan.py.

    python tests/golden/make_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import plan as P          # noqa: E402
from workloads import WORKLOADS       # noqa: E402


def main():
    lines = ["# config world n_tensors E S total num_scales first_offsets(<=6) "
             "| oracle planner, Algorithm 1 (Section 5), default order"]
    for idx, wl in WORKLOADS.items():
        specs = [P.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
        pl = P.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)
        offs = ",".join(str(o) for o in pl.offsets[:6])
        lines.append(f"{idx} {wl.world} {len(specs)} {pl.payload} {pl.S} {pl.total} "
                     f"{pl.scale_bases()[-1]} {offs}")
    with open(os.path.join(HERE, "plan_sizes.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
