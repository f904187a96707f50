"""Writes the stored expected values under tests/golden/.

Calls only the seeded input generator and the CPU oracle (never the HIP
library).  The paper prints no numeric value of g, L, a predicted time or a
chosen strategy, so nothing here is the paper's; these files freeze the
oracle's own output on config 1 (the 100 Mbit/s-like table: L = 55 us,
11.5 MB/s, P = 2..50, m up to 1 MiB, the scale of the paper's Section 2
cluster) so that a later change to the oracle or to the generator shows up
as a diff that has to be justified.

    python tests/golden/make_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from oracle import plogp_cutover  # noqa: E402
from plogp_workloads import make_workload  # noqa: E402


def main():
    wl = make_workload(1)
    out, _ = oracle.tune_workload(wl)
    with open(os.path.join(HERE, "cfg1_table.txt"), "w") as f:
        f.write("# config 1 pLogP table: size_bytes gap_us(hex float); L = %s\n" % float(wl.L[0]).hex())
        for x, y in zip(wl.sizes[0], wl.gaps[0]):
            f.write("%d %s\n" % (int(x), float(y).hex()))
    with open(os.path.join(HERE, "cfg1_decisions.txt"), "w") as f:
        f.write("# config 1 Broadcast decision table from the CPU oracle:\n")
        f.write("# m_index m_bytes P strategy s time_us(hex float)\n")
        for mi in range(0, len(wl.m), 3):
            for pi in (0, 1, 2, 6, 14, 30, 48):
                c = out[0, 0, mi, pi]
                f.write("%d %d %d %d %d %s\n" % (mi, int(wl.m[mi]), int(wl.P[pi]), int(c["strategy"]),
                                                 int(c["s"]), float(c["time"]).hex()))
    off, runs = plogp_cutover.cutovers(out, wl.m, 0)
    with open(os.path.join(HERE, "cfg1_cutovers.txt"), "w") as f:
        f.write("# config 1, Broadcast plane: the runs of equal strategy along m for some P\n")
        f.write("# P m_from strategy s   (s of the first cell of the run)\n")
        for pi in (0, 1, 2, 6, 14, 30, 48):
            for k in range(int(off[pi]), int(off[pi + 1])):      # plane 0, table 0: row index = pi
                f.write("%d %d %d %d\n" % (int(wl.P[pi]), int(runs["m_from"][k]), int(runs["strategy"][k]),
                                          int(runs["s"][k])))


if __name__ == "__main__":
    main()
