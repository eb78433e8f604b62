#!/usr/bin/env python3
"""Writes the CPU oracle's result on a whole named workload to a text file under tests/golden/.

Only for workloads the oracle cannot redo inside a test run (the unpruned sub-word workload:
65 536 candidates per frame, some 3.4e9 candidate updates).  Imports the oracle and the seeded
input generators, nothing else of the repository: no value in the file comes from the HIP path.

    python tests/golden/make_workload_golden.py cfg4_subword1024 0.0 [threads]

File format (text): '#' comment lines; one line `stats <key>=<int> ...` with the oracle's integer
statistics over the batch; then one line per utterance:
    <utterance> <score as C99 hex float (exact fp64)> <number of tokens> <token ids ...>
"""
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2510_09085_amd import synth  # noqa: E402

STAT_KEYS = ("frames", "sum_survivors", "sum_candidates", "peak_candidates", "sum_beam")


def golden_path(workload: str, r: float) -> str:
    return os.path.join(ROOT, "tests", "golden", f"{workload}_r{r:g}_oracle.txt")


def main():
    name, r = sys.argv[1], float(sys.argv[2])
    threads = int(sys.argv[3]) if len(sys.argv) > 3 else max(1, (os.cpu_count() or 2) - 1)
    w = synth.WORKLOADS[name]
    lp, ln = synth.make_emissions(w)
    lm = synth.make_bigram_lm(w.V) if w.use_lm else None
    t0 = time.time()
    toks, scores, st = oracle.decode(lp, ln, w.beam, r, lm_table=lm, lm_weight=w.lm_weight,
                                     insertion_bonus=w.insertion_bonus, n_threads=threads)
    dt = time.time() - t0
    assert st["hash_collisions"] == 0
    with open(golden_path(name, r), "w") as fh:
        fh.write(f"# CPU oracle (oracle/fltop_oracle.cpp, Algorithm 1 with the two-mass CTC collapse) on the\n"
                 f"# whole workload {name}: B={w.B} T={w.T} V={w.V} beam={w.beam} rel_threshold={r:g}\n"
                 f"# seed={w.seed}, inputs from paper_2510_09085_amd/synth.py.  Written by\n"
                 f"#   python tests/golden/make_workload_golden.py {name} {r:g}\n"
                 f"# ({dt:.0f} s on {threads} threads).  Not a value printed in the paper.\n")
        fh.write("stats " + " ".join(f"{k}={int(st[k])}" for k in STAT_KEYS) + "\n")
        for b in range(w.B):
            fh.write(f"{b} {float(scores[b]).hex()} {len(toks[b])} "
                     + " ".join(str(t) for t in toks[b]) + "\n")
    print(f"wrote {golden_path(name, r)} in {dt:.0f} s")


if __name__ == "__main__":
    main()
