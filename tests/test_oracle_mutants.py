"""Do the pins notice a mistake in the oracle?  Each case below plants ONE plausible mistake in
a copy of oracle/fltop_oracle.cpp (a wrong source mass, a dropped term, a flipped comparison,
a transposed index ...), builds that copy in a temporary directory, and runs the pin suites
(tests/test_oracle_pins.py, tests/test_oracle_options.py) against it in a child process: the
suites must FAIL.  CPU only; the mistakes never reach the GPU path (which shares no code with
the oracle).

Two mistakes that were tried are left out because they give the same program: `continue`
instead of `break` in the descending walk of frame_survivors (the list is sorted, so nothing
after the first failure passes), and giving a prefix that re-enters through an extension a
new birth record (such an extension's token is the prefix's last token, so the prefix's own
repeat route runs in the same frame and restores the record)."""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "fltop_oracle.cpp")
PIN_SUITES = ["tests/test_oracle_pins.py", "tests/test_oracle_options.py"]

MUTANTS = [
    # ---- expansion (blank / repeat / extend) ----------------------------------------------
    ("repeat-extension takes the whole mass",
     "e.pnb = log_add(e.pnb, m.pb + x + lm.term(last, s));",
     "e.pnb = log_add(e.pnb, p_tot + x + lm.term(last, s));"),
    ("repeat-extension drops the LM term",
     "e.pnb = log_add(e.pnb, m.pb + x + lm.term(last, s));",
     "e.pnb = log_add(e.pnb, m.pb + x);"),
    ("extension drops the LM term",
     "e.pnb = log_add(e.pnb, p_tot + x + lm.term(last, s));",
     "e.pnb = log_add(e.pnb, p_tot + x);"),
    ("repeat-stay takes the whole mass",
     "d.pnb = log_add(d.pnb, m.pnb + x);",
     "d.pnb = log_add(d.pnb, p_tot + x);"),
    ("blank takes the blank mass only",
     "d.pb = log_add(d.pb, p_tot + x);",
     "d.pb = log_add(d.pb, m.pb + x);"),
    ("merge keeps the larger mass instead of adding",
     "return hi + std::log1p(std::exp(lo - hi));",
     "return hi;"),
    # ---- LM term ----------------------------------------------------------------------------
    ("first token reads the token's own row",
     "int32_t row = last < 0 ? 0 : last;",
     "int32_t row = last < 0 ? cur : last;"),
    ("transposed LM index",
     "return alpha * (double)table[(int64_t)row * V + cur] + beta;",
     "return alpha * (double)table[(int64_t)cur * V + row] + beta;"),
    ("insertion bonus dropped",
     "return alpha * (double)table[(int64_t)row * V + cur] + beta;",
     "return alpha * (double)table[(int64_t)row * V + cur];"),
    # ---- frame-level pruning ---------------------------------------------------------------
    ("strict threshold comparison",
     "if (!(row[v] >= thr)) break;",
     "if (!(row[v] > thr)) break;"),
    ("threshold mixes the domains",
     "volatile float thr = m + ln_r;",
     "volatile float thr = m * 1.0f + ln_r * 0.5f;"),
    ("top-N ties by descending token",
     "if (row[a] != row[b]) return row[a] > row[b];\n        return a < b;",
     "if (row[a] != row[b]) return row[a] > row[b];\n        return a > b;"),
    ("top-N keeps the worst",
     "if (row[a] != row[b]) return row[a] > row[b];",
     "if (row[a] != row[b]) return row[a] < row[b];"),
    ("top-N off by one",
     "const int32_t n = (top_n <= 0 || top_n > V) ? V : top_n;",
     "const int32_t n = (top_n <= 0 || top_n > V) ? V : top_n + 1;"),
    # ---- SelectTopK -------------------------------------------------------------------------
    ("beam cut off by one",
     "order.resize(beam);",
     "order.resize(beam + 1);"),
    ("dead entries kept",
     "if (tot == NEG_INF) continue; /* dead: every route into it was pruned */",
     ""),
    ("worst first",
     "if (x.total != y.total) return x.total > y.total;",
     "if (x.total != y.total) return x.total < y.total;"),
    ("ties by larger hash",
     "return x.hash < y.hash;",
     "return x.hash > y.hash;"),
    ("window floor above the best",
     "const double floor_score = order[0].total - beam_threshold;",
     "const double floor_score = order[0].total + beam_threshold;"),
    ("window measured from the worst",
     "const double floor_score = order[0].total - beam_threshold;",
     "const double floor_score = order.back().total - beam_threshold;"),
    ("window twice as wide",
     "const double floor_score = order[0].total - beam_threshold;",
     "const double floor_score = order[0].total - 2.0 * beam_threshold;"),
    ("candidate on the window floor dropped",
     "while (inside < order.size() && order[inside].total >= floor_score) ++inside;",
     "while (inside < order.size() && order[inside].total > floor_score) ++inside;"),
    # ---- hash, final result, statistics ----------------------------------------------------
    ("hash mixing shift",
     "z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;",
     "z = (z ^ (z >> 29)) * 0x94D049BB133111EBULL;"),
    ("hash seed",
     "uint64_t h = GOLDEN;\n    for (size_t i = 0; i < p.size(); ++i)",
     "uint64_t h = 0;\n    for (size_t i = 0; i < p.size(); ++i)"),
    ("birth frame off by one",
     "fresh.born.push_back(t);",
     "fresh.born.push_back(t + 1);"),
    ("hypotheses per step counted before the cut",
     "if (spec.frame_beam) spec.frame_beam[t] = (int32_t)cur.size();",
     "if (spec.frame_beam) spec.frame_beam[t] = (int32_t)next.size();"),
    ("token rank counts the tokens behind",
     "if (v != tokens[i] && before(v, tokens[i])) ++ahead;",
     "if (v != tokens[i] && !before(v, tokens[i])) ++ahead;"),
    # ---- the separately written textbook search ---------------------------------------------
    ("textbook: repeat-extension takes the whole mass",
     "const double from = (v == tail) ? src.blank_mass : whole;",
     "const double from = whole;"),
]


def _build_and_run(job):
    idx, (label, old, new), workdir, original = job
    assert original.count(old) == 1, f"mutant '{label}': its anchor text must occur exactly once"
    src = os.path.join(workdir, f"mutant{idx}.cpp")
    lib = os.path.join(workdir, f"libmutant{idx}.so")
    with open(src, "w") as fh:
        fh.write(original.replace(old, new))
    subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                    "-I", os.path.join(ROOT, "oracle"), src, "-o", lib], check=True)
    env = dict(os.environ, FLTOP_ORACLE_LIB=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", *PIN_SUITES, "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True,
                         text=True)
    return label, run.returncode, run.stdout[-400:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    if "FLTOP_ORACLE_LIB" in os.environ:
        pytest.skip("already running against a substituted oracle")
    with open(SRC) as fh:
        original = fh.read()
    shutil.copy(os.path.join(ROOT, "oracle", "fltop_oracle.h"), tmp_path)
    jobs = [(i, m, str(tmp_path), original) for i, m in enumerate(MUTANTS)]
    workers = max(1, min(8, (os.cpu_count() or 2)))
    with concurrent.futures.ThreadPoolExecutor(workers) as pool:
        results = list(pool.map(_build_and_run, jobs))
    survivors = [label for label, rc, _ in results if rc == 0]
    broken = [(label, rc, tail) for label, rc, tail in results if rc not in (0, 1)]
    assert not broken, f"pin suites did not run properly: {broken}"
    assert not survivors, f"mistakes no pin notices: {survivors}"
