"""Pins for the oracle's optional stages: the static top-N token stage of Alg. 1, the
score window of SelectTopK, and the statistics traces (paper Sec. 4.1 / 4.4).

Each is checked against something other than the oracle: numpy's sort, exhaustive
alignment enumeration, the arg-max path, a hand-worked example
(tests/golden/beam_window_example.txt), closed-form counts.  No GPU needed.
"""
import itertools
import math
import os

import numpy as np
import pytest

from paper_2510_09085_amd import synth
from test_oracle_pins import NEG_INF, collapse, logsumexp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def top_n_survivors_by_sorting(row, r, n):
    """Alg. 1's token stage from numpy's sort: N best (ties: lower id first), then p >= r * p_top."""
    row = np.asarray(row, dtype=np.float32)
    V = len(row)
    order = np.lexsort((np.arange(V), -row.astype(np.float64)))  # last key is the primary one
    if 0 < n < V:
        order = order[:n]
    with np.errstate(divide="ignore"):
        ln_r = np.float32(np.log(np.float64(r)))
    thr = np.float32(row[order[0]] + ln_r)
    return sorted(int(v) for v in order if row[v] >= thr)


def tied_emissions(seed, F, V, levels=6):
    """Rows drawn from a few distinct values, so that equal emissions are common."""
    rng = np.random.default_rng(seed)
    vals = -np.arange(levels, dtype=np.float32) * np.float32(0.75)
    return vals[rng.integers(0, levels, size=(F, V))]


# --------------------------------------------------------------------------- top-N stage
@pytest.mark.parametrize("V", [2, 5, 32, 257])
def test_top_n_survivor_sets_match_a_library_sort(oracle_lib, V):
    F = 60
    rows = np.concatenate([synth.random_emissions(400 + V, 1, F, V, flat=2.0)[0],
                           tied_emissions(V, F, V)])
    for n in (0, 1, 2, 4, V - 1, V, V + 7):
        for r in (0.0, 0.01, 0.5, 1.0):
            counts, toks, fmax = oracle_lib.survivors(rows, r, top_n=n)
            for f in range(rows.shape[0]):
                want = top_n_survivors_by_sorting(rows[f], r, n)
                assert toks[f, :counts[f]].tolist() == want, (V, n, r, f)
                assert fmax[f] == rows[f].max()
                if n > 0:
                    assert counts[f] <= n


def test_top_n_ties_prefer_the_lower_token_id(oracle_lib):
    row = np.log(np.array([[0.25, 0.25, 0.25, 0.15, 0.10]], dtype=np.float64)).astype(np.float32)
    for n, want in ((1, [0]), (2, [0, 1]), (3, [0, 1, 2]), (4, [0, 1, 2, 3])):
        counts, toks, _ = oracle_lib.survivors(row, 0.0, top_n=n)
        assert toks[0, :counts[0]].tolist() == want
    # the threshold still applies inside the N best: 0.15 < 0.9 * 0.25
    counts, toks, _ = oracle_lib.survivors(row, 0.9, top_n=4)
    assert toks[0, :counts[0]].tolist() == [0, 1, 2]


def test_top_n_sets_grow_with_n_and_saturate(oracle_lib):
    rows = synth.random_emissions(9, 1, 200, 32, flat=2.0)[0]
    prev = None
    for n in (1, 2, 3, 4, 8, 16, 32):
        counts, toks, _ = oracle_lib.survivors(rows, 0.001, top_n=n)
        cur = [set(toks[f, :counts[f]].tolist()) for f in range(200)]
        if prev is not None:
            assert all(a <= b for a, b in zip(prev, cur))
        prev = cur
    full = oracle_lib.survivors(rows, 0.001, top_n=0)
    assert [set(full[1][f, :full[0][f]].tolist()) for f in range(200)] == prev


def brute_force_masses_top_n(lp, r, n, lm=None, alpha=0.0, beta=0.0):
    T, V = lp.shape
    keep = [set(top_n_survivors_by_sorting(lp[t], r, n)) for t in range(T)]
    acc = {}
    for path in itertools.product(range(V), repeat=T):
        if any(path[t] not in keep[t] for t in range(T)):
            continue
        acc.setdefault(collapse(path), []).append(sum(float(lp[t, path[t]]) for t in range(T)))
    out = {}
    for label, scores in acc.items():
        tot = logsumexp(scores)
        if lm is not None:
            prev = 0
            for c in label:
                tot += alpha * float(lm[prev, c]) + beta
                prev = c
        if tot != NEG_INF:
            out[label] = tot
    return out


@pytest.mark.parametrize("T,V", [(3, 3), (5, 4), (6, 4)])
@pytest.mark.parametrize("n", [1, 2, 3])
@pytest.mark.parametrize("r", [0.0, 0.2])
@pytest.mark.parametrize("with_lm", [False, True])
def test_top_n_search_equals_alignment_enumeration(oracle_lib, T, V, n, r, with_lm):
    for seed in range(3):
        lp = synth.random_emissions(7000 + 100 * T + 10 * V + seed, 1, T, V, flat=1.5)[0]
        lm = synth.make_bigram_lm(V, seed=15 + seed) if with_lm else None
        alpha, beta = (0.75, 0.5) if with_lm else (0.0, 0.0)
        want = brute_force_masses_top_n(lp, r, n, lm, alpha, beta)
        entries = oracle_lib.decode_beam(lp, 100000, r, top_n=n, lm_table=lm, lm_weight=alpha,
                                         insertion_bonus=beta, max_entries=100000)
        got = {tok: logsumexp([pb, pnb]) for tok, pb, pnb in entries}
        assert set(got) == set(want)
        for label, mass in want.items():
            assert got[label] == pytest.approx(mass, abs=1e-12)


def test_top_one_is_the_argmax_path_for_any_beam(oracle_lib):
    lp = synth.random_emissions(21, 2, 90, 11, flat=3.0)
    ln = np.array([90, 57], dtype=np.int32)
    for beam in (1, 5, 40):
        toks, sc, st = oracle_lib.decode(lp, ln, beam, 0.0, top_n=1)
        for b in range(2):
            rows = lp[b, :ln[b]]
            assert tuple(toks[b]) == collapse(rows.argmax(axis=1))
            assert sc[b] == pytest.approx(float(rows.max(axis=1).astype(np.float64).sum()),
                                          abs=1e-9)
        assert st["sum_survivors"] == int(ln.sum())


def test_top_n_of_the_whole_vocabulary_changes_nothing(oracle_lib):
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(2))
    base = oracle_lib.decode(lp, ln, 16, 0.01)
    for n in (w.V, w.V + 1):
        got = oracle_lib.decode(lp, ln, 16, 0.01, top_n=n)
        assert got[0] == base[0]
        assert np.array_equal(got[1], base[1])
    # and a real N changes the candidate counts in the expected direction
    few = oracle_lib.decode(lp, ln, 16, 0.0, top_n=4)
    allv = oracle_lib.decode(lp, ln, 16, 0.0)
    assert few[2]["sum_survivors"] == 4 * int(ln.sum())
    assert few[2]["sum_candidates"] < allv[2]["sum_candidates"]


# --------------------------------------------------------------------------- score window
def test_hand_worked_score_window_example(oracle_lib):
    probs = np.array([[0.5, 0.3, 0.2], [0.2, 0.5, 0.3]])
    lp = np.log(probs).astype(np.float32)
    expected = {}
    with open(os.path.join(GOLDEN, "beam_window_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            case, base, prefix, mass = line.split()
            toks = () if prefix == "-" else tuple(int(x) for x in prefix.split(","))
            expected.setdefault((case, float(base)), {})[toks] = float(mass)
    assert len(expected) == 3
    for (case, base), table in expected.items():
        entries = oracle_lib.decode_beam(lp, 100, 0.0, beam_threshold=math.log(base) + 1e-6,
                                         max_entries=100)
        got = {tok: logsumexp([pb, pnb]) for tok, pb, pnb in entries}
        assert set(got) == set(table), (case, got)
        for toks, mass in table.items():
            assert math.exp(got[toks]) == pytest.approx(mass, rel=1e-6)


def test_candidate_exactly_on_the_window_floor_is_kept(oracle_lib):
    """tests/golden/beam_window_floor_tie.txt: scores that are exact multiples of fp32(ln 2),
    window = that same number, so two candidates sit on the floor bit for bit."""
    L = float(np.float32(math.log(2.0)))
    assert L == 0.693147182464599609375
    expected = {}
    with open(os.path.join(GOLDEN, "beam_window_floor_tie.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            T, prefix, mass = line.split()
            toks = () if prefix == "-" else tuple(int(x) for x in prefix.split(","))
            expected.setdefault(int(T), {})[toks] = float(mass)
    assert sorted(expected) == [1, 2]
    for T, table in expected.items():
        lp = np.tile(np.array([-L, -2 * L, -2 * L], dtype=np.float32), (T, 1))
        assert float(lp[0, 1]) == -2 * L  # exact in fp32
        entries = oracle_lib.decode_beam(lp, 100, 0.0, beam_threshold=L, max_entries=100)
        got = {tok: logsumexp([pb, pnb]) for tok, pb, pnb in entries}
        assert set(got) == set(table), (T, got)
        for toks, mass in table.items():
            assert math.exp(got[toks]) == pytest.approx(mass, rel=1e-6)
    # the tie is real: at T = 1 the two kept candidates score exactly best - window
    one = oracle_lib.decode_beam(np.array([[-L, -2 * L, -2 * L]], dtype=np.float32), 100, 0.0,
                                 beam_threshold=L, max_entries=100)
    totals = sorted(logsumexp([pb, pnb]) for _, pb, pnb in one)
    assert totals == [-2 * L, -2 * L, -L] and totals[2] - L == totals[0]


def test_huge_window_is_no_window(oracle_lib):
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(3))
    base = oracle_lib.decode(lp, ln, 12, 0.01)
    wide = oracle_lib.decode(lp, ln, 12, 0.01, beam_threshold=1e30)
    assert wide[0] == base[0]
    assert np.array_equal(wide[1], base[1])
    assert wide[2]["sum_beam"] == base[2]["sum_beam"]


def test_vanishing_window_is_a_beam_of_one(oracle_lib):
    lp = synth.random_emissions(33, 3, 70, 8, flat=2.0)
    ln = np.array([70, 70, 35], dtype=np.int32)
    one = oracle_lib.decode(lp, ln, 1, 0.0)
    narrow = oracle_lib.decode(lp, ln, 50, 0.0, beam_threshold=1e-9, traces=True)
    assert narrow[0] == one[0]
    np.testing.assert_allclose(narrow[1], one[1], rtol=0, atol=1e-12)
    fb = narrow[2]["frame_beam"]
    for b in range(3):
        assert np.all(fb[b, :ln[b]] == 1)


@pytest.mark.parametrize("window", [0.5, 3.0, 8.0])
def test_final_beam_lies_inside_the_window(oracle_lib, window):
    lp = synth.random_emissions(44, 1, 60, 6, flat=1.5)[0]
    entries = oracle_lib.decode_beam(lp, 64, 0.0, beam_threshold=window, max_entries=64)
    totals = [logsumexp([pb, pnb]) for _, pb, pnb in entries]
    assert totals == sorted(totals, reverse=True)
    assert all(t >= totals[0] - window for t in totals)
    # a wider window can only keep more of the same frame's candidates; on the final beam of
    # the no-window search the window predicate marks exactly a leading run
    free = oracle_lib.decode_beam(lp, 64, 0.0, max_entries=64)
    assert len(entries) <= len(free)


def test_window_shrinks_the_live_beam(oracle_lib):
    """The paper's Sec. 4.4 measures hypotheses per time step; the window is what lets that
    number fall below beam_size."""
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(2))
    free = oracle_lib.decode(lp, ln, 32, 0.0, traces=True)[2]
    cut = oracle_lib.decode(lp, ln, 32, 0.0, beam_threshold=6.0, traces=True)[2]
    assert cut["sum_beam"] < free["sum_beam"]
    assert cut["frame_beam"].max() <= 32 and cut["frame_beam"][:, :ln[0]].min() >= 1
    assert int(cut["frame_beam"][cut["frame_beam"] >= 0].sum()) == cut["sum_beam"]
    assert int(free["frame_beam"][free["frame_beam"] >= 0].sum()) == free["sum_beam"]


# --------------------------------------------------------------------------- traces
def run_starts(path):
    """Frames at which the collapsed output of an alignment gains a token."""
    out = []
    prev = None
    for t, s in enumerate(path):
        if s != prev and s != 0:
            out.append(t)
        prev = s
    return out


def test_token_frames_on_deterministic_paths(oracle_lib):
    rng = np.random.default_rng(8)
    T, V = 60, 6
    path = rng.integers(0, V, size=T)
    lp = np.full((1, T, V), -np.inf, dtype=np.float32)
    lp[0, np.arange(T), path] = 0.0
    for beam in (1, 6):
        toks, _, st = oracle_lib.decode(lp, np.array([T], np.int32), beam, 0.0, traces=True)
        assert tuple(toks[0]) == collapse(path)
        assert st["token_frames"][0] == run_starts(path)
    # arbitrary emissions, beam 1, r = 1: the single hypothesis follows the arg-max path
    lp = synth.random_emissions(12, 2, 80, 9, flat=3.0)
    ln = np.array([80, 33], dtype=np.int32)
    toks, _, st = oracle_lib.decode(lp, ln, 1, 1.0, traces=True)
    for b in range(2):
        assert st["token_frames"][b] == run_starts(lp[b, :ln[b]].argmax(axis=1))


def test_token_frames_are_increasing_and_point_at_survivors(oracle_lib):
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(3))
    toks, _, st = oracle_lib.decode(lp, ln, 16, 0.01, top_n=4, traces=True)
    for b in range(3):
        fr = st["token_frames"][b]
        assert len(fr) == len(toks[b])
        assert all(x < y for x, y in zip(fr, fr[1:]))
        for tok, f in zip(toks[b], fr):
            assert 0 <= f < ln[b]
            assert tok in top_n_survivors_by_sorting(lp[b, f], 0.01, 4)


def test_live_beam_count_for_a_two_symbol_alphabet(oracle_lib):
    """V = 2, nothing pruned, beam large: after t+1 frames the reachable prefixes are a^k with
    k <= ceil((t+1)/2) (a repeated token needs a blank in between)."""
    T = 15
    lp = synth.random_emissions(2, 1, T, 2, flat=1.0)
    st = oracle_lib.decode(lp, np.array([T], np.int32), 1000, 0.0, traces=True)[2]
    want = [math.ceil((t + 1) / 2) + 1 for t in range(T)]
    assert st["frame_beam"][0].tolist() == want


def test_token_ranks_match_a_library_sort(oracle_lib):
    T, V = 40, 13
    lp = np.concatenate([synth.random_emissions(5, 1, T // 2, V, flat=2.0)[0],
                         tied_emissions(6, T // 2, V)])
    rng = np.random.default_rng(1)
    frames = rng.integers(0, T, size=200)
    tokens = rng.integers(0, V, size=200)
    got = oracle_lib.token_ranks(lp, tokens, frames)
    for i in range(200):
        row = lp[frames[i]]
        order = np.lexsort((np.arange(V), -row.astype(np.float64)))
        assert got[i] == int(np.nonzero(order == tokens[i])[0][0])


def test_option_argument_errors(oracle_lib):
    lp = synth.random_emissions(1, 1, 4, 3)
    ln = np.array([4], np.int32)
    with pytest.raises(ValueError):
        oracle_lib.decode(lp, ln, 4, 0.1, top_n=-1)
    with pytest.raises(ValueError):
        oracle_lib.decode(lp, ln, 4, 0.1, beam_threshold=float("nan"))
    with pytest.raises(ValueError):
        oracle_lib.decode(lp, ln, 4, 0.0, top_n=2, variant=oracle_lib.TEXTBOOK)
    with pytest.raises(ValueError):
        oracle_lib.decode(lp, ln, 4, 0.0, beam_threshold=1.0, variant=oracle_lib.TEXTBOOK)
    with pytest.raises(ValueError):
        oracle_lib.survivors(lp, 0.1, top_n=-2)


def test_token_frames_keep_the_first_entry_while_the_prefix_stays_in_the_beam(oracle_lib):
    """V = 2, nothing pruned, beam large: a^j can first exist after the frames a,-,a,...,a
    (2j-1 of them), enters the beam then and never leaves it, although its parent keeps
    extending into it at every later frame."""
    T = 9
    probs = np.empty((1, T, 2))
    probs[0, 0::2] = [0.2, 0.8]  # even frames favour 'a'
    probs[0, 1::2] = [0.7, 0.3]  # odd frames favour blank
    lp = np.log(probs).astype(np.float32)
    toks, _, st = oracle_lib.decode(lp, np.array([T], np.int32), 1000, 0.0, traces=True)
    k = len(toks[0])
    assert k >= 3 and toks[0] == [1] * k
    assert st["token_frames"][0] == [2 * j for j in range(k)]


# --------------------------------------------------------------------------- structural ties
def test_quantised_emissions_make_exact_score_ties(oracle_lib):
    """Emissions on a grid of 1/2 make different prefixes score the same: the five best final
    prefixes of this seeded utterance are bit-equal in the oracle, its choice among them is the
    hash order, and the margin it reports is 0 (tests/test_gpu_ties.py says what the GPU path
    owes on such inputs)."""
    lp = synth.random_emissions(22191, 300, 13, 5, flat=1.0)
    lp = (np.round(lp * 2) / 2).astype(np.float32)[215, :12]
    final = oracle_lib.decode_beam(lp, 128, 1.0, top_n=20, max_entries=128)
    totals = [float(np.logaddexp(pb, pnb)) for _, pb, pnb in final]
    assert len(totals) >= 5 and len(set(totals[:5])) == 1
    hashes = [oracle_lib.prefix_hash(tok) for tok, _, _ in final[:5]]
    assert hashes == sorted(hashes)
    toks, sc, st = oracle_lib.decode(lp[None], np.array([12], np.int32), 128, 1.0, top_n=20)
    assert tuple(toks[0]) == final[0][0] and st["min_decision_margin"] == 0.0
    # and a workload with continuous emissions has none
    w = synth.WORKLOADS["cfg2_batch64"]
    lp2, ln2 = synth.make_emissions(w, utterances=range(4))
    st2 = oracle_lib.decode(lp2, ln2, w.beam, 0.01, n_threads=4)[2]
    assert st2["min_decision_margin"] > 1e-9 and min(st2["margins"]) > 1e-9
