"""GPU parity on seeded random configurations: vocabulary, beam, threshold, top-N, score
window, LM, tie-heavy (coarsely quantised) emissions and ragged lengths are drawn together,
so that corners no hand-written case names get visited.  Same bar as the other parity
tests: tokens, lengths and integer statistics exact, scores within 1e-4, per-frame beam
sizes exact."""
import numpy as np
import pytest
import torch

from paper_2510_09085_amd import binding, synth

pytestmark = pytest.mark.gpu

SCORE_TOL = 1e-4
VOCABS = [2, 3, 7, 32, 33, 64, 65, 100, 500, 1024, 2933, 4096]
BEAMS = [1, 2, 7, 32, 64, 65, 128, 129, 300, 512]


def draw_case(rng, seed, vocabs=VOCABS, beams=BEAMS):
    V = int(rng.choice(vocabs))
    beam = int(rng.choice(beams))
    r = float(rng.choice([0.0, 0.0, 1e-4, 1e-3, 0.01, 0.1, 0.5, 1.0]))
    top_n = int(rng.choice([0, 0, 1, 2, 4, 7, 50]))
    window = float(rng.choice([0.0, 0.0, 0.5, 3.0, 25.0]))
    use_lm = bool(rng.random() < 0.4)
    flat = float(rng.choice([0.3, 1.0, 2.0, 4.0]))
    quantised = bool(rng.random() < 0.25)
    # keep the oracle's work per case to a few million candidate updates
    per_frame = beam * (V if r < 1e-3 and top_n == 0 else min(V, 16))
    T = int(rng.integers(2, int(max(2, min(60, 6e6 // per_frame))) + 1))
    B = int(rng.choice([1, 2, 5]))
    if per_frame * T * B > 3e7:
        B = 1
    lp = synth.random_emissions(seed, B, T, V, flat=flat)
    if quantised:
        lp = (np.round(lp * 2) / 2).astype(np.float32)
    ln = rng.integers(0, T + 1, size=B).astype(np.int32)
    ln[0] = T
    lm = synth.make_bigram_lm(V, seed=seed) if use_lm else None
    if lm is not None and quantised:
        lm = np.round(lm).astype(np.float32)
    label = (f"B{B} T{T} V{V} beam{beam} r{r} N{top_n} window{window} lm{use_lm} "
             f"flat{flat} quantised{quantised}")
    return lp, ln, beam, r, top_n, window, lm, label


@pytest.mark.parametrize("seed0", [11, 12, 13])
def test_random_configurations(oracle_lib, seed0):
    assert torch.cuda.is_available(), "these tests need the MI355X"
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed0)
    for case in range(60):
        lp, ln, beam, r, top_n, window, lm, label = draw_case(rng, seed0 * 1000 + case)
        label = f"seed {seed0} case {case}: {label}"
        okw = dict(top_n=top_n, beam_threshold=window)
        gkw = dict(okw)
        if lm is not None:
            okw.update(lm_table=lm, lm_weight=0.7, insertion_bonus=0.3)
            gkw.update(lm_table=torch.from_numpy(lm).to(dev), lm_weight=0.7, insertion_bonus=0.3)
        want_tok, want_sc, want_st = oracle_lib.decode(lp, ln, beam, r, n_threads=8, traces=True,
                                                       **okw)
        out = binding.decode(torch.from_numpy(lp).to(dev), torch.from_numpy(ln).to(dev), beam, r,
                             want_stats=True, want_traces=True, **gkw)
        torch.cuda.synchronize()
        lens = out["lengths"].cpu().numpy()
        toks = out["tokens"].cpu().numpy()
        for b in range(len(ln)):
            assert toks[b, :lens[b]].tolist() == want_tok[b], f"{label}: utterance {b}"
        ws = np.asarray(want_sc, dtype=np.float64).astype(np.float32)
        gs = out["scores"].cpu().numpy()
        fin = np.isfinite(ws)
        assert np.all(np.abs(gs[fin].astype(np.float64) - ws[fin]) <= SCORE_TOL), label
        assert np.all(gs[~fin] == ws[~fin]), label
        st = binding.stats_dict(out["stats"])
        for key in ("frames", "sum_survivors", "sum_candidates", "peak_candidates", "sum_beam"):
            assert st[key] == want_st[key], (label, key)
        assert st["overflow_drops"] == 0, label
        fb = out["frame_beam"].cpu().numpy()
        for b in range(len(ln)):
            np.testing.assert_array_equal(fb[b, :ln[b]], want_st["frame_beam"][b, :ln[b]], label)


@pytest.mark.parametrize("seed0", [21, 22])
def test_random_configurations_with_beams_beyond_512(oracle_lib, seed0):
    """The same generator over the beam sizes of the 1024-entry build (and a few below, so
    that the three capacities alternate), vocabularies up to its limit.  Utterances the oracle
    reports as decided by an exact tie (quantised emissions) are held to the tie contract of
    tests/test_gpu_ties.py, all others to the full bar."""
    from test_gpu_ties import check_case
    assert torch.cuda.is_available(), "these tests need the MI355X"
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed0)
    for case in range(40):
        lp, ln, beam, r, top_n, window, lm, label = draw_case(
            rng, seed0 * 1000 + case, vocabs=[2, 5, 32, 33, 100, 700, binding.MAX_VOCAB_WIDE_BEAM],
            beams=[100, 512, 513, 600, 1000, 1023, binding.MAX_BEAM])
        check_case(dev, oracle_lib, lp, ln, beam, r, top_n, window,
                   f"seed {seed0} case {case}: {label}", lm=lm, lm_weight=0.7, insertion_bonus=0.3)


@pytest.mark.parametrize("seed0", [31, 32])
def test_random_configurations_on_peaky_emissions(oracle_lib, seed0):
    """Emissions of the workload generator (a dominant token per frame, so a threshold leaves
    runs of blank-only frames of every length, also across the 32-frame header chunks of the
    search kernel), with utterance lengths, beams of all three capacities, thresholds, top-N,
    windows and bigram tables drawn at random.  Same bars as above."""
    from test_gpu_ties import check_case
    assert torch.cuda.is_available(), "these tests need the MI355X"
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed0)
    for case in range(50):
        V = int(rng.choice([2, 3, 32, 32, 33, 100, 1024]))
        beam = int(rng.choice([1, 8, 32, 64, 100, 128, 129, 513, 1000]))
        r = float(rng.choice([1e-3, 0.007, 0.01, 0.01, 0.1, 0.5, 1.0]))
        top_n = int(rng.choice([0, 0, 1, 4]))
        window = float(rng.choice([0.0, 0.0, 3.0, 25.0]))
        B = int(rng.choice([1, 3, 9]))
        T = int(rng.integers(2, 400))
        w = synth.Workload("random", B=B, T=T, V=V, beam=beam, rel_thresholds=(r,),
                           seed=seed0 * 100000 + case,
                           hard_rate=float(rng.choice([0.1, 0.25, 0.5])))
        lp, _ = synth.make_emissions(w)
        ln = rng.integers(0, T + 1, size=B).astype(np.int32)
        ln[0] = T
        lm = synth.make_bigram_lm(V, seed=case) if rng.random() < 0.3 else None
        check_case(dev, oracle_lib, lp, ln, beam, r, top_n, window,
                   f"seed {seed0} case {case}: B{B} T{T} V{V} beam{beam} r{r} N{top_n} "
                   f"window{window} lm{lm is not None}", lm=lm, lm_weight=0.7, insertion_bonus=0.3)
