"""Structural score ties: what the GPU path must still satisfy where bit-exact tokens are not
defined.

Both sides evaluate the same expression (same order of additions, same two-operand
log-sum-exps), in fp64; they differ only in how exp and log1p round their last bit.  On
emissions drawn from a continuous distribution every comparison the search makes is decided by
gaps many orders of magnitude above that (the oracle reports the smallest gap that decided
anything: `min_decision_margin`), and tokens must agree bit for bit.  Emissions quantised to
multiples of 1/2 make different prefixes score *mathematically* the same; whether two such
scores come out bit-equal (then the hash order decides) or one ulp apart (then the score
decides) depends on the last bit of exp/log1p, so the two sides may resolve such a tie
differently.  For an utterance whose oracle margin is at or below TIE_MARGIN the bar is:
  * the GPU's prefix is in the oracle's final beam,
  * its oracle score is within TIE_MARGIN of the oracle's best score (it IS one of the tied bests),
  * the GPU's score agrees with that oracle score to 1e-4,
and for every other utterance the full bar (tokens, lengths, per-frame beam sizes exact).

The first two cases are the two mismatches a 200-case random sweep once showed (an earlier
kernel also kept scores relative to a shared offset, which changed the association of the
additions; it no longer does)."""
import numpy as np
import pytest
import torch

from paper_2510_09085_amd import binding, synth

pytestmark = pytest.mark.gpu

TIE_MARGIN = 1e-9
SCORE_TOL = 1e-4


def quantised(seed, B, T, V, flat):
    lp = synth.random_emissions(seed, B, T, V, flat=flat)
    return (np.round(lp * 2) / 2).astype(np.float32)


def check_case(dev, oracle_lib, lp, ln, beam, r, top_n, window, label, lm=None, lm_weight=0.0,
               insertion_bonus=0.0):
    B, T, V = lp.shape
    okw = dict(top_n=top_n, beam_threshold=window)
    gkw = dict(okw)
    if lm is not None:
        okw.update(lm_table=lm, lm_weight=lm_weight, insertion_bonus=insertion_bonus)
        gkw.update(lm_table=torch.from_numpy(lm).to(dev), lm_weight=lm_weight,
                   insertion_bonus=insertion_bonus)
    want_tok, want_sc, st = oracle_lib.decode(lp, ln, beam, r, n_threads=8, traces=True, **okw)
    out = binding.decode(torch.from_numpy(lp).to(dev), torch.from_numpy(ln).to(dev), beam, r,
                         want_traces=True, want_stats=True, **gkw)
    torch.cuda.synchronize()
    lens = out["lengths"].cpu().numpy()
    toks = out["tokens"].cpu().numpy()
    scores = out["scores"].cpu().numpy()
    fb = out["frame_beam"].cpu().numpy()
    got_st = binding.stats_dict(out["stats"])
    assert got_st["overflow_drops"] == 0
    assert got_st["frames"] == st["frames"] and got_st["sum_survivors"] == st["sum_survivors"]
    if min(st["margins"], default=1.0) > TIE_MARGIN:  # no tie anywhere: every count must agree
        for key in ("sum_candidates", "peak_candidates", "sum_beam"):
            assert got_st[key] == st[key], (label, key)
    n_tied = n_other_choice = 0
    for b in range(B):
        got = toks[b, :lens[b]].tolist()
        if st["margins"][b] > TIE_MARGIN:  # nothing was close: the full bar
            assert got == want_tok[b], f"{label}: utterance {b} tokens differ"
            if np.isfinite(want_sc[b]):
                assert abs(float(scores[b]) - float(np.float32(want_sc[b]))) <= SCORE_TOL
            else:
                assert scores[b] == np.float32(want_sc[b])
            np.testing.assert_array_equal(fb[b, :ln[b]], st["frame_beam"][b, :ln[b]])
            continue
        n_tied += 1
        if ln[b] == 0:
            assert got == []
            continue
        final = oracle_lib.decode_beam(lp[b, :ln[b]], beam, r, max_entries=beam, **okw)
        totals = {tok: np.logaddexp(pb, pnb) for tok, pb, pnb in final}
        assert tuple(got) in totals, f"{label}: utterance {b}: GPU prefix not in the oracle's final beam"
        mine = totals[tuple(got)]
        assert want_sc[b] - mine <= TIE_MARGIN, \
            f"{label}: utterance {b}: GPU prefix scores {mine!r}, the oracle's best {want_sc[b]!r}"
        assert abs(float(scores[b]) - float(np.float32(mine))) <= SCORE_TOL
        n_other_choice += got != want_tok[b]
    return n_tied, n_other_choice


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load()
    return torch.device("cuda:0")


def test_the_two_known_tie_cases(dev, oracle_lib):
    # (seed, B, T, V, flat, utterance, frames, beam, r, top_n, window)
    for seed, B, T, V, flat, b, n, beam, r, top_n, window in (
            (22191, 300, 13, 5, 1.0, 215, 12, 128, 1.0, 20, 0.0),
            (22199, 300, 40, 5, 2.0, 187, 38, 65, 0.1, 20, 3.0)):
        lp = quantised(seed, B, T, V, flat)[b:b + 1].copy()
        ln = np.array([n], dtype=np.int32)
        lp[0, n:] = np.nan
        tied, _ = check_case(dev, oracle_lib, lp, ln, beam, r, top_n, window, f"seed {seed}")
        assert tied == 1  # the oracle itself says this utterance was decided by a tie


@pytest.mark.parametrize("seed", range(6))
def test_tie_heavy_batches(dev, oracle_lib, seed):
    """Batches of quantised emissions with thresholds, token stages and windows that sit on the
    quantisation grid (r = 1 keeps exactly the ties of the top; a window of 3.0 or 0.5 puts
    candidates on the floor)."""
    rng = np.random.default_rng(4400 + seed)
    V = int(rng.choice([3, 5, 8, 32]))
    beam = int(rng.choice([4, 32, 65, 128, 300]))
    r = float(rng.choice([0.0, 0.1, 1.0]))
    top_n = int(rng.choice([0, 4, 20]))
    window = float(rng.choice([0.0, 0.5, 3.0]))
    flat = float(rng.choice([1.0, 2.0]))
    B, T = 120, int(rng.integers(8, 41))
    lp = quantised(5500 + seed, B, T, V, flat)
    ln = rng.integers(0, T + 1, size=B).astype(np.int32)
    ln[0] = T
    tied, other = check_case(dev, oracle_lib, lp, ln, beam, r, top_n, window,
                             f"seed {seed} V{V} beam{beam} r{r} N{top_n} win{window}")
    print(f"seed {seed}: {tied} of {B} utterances decided by a tie, {other} resolved differently")
