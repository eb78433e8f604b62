"""The seeded input generators: both the oracle and the HIP path read their bytes, so they
are pinned here -- shapes, determinism, independence of an utterance from its batch, and
the statistics the workload recipe states (blank rate, hard-frame rate, length range, rows
that are log-probabilities, a finite bigram table)."""
import hashlib

import numpy as np
import pytest

from paper_2510_09085_amd import synth


def test_workload_table_matches_the_five_configurations():
    w = synth.WORKLOADS
    assert (w["cfg1_single"].B, w["cfg1_single"].T, w["cfg1_single"].V, w["cfg1_single"].beam) == (1, 200, 32, 8)
    assert (w["cfg2_batch64"].B, w["cfg2_batch64"].T, w["cfg2_batch64"].V, w["cfg2_batch64"].beam) == (64, 500, 32, 32)
    assert tuple(w["cfg2_batch64"].rel_thresholds) == (0.1, 0.01, 0.001, 0.0)
    c3 = w["cfg3_varlen256"]
    assert (c3.B, c3.T, c3.V, c3.beam, c3.hard_rate, tuple(c3.variable_lengths)) == (256, 1500, 32, 100, 0.25, (250, 1500))
    c4 = w["cfg4_subword1024"]
    assert (c4.B, c4.T, c4.V, c4.beam, c4.zipf_s) == (128, 400, 1024, 64, 1.1)
    c5 = w["cfg5_bigram_lm"]
    assert (c5.B, c5.T, c5.V, c5.beam, c5.use_lm, c5.lm_weight, c5.insertion_bonus) == (128, 500, 32, 64, True, 0.5, 1.0)
    assert synth.FRAMES_PER_SECOND == 50


def test_same_seed_same_bytes_and_utterances_do_not_depend_on_the_batch():
    w = synth.WORKLOADS["cfg2_batch64"]
    a, la = synth.make_emissions(w, utterances=[3, 17, 40])
    b, lb = synth.make_emissions(w, utterances=[17])
    c, lc = synth.make_emissions(w, utterances=[3, 17, 40])
    assert hashlib.sha256(a.tobytes()).hexdigest() == hashlib.sha256(c.tobytes()).hexdigest()
    np.testing.assert_array_equal(a[1], b[0])
    np.testing.assert_array_equal(la, lc)
    assert not np.array_equal(a[0], a[1])
    other = synth.utterance_emissions(w.seed + 1, 3, w.T, w.V)
    assert not np.array_equal(other, a[0])


@pytest.mark.parametrize("name", ["cfg2_batch64", "cfg3_varlen256", "cfg4_subword1024"])
def test_rows_are_log_probabilities_with_the_stated_peakiness(name):
    w = synth.WORKLOADS[name]
    lp, ln = synth.make_emissions(w, pad_value=0.0, utterances=range(6))
    assert lp.dtype == np.float32 and lp.shape == (6, w.T, w.V)
    valid = np.concatenate([lp[b, :ln[b]] for b in range(6)])
    np.testing.assert_allclose(np.exp(valid.astype(np.float64)).sum(axis=1), 1.0, atol=1e-5)
    top = valid.argmax(axis=1)
    blank_rate = float((top == 0).mean())
    assert abs(blank_rate - w.p_blank) < 0.06          # boost 6..12 nearly always wins the frame
    # survivors at r = 0.01: one on plain frames, two or more mostly on hard frames
    thr = valid.max(axis=1, keepdims=True) + np.float32(np.log(0.01))
    multi = float(((valid >= thr).sum(axis=1) > 1).mean())
    assert 0.3 * w.hard_rate < multi < 3.0 * w.hard_rate + 0.25


def test_variable_lengths_and_padding():
    w = synth.WORKLOADS["cfg3_varlen256"]
    ln = synth.make_lengths(w)
    assert ln.dtype == np.int32 and ln.shape == (256,)
    assert ln.min() >= 250 and ln.max() <= 1500 and len(set(ln.tolist())) > 100
    np.testing.assert_array_equal(ln, synth.make_lengths(w))
    lp, l2 = synth.make_emissions(w, utterances=[0, 1])
    for b in range(2):
        assert np.isnan(lp[b, l2[b]:]).all() and not np.isnan(lp[b, :l2[b]]).any()
    assert (synth.make_lengths(synth.WORKLOADS["cfg2_batch64"]) == 500).all()


def test_zipf_prior_favours_low_token_ids():
    w = synth.WORKLOADS["cfg4_subword1024"]
    lp, _ = synth.make_emissions(w, utterances=[0])
    mean_lp = lp[0].astype(np.float64).mean(axis=0)
    assert mean_lp[1:17].mean() > mean_lp[500:516].mean() + 3.0   # -1.1 ln v


def test_bigram_table_is_finite_row_stochastic_and_seeded():
    for V in (6, 32, 1024):
        lm = synth.make_bigram_lm(V)
        assert lm.shape == (V, V) and lm.dtype == np.float32 and np.isfinite(lm).all()
        np.testing.assert_allclose(np.exp(lm.astype(np.float64)).sum(axis=1), 1.0, atol=1e-4)
        np.testing.assert_array_equal(lm, synth.make_bigram_lm(V))
    assert not np.array_equal(synth.make_bigram_lm(32, seed=1), synth.make_bigram_lm(32, seed=2))
    assert synth.make_bigram_lm(32).min() >= np.float32(np.log(1e-30)) - 1e-3
