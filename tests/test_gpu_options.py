"""GPU parity for the optional stages: static top-N token stage (Alg. 1), SelectTopK's score
window, the statistics traces (paper Sec. 4.1 / 4.4) and the token-rank statistic.  Same bar
as the main parity tests: integers bit-exact, scores within 1e-4 of the fp32-rounded oracle."""
import numpy as np
import pytest
import torch

from paper_2510_09085_amd import binding, synth

pytestmark = pytest.mark.gpu

SCORE_TOL = 1e-4


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load()
    return torch.device("cuda:0")


def tied_emissions(seed, B, T, V, levels=6):
    rng = np.random.default_rng(seed)
    vals = -np.arange(levels, dtype=np.float32) * np.float32(0.75)
    return vals[rng.integers(0, levels, size=(B, T, V))]


def gpu_decode(dev, lp, ln, beam, r, **kw):
    lp_d = torch.from_numpy(np.ascontiguousarray(lp)).to(dev)
    ln_d = torch.from_numpy(np.ascontiguousarray(ln, dtype=np.int32)).to(dev)
    lm = kw.pop("lm", None)
    if lm is not None:
        kw["lm_table"] = torch.from_numpy(np.ascontiguousarray(lm)).to(dev)
    out = binding.decode(lp_d, ln_d, beam, r, want_stats=True, want_traces=True, **kw)
    torch.cuda.synchronize()
    lens = out["lengths"].cpu().numpy()
    toks = out["tokens"].cpu().numpy()
    tf = out["token_frames"].cpu().numpy()
    return {
        "tokens": [toks[b, :lens[b]].tolist() for b in range(len(lens))],
        "token_frames": [tf[b, :lens[b]].tolist() for b in range(len(lens))],
        "frame_beam": out["frame_beam"].cpu().numpy(),
        "scores": out["scores"].cpu().numpy(),
        "stats": binding.stats_dict(out["stats"]),
        "dev": (lp_d, out),
    }


def check(got, want, ln, label):
    toks, scores, st = want
    for b in range(len(toks)):
        assert got["tokens"][b] == toks[b], f"{label}: utterance {b} tokens differ"
        assert got["token_frames"][b] == st["token_frames"][b], f"{label}: utterance {b} frames"
        n = int(ln[b])
        np.testing.assert_array_equal(got["frame_beam"][b, :n], st["frame_beam"][b, :n],
                                      err_msg=f"{label}: utterance {b} beam sizes")
        assert (got["frame_beam"][b, n:] == -1).all()  # padding frames are not touched
    ws = np.asarray(scores, dtype=np.float64).astype(np.float32)
    gs = got["scores"]
    both_inf = np.isneginf(ws) & np.isneginf(gs)
    with np.errstate(invalid="ignore"):
        close = np.abs(gs.astype(np.float64) - ws.astype(np.float64)) <= SCORE_TOL
    assert np.all(both_inf | close), f"{label}: scores differ {gs} vs {ws}"
    for key in ("frames", "sum_survivors", "sum_candidates", "peak_candidates", "sum_beam"):
        assert got["stats"][key] == st[key], (label, key)
    assert got["stats"]["overflow_drops"] == 0


# --------------------------------------------------------------------------- top-N stage
@pytest.mark.parametrize("V", [2, 3, 5, 29, 32, 33, 64, 100, 257, 1024, 1500])
def test_top_n_survivor_lists_are_byte_identical(dev, oracle_lib, V):
    B, T = 3, 37
    lp = np.concatenate([synth.random_emissions(3000 + V, B - 1, T, V, flat=2.5),
                         tied_emissions(V, 1, T, V)])
    lp[1, 5, V // 2] = -np.inf
    ln = np.array([T, 11, T], dtype=np.int32)
    lp[1, 11:] = np.nan
    lp_d = torch.from_numpy(lp).to(dev)
    ln_d = torch.from_numpy(ln).to(dev)
    for n in sorted({1, 2, 4, 7, V - 1, V, V + 3}):
        if n < 1:
            continue
        for r in (0.0, 1e-3, 0.3, 1.0):
            ws = binding.prune(lp_d, ln_d, 4, r, top_n=n)
            counts, tokens, values, fmax = [x.cpu().numpy() for x in
                                            binding.unpack_survivors(ws, ln_d, B, T, V, 4)]
            for b in range(B):
                m = ln[b]
                oc, ot, om = oracle_lib.survivors(lp[b, :m], r, top_n=n)
                sl = slice(b * T, b * T + m)
                np.testing.assert_array_equal(counts[sl], oc, err_msg=f"V={V} N={n} r={r} b={b}")
                np.testing.assert_array_equal(fmax[sl].view(np.uint32), om.view(np.uint32))
                for f in range(m):
                    k = oc[f]
                    np.testing.assert_array_equal(tokens[b * T + f, :k], ot[f, :k],
                                                  err_msg=f"V={V} N={n} r={r} b={b} f={f}")
                    np.testing.assert_array_equal(
                        values[b * T + f, :k].view(np.uint32),
                        lp[b, f, ot[f, :k]].view(np.uint32))


@pytest.mark.parametrize("name,n_utt", [("cfg2_batch64", 6), ("cfg3_varlen256", 3),
                                        ("cfg4_subword1024", 2), ("cfg5_bigram_lm", 4)])
def test_paper_arms_top4_and_fltop(dev, oracle_lib, name, n_utt):
    """The paper's Top-N arm (N = 4, R = 0) and FLToP arm (N = 4, R = 0.007) on the synthetic
    stand-ins of the workloads."""
    w = synth.WORKLOADS[name]
    lp, ln = synth.make_emissions(w, utterances=range(n_utt))
    lm = synth.make_bigram_lm(w.V) if w.use_lm else None
    kw = dict(lm=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus) if w.use_lm else {}
    okw = dict(lm_table=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus) if w.use_lm else {}
    for r in (0.0, 0.007):
        got = gpu_decode(dev, lp, ln, w.beam, r, top_n=4, **kw)
        want = oracle_lib.decode(lp, ln, w.beam, r, top_n=4, traces=True, n_threads=8, **okw)
        check(got, want, ln, f"{name} N=4 r={r}")


def test_top_n_with_ties_decodes_like_the_oracle(dev, oracle_lib):
    lp = tied_emissions(17, 4, 60, 12, levels=4)
    ln = np.array([60, 60, 31, 1], dtype=np.int32)
    for n in (1, 2, 3, 5):
        for r in (0.0, 0.2):
            got = gpu_decode(dev, lp, ln, 16, r, top_n=n)
            want = oracle_lib.decode(lp, ln, 16, r, top_n=n, traces=True)
            check(got, want, ln, f"ties N={n} r={r}")


# --------------------------------------------------------------------------- score window
@pytest.mark.parametrize("window", [0.25, 2.0, 6.0, 25.0, 1e30])
def test_score_window_small_cases(dev, oracle_lib, window):
    for seed, (B, T, V, beam) in enumerate([(3, 50, 6, 16), (2, 80, 32, 64), (2, 40, 200, 128)]):
        lp = synth.random_emissions(6100 + seed, B, T, V, flat=1.5)
        ln = np.array([T] * (B - 1) + [T // 2], dtype=np.int32)
        for r in (0.0, 0.01):
            got = gpu_decode(dev, lp, ln, beam, r, beam_threshold=window)
            want = oracle_lib.decode(lp, ln, beam, r, beam_threshold=window, traces=True)
            check(got, want, ln, f"window={window} case {seed} r={r}")


@pytest.mark.parametrize("name,n_utt,window", [("cfg2_batch64", 6, 6.0), ("cfg3_varlen256", 3, 10.0),
                                               ("cfg4_subword1024", 2, 3.0),
                                               ("cfg5_bigram_lm", 4, 6.0)])
def test_score_window_on_workloads(dev, oracle_lib, name, n_utt, window):
    w = synth.WORKLOADS[name]
    lp, ln = synth.make_emissions(w, utterances=range(n_utt))
    lm = synth.make_bigram_lm(w.V) if w.use_lm else None
    kw = dict(lm=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus) if w.use_lm else {}
    okw = dict(lm_table=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus) if w.use_lm else {}
    for r, n in ((0.01, 0), (0.007, 4)):
        got = gpu_decode(dev, lp, ln, w.beam, r, top_n=n, beam_threshold=window, **kw)
        want = oracle_lib.decode(lp, ln, w.beam, r, top_n=n, beam_threshold=window, traces=True,
                                 n_threads=8, **okw)
        check(got, want, ln, f"{name} window={window} r={r} N={n}")
        free = oracle_lib.decode(lp, ln, w.beam, r, top_n=n, n_threads=8, **okw)[2]
        assert got["stats"]["sum_beam"] < free["sum_beam"]  # the window does shrink the beam


def test_window_off_values_change_nothing(dev, oracle_lib):
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(4))
    base = gpu_decode(dev, lp, ln, w.beam, 0.01)
    for off in (0.0, -3.0):
        got = gpu_decode(dev, lp, ln, w.beam, 0.01, beam_threshold=off)
        assert got["tokens"] == base["tokens"]
        np.testing.assert_array_equal(got["scores"], base["scores"])
        np.testing.assert_array_equal(got["frame_beam"], base["frame_beam"])


# --------------------------------------------------------------------------- traces and ranks
@pytest.mark.parametrize("name,n_utt", [("cfg1_single", 1), ("cfg2_batch64", 8),
                                        ("cfg5_bigram_lm", 4)])
def test_traces_without_options(dev, oracle_lib, name, n_utt):
    w = synth.WORKLOADS[name]
    lp, ln = synth.make_emissions(w, utterances=range(n_utt))
    lm = synth.make_bigram_lm(w.V) if w.use_lm else None
    kw = dict(lm=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus) if w.use_lm else {}
    okw = dict(lm_table=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus) if w.use_lm else {}
    for r in w.rel_thresholds:
        got = gpu_decode(dev, lp, ln, w.beam, r, **kw)
        want = oracle_lib.decode(lp, ln, w.beam, r, traces=True, n_threads=8, **okw)
        check(got, want, ln, f"{name} r={r}")


def test_traces_on_dead_and_empty_utterances(dev, oracle_lib):
    lp = synth.random_emissions(5, 3, 12, 4)
    lp[1, 6, :] = -np.inf  # every route dies at frame 6
    ln = np.array([0, 12, 12], dtype=np.int32)
    got = gpu_decode(dev, lp, ln, 4, 0.1)
    want = oracle_lib.decode(lp, ln, 4, 0.1, traces=True)
    check(got, want, ln, "dead")
    assert (got["frame_beam"][1, 6:] == 0).all()


def test_token_rank_statistic(dev, oracle_lib):
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(8))
    B, T, V = lp.shape
    got = gpu_decode(dev, lp, ln, w.beam, 0.01)
    lp_d, out = got["dev"]
    ranks, count, lp_sum = binding.token_ranks(lp_d, out["tokens"], out["token_frames"],
                                               out["lengths"])
    torch.cuda.synchronize()
    ranks, count, lp_sum = ranks.cpu().numpy(), count.cpu().numpy(), lp_sum.cpu().numpy()
    want_count = np.zeros(V, dtype=np.int64)
    want_sum = np.zeros(V, dtype=np.float64)
    for b in range(B):
        toks, frames = got["tokens"][b], got["token_frames"][b]
        want = oracle_lib.token_ranks(lp[b], toks, frames)
        np.testing.assert_array_equal(ranks[b, :len(toks)], want)
        assert (ranks[b, len(toks):] == -1).all()
        for tok, f, k in zip(toks, frames, want):
            want_count[k] += 1
            want_sum[k] += float(lp[b, f, tok])
    np.testing.assert_array_equal(count, want_count)
    np.testing.assert_allclose(lp_sum, want_sum, rtol=0, atol=1e-9)
    assert count.sum() == sum(len(t) for t in got["tokens"])
    # tied emissions: the position counts equal values at lower token ids as "ahead"
    lp2 = tied_emissions(3, 2, 30, 9)
    ln2 = np.array([30, 30], dtype=np.int32)
    got2 = gpu_decode(dev, lp2, ln2, 8, 0.0)
    lp2_d, out2 = got2["dev"]
    r2 = binding.token_ranks(lp2_d, out2["tokens"], out2["token_frames"], out2["lengths"])[0]
    torch.cuda.synchronize()
    for b in range(2):
        want = oracle_lib.token_ranks(lp2[b], got2["tokens"][b], got2["token_frames"][b])
        np.testing.assert_array_equal(r2.cpu().numpy()[b, :len(want)], want)


def test_option_errors_reach_the_caller(dev):
    lp = torch.zeros((1, 4, 8), dtype=torch.float32, device=dev)
    ln = torch.full((1,), 4, dtype=torch.int32, device=dev)
    with pytest.raises(binding.FltopError) as e:
        binding.decode(lp, ln, 4, 0.1, top_n=-1)
    assert e.value.status == -9
    with pytest.raises(binding.FltopError) as e:
        binding.decode(lp, ln, 4, 0.1, beam_threshold=float("nan"))
    assert e.value.status == -9


# --------------------------------------------------------------------------- larger LM
def test_subword_vocabulary_with_global_memory_bigram_table(dev, oracle_lib):
    """V = 1024 with a dense bigram table (4 MB: gathered from global memory, not LDS), the
    whole batch on the GPU in its benchmark launch shape, a sample of it in the oracle."""
    w = synth.WORKLOADS["ext_subword1024_lm"]
    lp, ln = synth.make_emissions(w)
    lm = synth.make_bigram_lm(w.V)
    got = gpu_decode(dev, lp, ln, w.beam, 0.01, lm=lm, lm_weight=w.lm_weight,
                     insertion_bonus=w.insertion_bonus)
    idx = list(range(0, w.B, 16))
    want = oracle_lib.decode(lp[idx], ln[idx], w.beam, 0.01, lm_table=lm, lm_weight=w.lm_weight,
                             insertion_bonus=w.insertion_bonus, traces=True, n_threads=8)
    for k, b in enumerate(idx):
        assert got["tokens"][b] == want[0][k], f"utterance {b}"
        assert got["token_frames"][b] == want[2]["token_frames"][k]
        np.testing.assert_array_equal(got["frame_beam"][b, :ln[b]], want[2]["frame_beam"][k, :ln[b]])
        assert abs(float(got["scores"][b]) - float(np.float32(want[1][k]))) <= SCORE_TOL
    assert got["stats"]["frames"] == int(ln.sum())
    assert got["stats"]["overflow_drops"] == 0


# --------------------------------------------------------------------------- log-sum-exp
def test_log_add_against_extended_precision(dev):
    """The search stage's own log-sum-exp against numpy's in 80-bit arithmetic: the term
    log1p(exp(min - max)) within 2.5 ulp of itself, plus the half ulp of the final addition."""
    rng = np.random.default_rng(5)
    n = 200000
    a = -rng.random(n) * 400.0
    gap = np.concatenate([rng.random(n // 4) * 45.0, rng.random(n // 4) * 2.0,
                          np.ldexp(rng.random(n // 4), -rng.integers(0, 60, n // 4)),
                          30.0 + rng.random(n - 3 * (n // 4)) * 600.0])
    b = a - gap
    swap = rng.random(n) < 0.5
    a, b = np.where(swap, b, a), np.where(swap, a, b)
    a[:50] = -np.inf
    b[25:75] = -np.inf
    a[100:110] = b[100:110]  # equal operands: max + ln 2
    got = binding.log_add(torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)).cpu().numpy()
    with np.errstate(invalid="ignore"):
        ref = np.logaddexp(a.astype(np.longdouble), b.astype(np.longdouble))
        term = np.log1p(np.exp(-np.abs(a.astype(np.longdouble) - b.astype(np.longdouble))))
    both_inf = np.isneginf(got) & np.isneginf(ref.astype(np.float64))
    assert both_inf[25:50].all() and not np.isnan(got).any()
    fin = np.isfinite(a) & np.isfinite(b)
    bound = 0.5 * np.spacing(np.abs(ref[fin].astype(np.float64))) + \
        2.5 * np.spacing(term[fin].astype(np.float64))
    err = np.abs((got[fin].astype(np.longdouble) - ref[fin]).astype(np.float64))
    assert (err <= bound).all(), float((err / bound).max())
    np.testing.assert_array_equal(got[:25], b[:25])   # -inf is the neutral element
    np.testing.assert_array_equal(got[50:75], a[50:75])
    # symmetric in its operands, bit for bit
    back = binding.log_add(torch.from_numpy(b).to(dev), torch.from_numpy(a).to(dev)).cpu().numpy()
    np.testing.assert_array_equal(got, back)
