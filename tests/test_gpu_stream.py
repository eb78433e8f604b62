"""GPU parity for streaming (chunked) decoding: feeding an utterance in pieces with the beam
carried between calls must give what the oracle gives on the whole utterance, and after
every chunk what the oracle gives on the frames seen so far."""
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


def feed_in_chunks(dev, lp, ln, chunk, beam, r, check_at=(), oracle_lib=None, okw=None, **kw):
    B, T, V = lp.shape
    lm = kw.pop("lm", None)
    if lm is not None:
        kw["lm_table"] = torch.from_numpy(np.ascontiguousarray(lm)).to(dev)
    st = binding.Stream(B, T, chunk, V, beam, r, dev, want_traces=True, **kw)
    totals = {k: 0 for k in ("frames", "sum_survivors", "sum_candidates", "sum_beam")}
    peak = 0
    for t0 in range(0, T, chunk):
        tc = min(chunk, T - t0)
        piece = np.ascontiguousarray(lp[:, t0:t0 + tc])
        piece_len = np.clip(ln - t0, 0, tc).astype(np.int32)
        st.stats.zero_()
        st.feed(torch.from_numpy(piece).to(dev), torch.from_numpy(piece_len).to(dev))
        torch.cuda.synchronize()
        s = binding.stats_dict(st.stats)
        for k in totals:
            totals[k] += s[k]
        peak = max(peak, s["peak_candidates"])
        assert s["overflow_drops"] == 0
        if t0 + tc in check_at:  # partial transcript = decode of the frames seen so far
            seen = np.minimum(ln, t0 + tc).astype(np.int32)
            want = oracle_lib.decode(lp[:, :t0 + tc], seen, beam, r, n_threads=4, **(okw or {}))
            lens = st.lengths.cpu().numpy()
            toks = st.tokens.cpu().numpy()
            for b in range(B):
                assert toks[b, :lens[b]].tolist() == want[0][b], f"partial at {t0 + tc}, b={b}"
            ws = want[1].astype(np.float32)
            assert np.all(np.abs(st.scores.cpu().numpy().astype(np.float64) - ws) <= SCORE_TOL)
    lens = st.lengths.cpu().numpy()
    toks = st.tokens.cpu().numpy()
    tf = st.token_frames.cpu().numpy()
    totals["peak_candidates"] = peak
    return {"tokens": [toks[b, :lens[b]].tolist() for b in range(B)],
            "token_frames": [tf[b, :lens[b]].tolist() for b in range(B)],
            "frame_beam": st.frame_beam.cpu().numpy(), "scores": st.scores.cpu().numpy(),
            "stats": totals}


def check_final(got, want, ln, label):
    toks, scores, st = want
    for b in range(len(toks)):
        assert got["tokens"][b] == toks[b], f"{label}: utterance {b} tokens differ"
        assert got["token_frames"][b] == st["token_frames"][b], f"{label}: utterance {b} frames"
        n = int(ln[b])
        np.testing.assert_array_equal(got["frame_beam"][b, :n], st["frame_beam"][b, :n])
        assert (got["frame_beam"][b, n:] == -1).all()
    ws = np.asarray(scores, dtype=np.float64).astype(np.float32)
    assert np.all(np.abs(got["scores"].astype(np.float64) - ws) <= SCORE_TOL), label
    for key in ("frames", "sum_survivors", "sum_candidates", "peak_candidates", "sum_beam"):
        assert got["stats"][key] == st[key], (label, key)


@pytest.mark.parametrize("chunk", [1, 7, 32, 100, 333, 500])
def test_chunked_decode_equals_whole_decode(dev, oracle_lib, chunk):
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w, utterances=range(4 if chunk == 1 else 8))
    want = oracle_lib.decode(lp, ln, w.beam, 0.01, traces=True, n_threads=8)
    got = feed_in_chunks(dev, lp, ln, chunk, w.beam, 0.01)
    check_final(got, want, ln, f"chunk {chunk}")
    # and bit-identical to the one-shot GPU decode (same arithmetic in the same order)
    lp_d, ln_d = torch.from_numpy(lp).to(dev), torch.from_numpy(ln).to(dev)
    one = binding.decode(lp_d, ln_d, w.beam, 0.01)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(one["scores"].cpu().numpy(), got["scores"])


def test_streams_of_different_lengths_with_partial_transcripts(dev, oracle_lib):
    w = synth.WORKLOADS["cfg3_varlen256"]
    all_len = synth.make_lengths(w)
    order = np.argsort(all_len)
    idx = sorted({int(order[0]), int(order[1]), int(order[len(order) // 2]), int(order[-1])})
    lp, ln = synth.make_emissions(w, pad_value=0.0, utterances=idx)
    want = oracle_lib.decode(lp, ln, w.beam, 0.01, traces=True, n_threads=8)
    got = feed_in_chunks(dev, lp, ln, 160, w.beam, 0.01, check_at=(160, 480, 1120),
                         oracle_lib=oracle_lib)
    check_final(got, want, ln, "varlen chunks of 160")


def test_chunked_decode_with_lm_top_n_and_window(dev, oracle_lib):
    w = synth.WORKLOADS["cfg5_bigram_lm"]
    lp, ln = synth.make_emissions(w, utterances=range(4))
    lm = synth.make_bigram_lm(w.V)
    okw = dict(lm_table=lm, lm_weight=w.lm_weight, insertion_bonus=w.insertion_bonus, top_n=4,
               beam_threshold=6.0)
    want = oracle_lib.decode(lp, ln, w.beam, 0.007, traces=True, n_threads=4, **okw)
    got = feed_in_chunks(dev, lp, ln, 64, w.beam, 0.007, lm=lm, lm_weight=w.lm_weight,
                         insertion_bonus=w.insertion_bonus, top_n=4, beam_threshold=6.0,
                         check_at=(128,), oracle_lib=oracle_lib, okw=okw)
    check_final(got, want, ln, "lm + top-4 + window, chunks of 64")


def test_unpruned_chunks_and_restart(dev, oracle_lib):
    lp = synth.random_emissions(91, 2, 90, 40, flat=2.0)
    ln = np.array([90, 61], dtype=np.int32)
    want = oracle_lib.decode(lp, ln, 128, 0.0, traces=True, n_threads=2)
    got = feed_in_chunks(dev, lp, ln, 25, 128, 0.0)
    check_final(got, want, ln, "unpruned beam 128")
    # begin() again: the same state decodes a fresh pair of streams
    st = binding.Stream(2, 90, 45, 40, 128, 0.0, dev)
    for rep in range(2):
        st.begin()
        for t0 in (0, 45):
            piece_len = np.clip(ln - t0, 0, 45).astype(np.int32)
            st.feed(torch.from_numpy(np.ascontiguousarray(lp[:, t0:t0 + 45])).to(dev),
                    torch.from_numpy(piece_len).to(dev))
        torch.cuda.synchronize()
        lens = st.lengths.cpu().numpy()
        toks = st.tokens.cpu().numpy()
        for b in range(2):
            assert toks[b, :lens[b]].tolist() == want[0][b], f"restart {rep}"


def test_chunked_decode_with_a_large_beam(dev, oracle_lib):
    lp = synth.random_emissions(92, 2, 90, 32, flat=1.5)
    ln = np.array([90, 61], dtype=np.int32)
    want = oracle_lib.decode(lp, ln, 300, 0.001, traces=True, n_threads=2)
    got = feed_in_chunks(dev, lp, ln, 40, 300, 0.001)
    check_final(got, want, ln, "beam 300 in chunks of 40")


def test_chunked_decode_of_a_batch_larger_than_the_chip_holds(dev, oracle_lib):
    """Above two workgroups per compute unit the halved-register build of the search kernel
    runs; its carried state must round-trip like the other build's."""
    B, T, V, beam = 520, 48, 32, 24
    lp = synth.random_emissions(93, B, T, V, flat=1.5)
    ln = np.random.default_rng(93).integers(0, T + 1, size=B).astype(np.int32)
    want = oracle_lib.decode(lp, ln, beam, 1e-3, traces=True, n_threads=8)
    got = feed_in_chunks(dev, lp, ln, 20, beam, 1e-3)
    check_final(got, want, ln, "520 streams in chunks of 20")


def test_transcript_is_rewritten_only_where_it_changed(dev, oracle_lib):
    """A streaming decode keeps the trie node behind every token it has written and stops a
    rewrite where it meets one.  Partial transcripts after every chunk (they grow, switch
    and now and then shrink on flat emissions) must equal a fresh decode of the frames so
    far; changing the output rows between calls must give a full rewrite."""
    B, T, V, beam, r, chunk = 6, 60, 3, 16, 0.0, 1
    lp = synth.random_emissions(106, B, T, V, flat=0.3)
    ln = np.array([60, 60, 60, 41, 60, 7], dtype=np.int32)
    st = binding.Stream(B, T, chunk, V, beam, r, dev, want_traces=True)
    spare_tokens = torch.full_like(st.tokens, -7)
    shrank = 0
    prev = None
    for t0 in range(0, T, chunk):
        if t0 == 30:  # from here on the transcripts go to other rows
            st.tokens = spare_tokens
        piece_len = np.clip(ln - t0, 0, chunk).astype(np.int32)
        st.feed(torch.from_numpy(np.ascontiguousarray(lp[:, t0:t0 + chunk])).to(dev),
                torch.from_numpy(piece_len).to(dev))
        torch.cuda.synchronize()
        seen = np.minimum(ln, t0 + chunk).astype(np.int32)
        want = oracle_lib.decode(lp[:, :t0 + chunk], seen, beam, r, traces=True, n_threads=4)
        lens = st.lengths.cpu().numpy()
        toks = st.tokens.cpu().numpy()
        tf = st.token_frames.cpu().numpy()
        for b in range(B):
            assert toks[b, :lens[b]].tolist() == want[0][b], f"after {t0 + chunk} frames, b={b}"
            assert tf[b, :lens[b]].tolist() == want[2]["token_frames"][b], f"frames, b={b}"
        if prev is not None:
            shrank += int((lens < prev).sum())
        prev = lens.copy()
    assert shrank > 0, "the case is meant to contain transcripts that get shorter"


def test_stream_argument_errors(dev):
    assert binding.load().fltop_ctc_stream_state_bytes(0, 10, 4) == 0
    assert binding.load().fltop_ctc_stream_state_bytes(2, 10, binding.MAX_BEAM_STREAMING + 1) == 0
    st = binding.Stream(1, 8, 4, 8, 4, 0.1, dev)
    with pytest.raises(ValueError):
        st.feed(torch.zeros((1, 5, 8), dtype=torch.float32, device=dev),
                torch.full((1,), 5, dtype=torch.int32, device=dev))
    # frames beyond T_total are ignored, not written
    for _ in range(3):
        st.feed(torch.zeros((1, 4, 8), dtype=torch.float32, device=dev).log_softmax(-1),
                torch.full((1,), 4, dtype=torch.int32, device=dev))
    torch.cuda.synchronize()
    assert int(st.stats.cpu()[0]) >= 8  # frames counted: 4 + 4 (+ 0 for the chunk beyond the end)


def test_decode_can_be_captured_in_a_graph_and_replayed(dev, oracle_lib):
    """The entry points only enqueue kernels on the given stream (no allocation, no memset, no
    host synchronisation), so a serving loop can capture a decode once and replay it: every
    replay, with fresh emissions copied into the captured input buffer and the program's own
    eager work in between, must give what an eager call gives."""
    w = synth.WORKLOADS["cfg2_batch64"]
    lp_all, ln_all = synth.make_emissions(w, utterances=range(12))
    B = 4
    static_lp = torch.empty((B, w.T, w.V), dtype=torch.float32, device=dev)
    static_ln = torch.empty(B, dtype=torch.int32, device=dev)
    ws = binding.alloc_workspace(B, w.T, w.V, w.beam, dev)
    tok = torch.full((B, w.T), -1, dtype=torch.int32, device=dev)
    olen = torch.zeros(B, dtype=torch.int32, device=dev)
    sc = torch.zeros(B, dtype=torch.float32, device=dev)
    p = binding.FltopParams()
    p.beam = w.beam
    p.rel_threshold = 0.01
    static_lp.copy_(torch.from_numpy(lp_all[:B]))
    static_ln.copy_(torch.from_numpy(ln_all[:B]))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up outside the capture
        assert binding.decode_raw(static_lp, static_ln, p, ws, ws.numel(), tok, olen, sc, None) == 0
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rc = binding.decode_raw(static_lp, static_ln, p, ws, ws.numel(), tok, olen, sc, None)
    assert rc == 0
    for rep in range(3):
        sl = slice(rep * B, rep * B + B)
        static_lp.copy_(torch.from_numpy(lp_all[sl]))
        static_ln.copy_(torch.from_numpy(ln_all[sl]))
        tok.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        eager = binding.decode(static_lp, static_ln, w.beam, 0.01)  # eager work between replays
        torch.cuda.synchronize()
        want = oracle_lib.decode(lp_all[sl], ln_all[sl], w.beam, 0.01, n_threads=4)
        lens = olen.cpu().numpy()
        toks = tok.cpu().numpy()
        for b in range(B):
            assert toks[b, :lens[b]].tolist() == want[0][b], f"replay {rep}, utterance {b}"
        np.testing.assert_array_equal(sc.cpu().numpy(), eager["scores"].cpu().numpy())
        np.testing.assert_array_equal(lens, eager["lengths"].cpu().numpy())
