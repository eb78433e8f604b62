"""fltop_ctc_decode_static (the entry point for callers that cannot allocate: its workspace is
an array inside the library's device image) against fltop_ctc_decode, through the C ABI: same
tokens, lengths, scores and statistics, bit for bit, on two calls in a row, the second with a
smaller input (so it runs over what the first left in the array), then on a larger one again;
shapes beyond the array are refused."""
import numpy as np
import pytest
import torch

from paper_2510_09085_amd import binding, synth

pytestmark = pytest.mark.gpu


def _both(dev, lp, ln, beam, r, lm=None, alpha=0.0, beta=0.0, window=0.0):
    B, T, V = lp.shape
    lp_d = torch.from_numpy(np.ascontiguousarray(lp)).to(dev)
    ln_d = torch.from_numpy(np.ascontiguousarray(ln, dtype=np.int32)).to(dev)
    lm_d = None if lm is None else torch.from_numpy(np.ascontiguousarray(lm)).to(dev)
    p = binding.FltopParams()
    p.beam, p.rel_threshold, p.beam_threshold = int(beam), float(r), float(window)
    if lm_d is not None:
        p.lm_table, p.lm_weight, p.insertion_bonus = lm_d.data_ptr(), alpha, beta
    res = []
    ws = binding.alloc_workspace(B, T, V, beam, dev)
    for static in (True, False):
        tok = torch.full((B, T), -1, dtype=torch.int32, device=dev)
        olen = torch.full((B,), -7, dtype=torch.int32, device=dev)
        sc = torch.full((B,), 123.0, dtype=torch.float32, device=dev)
        st = torch.zeros(binding.STATS_WORDS, dtype=torch.int64, device=dev)
        if static:
            rc = binding.decode_static_raw(lp_d, ln_d, p, tok, olen, sc, st)
        else:
            rc = binding.decode_raw(lp_d, ln_d, p, ws, ws.numel(), tok, olen, sc, st)
        assert rc == 0, binding.status_string(rc)
        torch.cuda.synchronize()
        res.append((tok.cpu().numpy(), olen.cpu().numpy(), sc.cpu().numpy(),
                    st.cpu().numpy()[:len(binding.STATS_FIELDS)]))
    (t0, l0, s0, st0), (t1, l1, s1, st1) = res
    np.testing.assert_array_equal(l0, l1)
    np.testing.assert_array_equal(t0, t1)
    assert s0.tobytes() == s1.tobytes()
    np.testing.assert_array_equal(st0, st1)
    return t0, l0, s0


def test_static_workspace_decode_matches_the_plain_entry_point(oracle_lib):
    assert torch.cuda.is_available(), "needs the MI355X"
    binding.load()
    dev = torch.device("cuda:0")
    # first call: cfg 2's shapes (27 MB of workspace), with a ragged tail
    w = synth.WORKLOADS["cfg2_batch64"]
    lp, ln = synth.make_emissions(w)
    ln = ln.copy()
    ln[-1] = 333
    assert binding.workspace_bytes(w.B, w.T, w.V, w.beam) <= binding.STATIC_SCRATCH_BYTES
    tok, olen, sc = _both(dev, lp, ln, w.beam, 0.01)
    want = oracle_lib.decode(lp[:4], ln[:4], w.beam, 0.01, n_threads=4)
    for b in range(4):
        assert tok[b, :olen[b]].tolist() == want[0][b]
        assert abs(float(sc[b]) - float(np.float32(want[1][b]))) <= 1e-4
    # second call, smaller in every dimension, other options: runs over the first call's leftovers
    lp2 = synth.random_emissions(77, 5, 61, 19, flat=1.5)
    ln2 = np.array([61, 60, 1, 0, 33], dtype=np.int32)
    lm2 = synth.make_bigram_lm(19, seed=5)
    tok2, olen2, sc2 = _both(dev, lp2, ln2, 12, 0.0, lm2, 0.5, 1.0, window=6.0)
    want2 = oracle_lib.decode(lp2, ln2, 12, 0.0, beam_threshold=6.0, lm_table=lm2, lm_weight=0.5,
                              insertion_bonus=1.0, n_threads=4)
    for b in range(5):
        assert tok2[b, :olen2[b]].tolist() == want2[0][b]
    # third call, large vocabulary (survivor records beyond the header) and back to a big shape
    lp3 = synth.random_emissions(78, 3, 40, 700, flat=1.0)
    ln3 = np.array([40, 17, 40], dtype=np.int32)
    _both(dev, lp3, ln3, 100, 0.0)
    # beyond the array: refused, nothing enqueued
    B, T, V, beam = 256, 1500, 32, 100
    assert binding.workspace_bytes(B, T, V, beam, max_records=0) > binding.STATIC_SCRATCH_BYTES
    lp_d = torch.empty((B, T, V), dtype=torch.float32, device=dev)
    ln_d = torch.zeros(B, dtype=torch.int32, device=dev)
    p = binding.FltopParams()
    p.beam, p.rel_threshold = beam, 0.01
    tok = torch.full((B, T), -1, dtype=torch.int32, device=dev)
    olen = torch.zeros(B, dtype=torch.int32, device=dev)
    sc = torch.zeros(B, dtype=torch.float32, device=dev)
    assert binding.decode_static_raw(lp_d, ln_d, p, tok, olen, sc, None) == -10
    assert "FLTOP_STATIC_SCRATCH_BYTES" in binding.status_string(-10)
    p.beam = 0  # bad arguments are still reported as what they are
    assert binding.decode_static_raw(lp_d, ln_d, p, tok, olen, sc, None) == -3
