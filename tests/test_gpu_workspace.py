"""The workspace shrinks with the pruning (the method's memory saving, paper Sec. 4.4): a frame's
first six survivors sit in its header, every further one takes an 8-byte record, and a caller
may size the record array for what the threshold leaves (fltop_ctc_workspace_bytes_for).  With
exactly the records a batch needs the results are those of the worst-case workspace; with
fewer, the utterances that meet a frame whose records did not fit are reported (length -1,
score NaN, counted), nothing is written out of bounds, and all others decode as before."""
import numpy as np
import pytest
import torch

from paper_2510_09085_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load()
    return torch.device("cuda:0")


def run(dev, lp_d, ln_d, beam, r, max_records=None, raw_records=None, **kw):
    """max_records: a workspace sized by the library for that budget; raw_records: the fixed
    regions plus exactly that many 8-byte places (less than the library would add for a budget)."""
    B, T, V = lp_d.shape
    if raw_records is None:
        ws = binding.alloc_workspace(B, T, V, beam, dev, max_records=max_records)
    else:
        fixed = binding.workspace_bytes(B, T, V, beam, max_records=0)
        ws = torch.empty(fixed + 8 * raw_records, dtype=torch.uint8, device=dev)
    ws.fill_(0xA5)  # whatever the memory held before
    guard = torch.full((4096,), 0x5A, dtype=torch.uint8, device=dev)  # allocated right behind
    out = binding.decode(lp_d, ln_d, beam, r, workspace=ws, want_stats=True, **kw)
    torch.cuda.synchronize()
    assert bool((guard == 0x5A).all().item())
    lens = out["lengths"].cpu().numpy()
    toks = out["tokens"].cpu().numpy()
    return {"lengths": lens, "scores": out["scores"].cpu().numpy(),
            "tokens": [toks[b, :max(0, lens[b])].tolist() for b in range(B)],
            "stats": binding.stats_dict(out["stats"]), "bytes": ws.numel()}


@pytest.mark.parametrize("case", ["subword_pruned", "chars_loose", "chars_unpruned"])
def test_workspace_sized_for_the_survivors(dev, oracle_lib, case):
    if case == "subword_pruned":
        w = synth.WORKLOADS["cfg4_subword1024"]
        lp, ln = synth.make_emissions(w, utterances=range(12))
        beam, r = 16, 0.01
    elif case == "chars_loose":
        w = synth.WORKLOADS["cfg3_varlen256"]
        lp, ln = synth.make_emissions(w, utterances=range(10))
        lp, ln = np.ascontiguousarray(lp[:, :400]), np.minimum(ln, 400).astype(np.int32)
        beam, r = 24, 1e-4
    else:
        lp = synth.random_emissions(31, 6, 90, 40, flat=1.0)
        ln = np.array([90, 90, 41, 0, 90, 7], dtype=np.int32)
        beam, r = 12, 0.0
    B, T, V = lp.shape
    counts = np.concatenate([oracle_lib.survivors(lp[b, :ln[b]], r)[0] for b in range(B)])
    needed = int(np.maximum(counts - 6, 0).sum())
    lp_d, ln_d = torch.from_numpy(lp).to(dev), torch.from_numpy(ln).to(dev)

    full = run(dev, lp_d, ln_d, beam, r)
    assert full["stats"]["survivor_records"] == needed
    assert full["stats"]["record_overflows"] == 0
    want = oracle_lib.decode(lp, ln, beam, r, n_threads=8)
    assert full["tokens"] == want[0]

    exact = run(dev, lp_d, ln_d, beam, r, max_records=needed)
    assert exact["bytes"] <= full["bytes"] and (needed == B * T * (V - 6) or exact["bytes"] < full["bytes"])
    assert exact["tokens"] == full["tokens"]
    assert exact["scores"].tobytes() == full["scores"].tobytes()
    assert exact["stats"] == full["stats"]

    # survivor lists as the prune stage left them in the small workspace
    ws = binding.alloc_workspace(B, T, V, beam, dev, max_records=needed)
    binding.prune(lp_d, ln_d, beam, r, workspace=ws)
    got_counts, got_tokens, got_values, _ = [x.cpu().numpy() for x in
                                             binding.unpack_survivors(ws, ln_d, B, T, V, beam)]
    at = 0
    for b in range(B):
        oc, ot, _ = oracle_lib.survivors(lp[b, :ln[b]], r) if ln[b] else (np.zeros(0, int), None, None)
        for f in range(ln[b]):
            k = oc[f]
            assert got_counts[b * T + f] == k
            np.testing.assert_array_equal(got_tokens[b * T + f, :k], ot[f, :k])
            np.testing.assert_array_equal(got_values[b * T + f, :k].view(np.uint32),
                                          lp[b, f, ot[f, :k]].view(np.uint32))
        at += ln[b]

    if needed == 0:
        return
    # too few records: some utterances are reported, the rest decode as before
    for budget in (needed // 2, 0):
        short = run(dev, lp_d, ln_d, beam, r, raw_records=budget)
        lost = short["lengths"] == -1
        assert lost.any()
        assert short["stats"]["record_overflows"] == int(lost.sum())
        assert short["stats"]["survivor_records"] == needed  # what to ask for next time
        assert np.isnan(short["scores"][lost]).all()
        for b in range(B):
            if not lost[b]:
                assert short["tokens"][b] == full["tokens"][b]
                assert short["scores"][b].tobytes() == full["scores"][b].tobytes()
        if budget == 0:  # exactly the utterances with a frame of more than six survivors
            per_utt = np.array([counts[sum(ln[:b]):sum(ln[:b + 1])].max(initial=0) for b in range(B)])
            np.testing.assert_array_equal(lost, per_utt > 6)


def test_named_workloads_need_a_fraction_of_the_worst_case(dev):
    """cfg 4 at r = 0.01: the worst-case record array is 427 MB, the survivors need a few MB."""
    w = synth.WORKLOADS["cfg4_subword1024"]
    lp, ln = synth.make_emissions(w, utterances=range(16))
    lp_d, ln_d = torch.from_numpy(lp).to(dev), torch.from_numpy(ln).to(dev)
    st = run(dev, lp_d, ln_d, w.beam, 0.01)["stats"]
    worst = 16 * w.T * (w.V - 6)
    assert 0 < st["survivor_records"] < worst // 50
    st0 = run(dev, lp_d, ln_d, w.beam, 0.0)["stats"]
    assert st0["survivor_records"] == worst
