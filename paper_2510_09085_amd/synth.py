"""Seeded synthetic inputs for the FLToP CTC decoder: emissions, lengths, bigram LM.

This module only *draws inputs*.  It contains none of the decoder's arithmetic
(no thresholding, no beam search, no hashing) and imports neither the HIP
binding nor the CPU oracle; both of those consume the arrays produced here.

The emissions stand in for what an acoustic encoder feeds a CTC decoder in the
paper's experiments (Sec. 4: a 32-token character vocabulary, one of them
playing the blank role, frame-level posteriors that are sharply peaked on most
frames).  Everything is drawn in fp64 with numpy's PCG64 ``default_rng`` and
cast to fp32 once at the end, so the bytes depend only on (seed, utterance
index, shape, recipe parameters).

Recipe for one utterance (T frames, V tokens, index 0 = blank):
  1. transcript: 60 tokens uniform on 1..V-1.
  2. base logits: N(0,1) for every (frame, token); with ``zipf_s > 0`` the
     non-blank token v additionally gets ``-zipf_s * ln(v)`` (a Zipf prior).
  3. primary boost U(6,12) on one token per frame: blank with probability
     ``p_blank`` (0.65), otherwise the next unread transcript token (the read
     pointer wraps modulo 60).
  4. on a fraction ``hard_rate`` of frames a second boost U(4,8) on one token
     drawn uniformly among the V-1 tokens other than the primary one.
  5. log-softmax over V.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Sequence

import numpy as np

TRANSCRIPT_LEN = 60
LM_SEED = 7777
FRAMES_PER_SECOND = 50  # 20 ms encoder stride, used only to report audio-seconds


@dataclasses.dataclass(frozen=True)
class Workload:
    """One named decoding workload (shapes + decoder settings + generator knobs)."""

    name: str
    B: int
    T: int
    V: int
    beam: int
    rel_thresholds: Sequence[float]
    seed: int
    hard_rate: float = 0.10
    p_blank: float = 0.65
    zipf_s: float = 0.0
    variable_lengths: Optional[Sequence[int]] = None  # (lo, hi) inclusive
    use_lm: bool = False
    lm_weight: float = 0.0
    insertion_bonus: float = 0.0


WORKLOADS = {
    "cfg1_single": Workload("cfg1_single", B=1, T=200, V=32, beam=8,
                            rel_thresholds=(0.01, 0.0), seed=1001),
    "cfg2_batch64": Workload("cfg2_batch64", B=64, T=500, V=32, beam=32,
                             rel_thresholds=(0.1, 0.01, 0.001, 0.0), seed=1002),
    "cfg3_varlen256": Workload("cfg3_varlen256", B=256, T=1500, V=32, beam=100,
                               rel_thresholds=(0.01,), seed=1003, hard_rate=0.25,
                               variable_lengths=(250, 1500)),
    "cfg4_subword1024": Workload("cfg4_subword1024", B=128, T=400, V=1024, beam=64,
                                 rel_thresholds=(0.01, 0.0), seed=1004, zipf_s=1.1),
    "cfg5_bigram_lm": Workload("cfg5_bigram_lm", B=128, T=500, V=32, beam=64,
                               rel_thresholds=(0.01, 0.0), seed=1005, use_lm=True,
                               lm_weight=0.5, insertion_bonus=1.0),
    # beyond the five base workloads: a sub-word vocabulary with a dense bigram table that no
    # longer fits in LDS (4 MB), so LM terms are gathered from global memory
    "ext_subword1024_lm": Workload("ext_subword1024_lm", B=128, T=400, V=1024, beam=64,
                                   rel_thresholds=(0.01,), seed=1006, zipf_s=1.1, use_lm=True,
                                   lm_weight=0.5, insertion_bonus=1.0),
}


def _log_softmax64(x: np.ndarray) -> np.ndarray:
    mx = x.max(axis=-1, keepdims=True)
    z = x - mx
    return z - np.log(np.exp(z).sum(axis=-1, keepdims=True))


def utterance_emissions(seed: int, b: int, T: int, V: int, *, hard_rate: float = 0.10,
                        p_blank: float = 0.65, zipf_s: float = 0.0) -> np.ndarray:
    """fp32 [T, V] log-softmax emissions of utterance ``b`` under ``seed``."""
    if V < 2:
        raise ValueError("need a blank and at least one token")
    rng = np.random.default_rng([int(seed), int(b)])
    transcript = rng.integers(1, V, size=TRANSCRIPT_LEN)
    logits = rng.standard_normal((T, V))
    if zipf_s > 0.0:
        logits[:, 1:] -= zipf_s * np.log(np.arange(1, V, dtype=np.float64))
    is_blank = rng.random(T) < p_blank
    read_ptr = np.cumsum(~is_blank) - 1
    primary = np.where(is_blank, 0, transcript[read_ptr % TRANSCRIPT_LEN])
    rows = np.arange(T)
    logits[rows, primary] += rng.uniform(6.0, 12.0, size=T)
    hard = rng.random(T) < hard_rate
    other = rng.integers(0, V - 1, size=T)
    other = other + (other >= primary)  # uniform over the V-1 tokens != primary
    second = rng.uniform(4.0, 8.0, size=T)
    logits[rows[hard], other[hard]] += second[hard]
    return _log_softmax64(logits).astype(np.float32)


def make_lengths(w: Workload) -> np.ndarray:
    """int32 [B] valid frame counts."""
    if w.variable_lengths is None:
        return np.full(w.B, w.T, dtype=np.int32)
    lo, hi = w.variable_lengths
    rng = np.random.default_rng([int(w.seed), 0x1E46])
    return rng.integers(lo, hi + 1, size=w.B).astype(np.int32)


def make_emissions(w: Workload, *, pad_value: float = np.nan,
                   utterances: Optional[Sequence[int]] = None):
    """(logprobs fp32 [n, T, V], lengths int32 [n]) for the workload.

    ``utterances`` selects a subset of utterance indices (same bytes those rows
    have in the full batch).  Frames at or beyond an utterance's length are
    filled with ``pad_value`` (NaN by default: a decoder that reads them shows).
    """
    all_len = make_lengths(w)
    idx = list(range(w.B)) if utterances is None else [int(u) for u in utterances]
    lp = np.empty((len(idx), w.T, w.V), dtype=np.float32)
    for row, b in enumerate(idx):
        lp[row] = utterance_emissions(w.seed, b, w.T, w.V, hard_rate=w.hard_rate,
                                      p_blank=w.p_blank, zipf_s=w.zipf_s)
        lp[row, all_len[b]:, :] = pad_value
    return lp, all_len[idx].copy()


def make_bigram_lm(V: int, seed: int = LM_SEED, concentration: float = 0.3) -> np.ndarray:
    """fp32 [V, V] log-probabilities; row a is a Dirichlet(concentration) draw.

    Probabilities are floored at 1e-30 before the log so the table is finite.
    """
    rng = np.random.default_rng(int(seed))
    p = rng.dirichlet(np.full(V, concentration, dtype=np.float64), size=V)
    return np.log(np.maximum(p, 1e-30)).astype(np.float32)


def random_emissions(seed: int, B: int, T: int, V: int, *, flat: float = 1.0) -> np.ndarray:
    """Unstructured fp32 [B, T, V] log-softmax rows (logits ~ flat * N(0,1)); test helper."""
    rng = np.random.default_rng(int(seed))
    return _log_softmax64(flat * rng.standard_normal((B, T, V))).astype(np.float32)
