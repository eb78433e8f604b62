"""ctypes access to the CPU oracle (test infrastructure; never a product path).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It shares nothing with the HIP decoder or its Python binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# FLTOP_ORACLE_LIB names another build of the oracle (the mutation test points it at oracles
# with a planted mistake to show that the pins notice)
LIB_PATH = os.environ.get("FLTOP_ORACLE_LIB") or os.path.join(_HERE, "libfltop_oracle.so")
FLTOP = 0
TEXTBOOK = 1


class OracleStats(ctypes.Structure):
    _fields_ = [
        ("frames", ctypes.c_int64),
        ("sum_survivors", ctypes.c_int64),
        ("sum_candidates", ctypes.c_int64),
        ("peak_candidates", ctypes.c_int64),
        ("sum_beam", ctypes.c_int64),
        ("max_addends", ctypes.c_int64),
        ("hash_collisions", ctypes.c_int64),
        ("min_cut_margin", ctypes.c_double),
        ("min_decision_margin", ctypes.c_double),
    ]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


def build(sanitize: bool = False) -> str:
    """Compile the oracle with g++ (always recompiles)."""
    out = LIB_PATH if not sanitize else os.path.join(_HERE, "libfltop_oracle_asan.so")
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
           "-ffp-contract=off", os.path.join(_HERE, "fltop_oracle.cpp"), "-o", out]
    if sanitize:
        cmd[1:1] = ["-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"]
    subprocess.run(cmd, check=True)
    return out


def build_sanitize_driver(out: str) -> str:
    """Compile sanitize_driver.cpp + the oracle into one executable under ASan and UBSan
    (runtime linked statically, so it runs whatever else the loader preloads)."""
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-pthread", "-Wall", "-Wextra", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
           "-fno-omit-frame-pointer", os.path.join(_HERE, "sanitize_driver.cpp"),
           os.path.join(_HERE, "fltop_oracle.cpp"), "-o", out]
    subprocess.run(cmd, check=True)
    return out


_lib = None


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        build()
    lib = ctypes.CDLL(LIB_PATH)
    f32p = ctypes.POINTER(ctypes.c_float)
    i32p = ctypes.POINTER(ctypes.c_int32)
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.fltop_oracle_prefix_hash.restype = ctypes.c_uint64
    lib.fltop_oracle_prefix_hash.argtypes = [i32p, ctypes.c_int32]
    lib.fltop_oracle_survivors.restype = ctypes.c_int
    lib.fltop_oracle_survivors.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float,
                                           ctypes.c_int32, i32p, i32p, f32p]
    lib.fltop_oracle_decode.restype = ctypes.c_int
    lib.fltop_oracle_decode.argtypes = [f32p, i32p, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                        ctypes.c_int32, ctypes.c_double, f32p,
                                        ctypes.c_float, ctypes.c_float, ctypes.c_int32, i32p,
                                        i32p, f64p, i32p, i32p, f64p, ctypes.POINTER(OracleStats),
                                        ctypes.c_int32]
    lib.fltop_oracle_decode_beam.restype = ctypes.c_int
    lib.fltop_oracle_token_ranks.restype = ctypes.c_int
    lib.fltop_oracle_token_ranks.argtypes = [f32p, ctypes.c_int32, ctypes.c_int32, i32p, i32p,
                                             ctypes.c_int32, i32p]
    lib.fltop_oracle_decode_beam.argtypes = [f32p, ctypes.c_int32, ctypes.c_int32,
                                             ctypes.c_int32, ctypes.c_float, ctypes.c_int32,
                                             ctypes.c_double, f32p,
                                             ctypes.c_float, ctypes.c_float, ctypes.c_int32,
                                             ctypes.c_int32, i32p, i32p, f64p, f64p]
    _lib = lib
    return lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def prefix_hash(tokens) -> int:
    arr, ptr = _i32(np.asarray(tokens, dtype=np.int32).reshape(-1))
    return int(load().fltop_oracle_prefix_hash(ptr, arr.size))


def survivors(logprobs: np.ndarray, rel_threshold: float, top_n: int = 0):
    """Per-frame survivor sets of [..., V] emissions -> (counts[F], tokens[F,V], frame_max[F])."""
    lp, lp_p = _f32(logprobs)
    V = lp.shape[-1]
    F = lp.size // V
    counts = np.zeros(F, dtype=np.int32)
    tokens = np.full((F, V), -1, dtype=np.int32)
    fmax = np.zeros(F, dtype=np.float32)
    rc = load().fltop_oracle_survivors(
        lp_p, F, V, float(rel_threshold), int(top_n),
        counts.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        tokens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        fmax.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError("fltop_oracle_survivors: bad arguments")
    return counts, tokens, fmax


def decode(logprobs: np.ndarray, lengths: np.ndarray, beam: int, rel_threshold: float, *,
           top_n: int = 0, beam_threshold: float = 0.0,
           lm_table: Optional[np.ndarray] = None, lm_weight: float = 0.0,
           insertion_bonus: float = 0.0, variant: int = FLTOP, n_threads: int = 1,
           traces: bool = False):
    """Best prefix per utterance -> (list of token lists, scores fp64 [B], stats dict).

    With traces=True the stats dict also holds "token_frames" (list per utterance: frame at
    which each output token's prefix entered the beam) and "frame_beam" ([B,T] int32, beam
    entries kept after each frame, -1 beyond the utterance's length)."""
    lp, lp_p = _f32(logprobs)
    B, T, V = lp.shape
    ln, ln_p = _i32(lengths)
    if lm_table is not None:
        lm, lm_p = _f32(lm_table)
        assert lm.shape == (V, V)
    else:
        lm, lm_p = None, None
    out_tok = np.full((B, max(T, 1)), -1, dtype=np.int32)
    out_len = np.zeros(B, dtype=np.int32)
    out_sc = np.zeros(B, dtype=np.float64)
    st = OracleStats()
    i32p = ctypes.POINTER(ctypes.c_int32)
    tok_frames = np.full((B, max(T, 1)), -1, dtype=np.int32) if traces else None
    frame_beam = np.full((B, max(T, 1)), -1, dtype=np.int32) if traces else None
    margins = np.full(B, np.inf, dtype=np.float64)
    rc = load().fltop_oracle_decode(
        lp_p, ln_p, B, T, V, int(beam), float(rel_threshold), int(top_n), float(beam_threshold),
        lm_p, float(lm_weight), float(insertion_bonus), int(variant),
        out_tok.ctypes.data_as(i32p), out_len.ctypes.data_as(i32p),
        out_sc.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        tok_frames.ctypes.data_as(i32p) if traces else None,
        frame_beam.ctypes.data_as(i32p) if traces else None,
        margins.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), ctypes.byref(st),
        int(n_threads))
    if rc != 0:
        raise ValueError("fltop_oracle_decode: bad arguments")
    toks = [out_tok[b, :out_len[b]].tolist() for b in range(B)]
    stats = st.as_dict()
    stats["margins"] = margins.tolist()  # per utterance: smallest score gap that decided anything
    if traces:
        stats["token_frames"] = [tok_frames[b, :out_len[b]].tolist() for b in range(B)]
        stats["frame_beam"] = frame_beam[:, :T]
    return toks, out_sc, stats


def token_ranks(logprobs: np.ndarray, tokens, frames) -> np.ndarray:
    """Position of tokens[i] in the descending sort of frame frames[i] of one [T,V] utterance."""
    lp, lp_p = _f32(logprobs)
    T, V = lp.shape
    tk, tk_p = _i32(np.asarray(tokens, dtype=np.int32).reshape(-1))
    fr, fr_p = _i32(np.asarray(frames, dtype=np.int32).reshape(-1))
    assert tk.size == fr.size
    ranks = np.zeros(tk.size, dtype=np.int32)
    rc = load().fltop_oracle_token_ranks(lp_p, T, V, tk_p, fr_p, tk.size,
                                         ranks.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != 0:
        raise ValueError("fltop_oracle_token_ranks: bad arguments")
    return ranks


def decode_beam(logprobs: np.ndarray, beam: int, rel_threshold: float, *,
                top_n: int = 0, beam_threshold: float = 0.0,
                lm_table: Optional[np.ndarray] = None, lm_weight: float = 0.0,
                insertion_bonus: float = 0.0, variant: int = FLTOP, max_entries: int = 0):
    """Whole final beam of one [T,V] utterance -> list of (tokens tuple, p_b, p_nb) in rank order."""
    lp, lp_p = _f32(logprobs)
    T, V = lp.shape
    if lm_table is not None:
        lm, lm_p = _f32(lm_table)
        assert lm.shape == (V, V)
    else:
        lm, lm_p = None, None
    cap = int(max_entries) if max_entries > 0 else int(beam)
    toks = np.full((cap, max(T, 1)), -1, dtype=np.int32)
    lens = np.zeros(cap, dtype=np.int32)
    pb = np.zeros(cap, dtype=np.float64)
    pnb = np.zeros(cap, dtype=np.float64)
    n = load().fltop_oracle_decode_beam(
        lp_p, T, V, int(beam), float(rel_threshold), int(top_n), float(beam_threshold), lm_p,
        float(lm_weight), float(insertion_bonus), int(variant), cap,
        toks.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        pb.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        pnb.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if n < 0:
        raise ValueError("fltop_oracle_decode_beam: bad arguments")
    return [(tuple(toks[i, :lens[i]].tolist()), float(pb[i]), float(pnb[i])) for i in range(n)]
