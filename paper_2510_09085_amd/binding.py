"""Thin ctypes binding of the C ABI in include/fltop_ctc.h (argument marshalling only).

Every step of the decode runs in the HIP library; torch is used for device
memory and the current stream.  There is no fallback: if the shared library is
missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FLTOP_CTC_LIB") or os.path.join(_PKG, "libfltop_ctc.so")

MAX_BEAM = 1024
MAX_BEAM_STREAMING = 512      # the streaming entry points
MAX_VOCAB_WIDE_BEAM = 2048    # vocabulary limit of decodes with beam > 512
MAX_VOCAB = 4096

STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("fltop_ctc_workspace_bytes", "fltop_ctc_workspace_bytes_for", "fltop_ctc_decode",
           "fltop_ctc_decode_static",
           "fltop_ctc_prune", "fltop_ctc_search",
           "fltop_ctc_unpack_survivors", "fltop_ctc_token_ranks", "fltop_ctc_stream_state_bytes",
           "fltop_ctc_stream_begin", "fltop_ctc_stream_decode", "fltop_ctc_log_add",
           "fltop_status_string")


class FltopParams(ctypes.Structure):
    _fields_ = [
        ("beam", ctypes.c_int32),
        ("rel_threshold", ctypes.c_float),
        ("top_n", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("beam_threshold", ctypes.c_double),
        ("lm_table", ctypes.c_void_p),
        ("lm_weight", ctypes.c_float),
        ("insertion_bonus", ctypes.c_float),
        ("nbest_count", ctypes.c_void_p),
        ("nbest_tokens", ctypes.c_void_p),
        ("nbest_lengths", ctypes.c_void_p),
        ("nbest_pb", ctypes.c_void_p),
        ("nbest_pnb", ctypes.c_void_p),
        ("frame_beam", ctypes.c_void_p),
        ("out_token_frames", ctypes.c_void_p),
    ]


STATS_FIELDS = ("frames", "sum_survivors", "sum_candidates", "peak_candidates", "sum_beam",
                "select_passes", "exact_rankings", "overflow_drops", "survivor_records",
                "record_overflows")
# words to allocate for a fltop_stats block: the ten counters, and room for the 4 x 16 phase
# clocks that a profiling build of the library (-DFLTOP_PHASE_CLOCKS) appends
STATS_WORDS = len(STATS_FIELDS) + 64

_lib = None


class FltopError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load():
    """Load the HIP library built in-tree; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2510_09085_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    lib.fltop_ctc_workspace_bytes.restype = sz
    lib.fltop_ctc_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.fltop_ctc_workspace_bytes_for.restype = sz
    lib.fltop_ctc_workspace_bytes_for.argtypes = [i32, i32, i32, i32, ctypes.c_uint64]
    lib.fltop_ctc_decode.restype = ctypes.c_int
    lib.fltop_ctc_decode.argtypes = [vp, vp, i32, i32, i32, ctypes.POINTER(FltopParams), vp, sz,
                                     vp, vp, vp, vp, vp]
    lib.fltop_ctc_decode_static.restype = ctypes.c_int
    lib.fltop_ctc_decode_static.argtypes = [vp, vp, i32, i32, i32, ctypes.POINTER(FltopParams),
                                            vp, vp, vp, vp, vp]
    lib.fltop_ctc_search.restype = ctypes.c_int
    lib.fltop_ctc_search.argtypes = [vp, i32, i32, i32, ctypes.POINTER(FltopParams), vp, sz,
                                     vp, vp, vp, vp, vp]
    lib.fltop_ctc_prune.restype = ctypes.c_int
    lib.fltop_ctc_prune.argtypes = [vp, vp, i32, i32, i32, i32, f32, i32, vp, sz, vp]
    lib.fltop_ctc_token_ranks.restype = ctypes.c_int
    lib.fltop_ctc_token_ranks.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.fltop_ctc_unpack_survivors.restype = ctypes.c_int
    lib.fltop_ctc_unpack_survivors.argtypes = [vp, sz, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.fltop_ctc_stream_state_bytes.restype = sz
    lib.fltop_ctc_stream_state_bytes.argtypes = [i32, i32, i32]
    lib.fltop_ctc_stream_begin.restype = ctypes.c_int
    lib.fltop_ctc_stream_begin.argtypes = [vp, sz, i32, i32, i32, vp]
    lib.fltop_ctc_stream_decode.restype = ctypes.c_int
    lib.fltop_ctc_stream_decode.argtypes = [vp, vp, i32, i32, i32, ctypes.POINTER(FltopParams),
                                            vp, sz, vp, sz, i32, vp, vp, vp, vp, vp]
    lib.fltop_ctc_log_add.restype = ctypes.c_int
    lib.fltop_ctc_log_add.argtypes = [vp, vp, vp, ctypes.c_int64, vp]
    lib.fltop_status_string.restype = ctypes.c_char_p
    lib.fltop_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().fltop_status_string(int(status)).decode()


def workspace_bytes(B: int, T: int, V: int, beam: int, max_records: Optional[int] = None) -> int:
    """Bytes that hold any input of these shapes, or (max_records given) the fixed regions plus
    room for that many survivor records beyond the six per frame that sit in the headers."""
    if max_records is None:
        return int(load().fltop_ctc_workspace_bytes(B, T, V, beam))
    return int(load().fltop_ctc_workspace_bytes_for(B, T, V, beam, int(max_records)))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_inputs(logprobs: torch.Tensor, lengths: torch.Tensor):
    if not (logprobs.is_cuda and lengths.is_cuda):
        raise ValueError("logprobs and lengths must be device tensors")
    if logprobs.dtype != torch.float32 or lengths.dtype != torch.int32:
        raise ValueError("logprobs must be float32 and lengths int32")
    if logprobs.dim() != 3 or not logprobs.is_contiguous() or not lengths.is_contiguous():
        raise ValueError("logprobs must be a contiguous [B,T,V] tensor")
    if lengths.numel() != logprobs.shape[0]:
        raise ValueError("lengths must have B entries")


def alloc_workspace(B: int, T: int, V: int, beam: int, device,
                    max_records: Optional[int] = None) -> torch.Tensor:
    n = workspace_bytes(B, T, V, beam, max_records)
    if n == 0:
        raise FltopError(-2, "fltop_ctc_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def decode_raw(logprobs, lengths, params: FltopParams, workspace, workspace_nbytes, out_tokens,
               out_lengths, out_scores, stats, stream=None) -> int:
    """Direct call of fltop_ctc_decode; returns the status code (no checks, no allocation)."""
    B, T, V = logprobs.shape
    return int(load().fltop_ctc_decode(_ptr(logprobs), _ptr(lengths), B, T, V,
                                       ctypes.byref(params), _ptr(workspace), workspace_nbytes,
                                       _ptr(out_tokens), _ptr(out_lengths), _ptr(out_scores),
                                       _ptr(stats), _stream_handle(stream)))


def decode_static_raw(logprobs, lengths, params: FltopParams, out_tokens, out_lengths, out_scores,
                      stats, stream=None) -> int:
    """Direct call of fltop_ctc_decode_static (workspace inside the library); returns the status."""
    B, T, V = logprobs.shape
    return int(load().fltop_ctc_decode_static(_ptr(logprobs), _ptr(lengths), B, T, V,
                                              ctypes.byref(params), _ptr(out_tokens),
                                              _ptr(out_lengths), _ptr(out_scores), _ptr(stats),
                                              _stream_handle(stream)))


def search_raw(lengths, shape, params: FltopParams, workspace, workspace_nbytes, out_tokens,
               out_lengths, out_scores, stats, stream=None) -> int:
    """Direct call of fltop_ctc_search on a workspace fltop_ctc_prune has filled."""
    B, T, V = shape
    return int(load().fltop_ctc_search(_ptr(lengths), B, T, V, ctypes.byref(params),
                                       _ptr(workspace), workspace_nbytes, _ptr(out_tokens),
                                       _ptr(out_lengths), _ptr(out_scores), _ptr(stats),
                                       _stream_handle(stream)))


def prune_raw(logprobs, lengths, beam, rel_threshold, workspace, workspace_nbytes,
              stream=None, top_n: int = 0) -> int:
    """Direct call of fltop_ctc_prune; returns the status code."""
    B, T, V = logprobs.shape
    return int(load().fltop_ctc_prune(_ptr(logprobs), _ptr(lengths), B, T, V, int(beam),
                                      float(rel_threshold), int(top_n), _ptr(workspace),
                                      workspace_nbytes, _stream_handle(stream)))


def decode(logprobs: torch.Tensor, lengths: torch.Tensor, beam: int, rel_threshold: float, *,
           top_n: int = 0, beam_threshold: float = 0.0,
           lm_table: Optional[torch.Tensor] = None, lm_weight: float = 0.0,
           insertion_bonus: float = 0.0, workspace: Optional[torch.Tensor] = None,
           want_stats: bool = False, want_nbest: bool = False, want_traces: bool = False,
           stream=None) -> dict:
    """fltop_ctc_decode on device tensors.  Returns device tensors (no host sync):
    tokens [B,T] int32, lengths [B] int32, scores [B] fp32, and optionally stats
    (uint64, see STATS_FIELDS), the n-best export, and the statistics traces
    (frame_beam [B,T], token_frames [B,T], both int32 and -1 where nothing was written)."""
    _check_inputs(logprobs, lengths)
    B, T, V = logprobs.shape
    dev = logprobs.device
    if workspace is None:
        workspace = alloc_workspace(B, T, V, beam, dev)
    out = {
        "tokens": torch.full((B, T), -1, dtype=torch.int32, device=dev),
        "lengths": torch.zeros(B, dtype=torch.int32, device=dev),
        "scores": torch.zeros(B, dtype=torch.float32, device=dev),
    }
    p = FltopParams()
    p.beam = int(beam)
    p.rel_threshold = float(rel_threshold)
    p.top_n = int(top_n)
    p.beam_threshold = float(beam_threshold)
    p.lm_weight = float(lm_weight)
    p.insertion_bonus = float(insertion_bonus)
    if lm_table is not None:
        if not (lm_table.is_cuda and lm_table.dtype == torch.float32 and lm_table.is_contiguous()
                and tuple(lm_table.shape) == (V, V)):
            raise ValueError("lm_table must be a contiguous float32 [V,V] device tensor")
        p.lm_table = lm_table.data_ptr()
    if want_nbest:
        out["nbest_count"] = torch.zeros(B, dtype=torch.int32, device=dev)
        out["nbest_tokens"] = torch.full((B, beam, T), -1, dtype=torch.int32, device=dev)
        out["nbest_lengths"] = torch.zeros((B, beam), dtype=torch.int32, device=dev)
        out["nbest_pb"] = torch.zeros((B, beam), dtype=torch.float64, device=dev)
        out["nbest_pnb"] = torch.zeros((B, beam), dtype=torch.float64, device=dev)
        p.nbest_count = out["nbest_count"].data_ptr()
        p.nbest_tokens = out["nbest_tokens"].data_ptr()
        p.nbest_lengths = out["nbest_lengths"].data_ptr()
        p.nbest_pb = out["nbest_pb"].data_ptr()
        p.nbest_pnb = out["nbest_pnb"].data_ptr()
    if want_traces:
        out["frame_beam"] = torch.full((B, T), -1, dtype=torch.int32, device=dev)
        out["token_frames"] = torch.full((B, T), -1, dtype=torch.int32, device=dev)
        p.frame_beam = out["frame_beam"].data_ptr()
        p.out_token_frames = out["token_frames"].data_ptr()
    stats = None
    if want_stats:
        stats = torch.zeros(STATS_WORDS, dtype=torch.int64, device=dev)
        out["stats"] = stats
    rc = decode_raw(logprobs, lengths, p, workspace, workspace.numel(), out["tokens"],
                    out["lengths"], out["scores"], stats, stream)
    if rc != 0:
        raise FltopError(rc, "fltop_ctc_decode")
    out["workspace"] = workspace
    return out


def prune(logprobs: torch.Tensor, lengths: torch.Tensor, beam: int, rel_threshold: float, *,
          top_n: int = 0, workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """fltop_ctc_prune: survivor lists into the workspace (returned)."""
    _check_inputs(logprobs, lengths)
    B, T, V = logprobs.shape
    if workspace is None:
        workspace = alloc_workspace(B, T, V, beam, logprobs.device)
    rc = int(load().fltop_ctc_prune(_ptr(logprobs), _ptr(lengths), B, T, V, int(beam),
                                    float(rel_threshold), int(top_n), _ptr(workspace),
                                    workspace.numel(), _stream_handle(stream)))
    if rc != 0:
        raise FltopError(rc, "fltop_ctc_prune")
    return workspace


def unpack_survivors(workspace: torch.Tensor, lengths: torch.Tensor, B: int, T: int, V: int,
                     beam: int, stream=None):
    """fltop_ctc_unpack_survivors -> (counts [B*T], tokens [B*T,V], values [B*T,V], frame_max [B*T])."""
    dev = workspace.device
    counts = torch.zeros(B * T, dtype=torch.int32, device=dev)
    tokens = torch.full((B * T, V), -1, dtype=torch.int32, device=dev)
    values = torch.zeros((B * T, V), dtype=torch.float32, device=dev)
    fmax = torch.zeros(B * T, dtype=torch.float32, device=dev)
    rc = int(load().fltop_ctc_unpack_survivors(_ptr(workspace), workspace.numel(),
                                               _ptr(lengths), B, T, V,
                                               int(beam), _ptr(counts), _ptr(tokens),
                                               _ptr(values), _ptr(fmax), _stream_handle(stream)))
    if rc != 0:
        raise FltopError(rc, "fltop_ctc_unpack_survivors")
    return counts, tokens, values, fmax


def token_ranks(logprobs: torch.Tensor, tokens: torch.Tensor, token_frames: torch.Tensor,
                token_counts: torch.Tensor, stream=None):
    """fltop_ctc_token_ranks -> (ranks [B,T] int32 (-1 where unused), rank_count [V] int64,
    rank_lp_sum [V] float64)."""
    B, T, V = logprobs.shape
    dev = logprobs.device
    ranks = torch.full((B, T), -1, dtype=torch.int32, device=dev)
    count = torch.zeros(V, dtype=torch.int64, device=dev)
    lp_sum = torch.zeros(V, dtype=torch.float64, device=dev)
    rc = int(load().fltop_ctc_token_ranks(_ptr(logprobs), B, T, V, _ptr(tokens),
                                          _ptr(token_frames), _ptr(token_counts), _ptr(ranks),
                                          _ptr(count), _ptr(lp_sum), _stream_handle(stream)))
    if rc != 0:
        raise FltopError(rc, "fltop_ctc_token_ranks")
    return ranks, count, lp_sum


class Stream:
    """Chunked decoding of a batch of B streams of up to T_total frames each: owns the
    carried state, the output tensors and a workspace for chunks of up to T_chunk frames.
    feed() enqueues one chunk; the outputs then describe everything decoded so far."""

    def __init__(self, B: int, T_total: int, T_chunk: int, V: int, beam: int,
                 rel_threshold: float, device, *, top_n: int = 0, beam_threshold: float = 0.0,
                 lm_table: Optional[torch.Tensor] = None, lm_weight: float = 0.0,
                 insertion_bonus: float = 0.0, want_traces: bool = False):
        lib = load()
        self.B, self.T_total, self.T_chunk, self.V = B, T_total, T_chunk, V
        nbytes = int(lib.fltop_ctc_stream_state_bytes(B, T_total, beam))
        if nbytes == 0:
            raise FltopError(-2, "fltop_ctc_stream_state_bytes")
        self.state = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.workspace = alloc_workspace(B, T_chunk, V, beam, device)
        self.tokens = torch.full((B, T_total), -1, dtype=torch.int32, device=device)
        self.lengths = torch.zeros(B, dtype=torch.int32, device=device)
        self.scores = torch.zeros(B, dtype=torch.float32, device=device)
        self.stats = torch.zeros(STATS_WORDS, dtype=torch.int64, device=device)
        p = FltopParams()
        p.beam = int(beam)
        p.rel_threshold = float(rel_threshold)
        p.top_n = int(top_n)
        p.beam_threshold = float(beam_threshold)
        p.lm_weight = float(lm_weight)
        p.insertion_bonus = float(insertion_bonus)
        self._lm = lm_table
        if lm_table is not None:
            p.lm_table = lm_table.data_ptr()
        self.frame_beam = self.token_frames = None
        if want_traces:
            self.frame_beam = torch.full((B, T_total), -1, dtype=torch.int32, device=device)
            self.token_frames = torch.full((B, T_total), -1, dtype=torch.int32, device=device)
            p.frame_beam = self.frame_beam.data_ptr()
            p.out_token_frames = self.token_frames.data_ptr()
        self.params = p
        self.begin()

    def begin(self, stream=None):
        rc = int(load().fltop_ctc_stream_begin(_ptr(self.state), self.state.numel(), self.B,
                                               self.T_total, self.params.beam,
                                               _stream_handle(stream)))
        if rc != 0:
            raise FltopError(rc, "fltop_ctc_stream_begin")

    def feed(self, logprobs: torch.Tensor, lengths: torch.Tensor, stream=None):
        """logprobs [B,Tc,V] (Tc <= T_chunk), lengths [B]: valid frames of this chunk."""
        _check_inputs(logprobs, lengths)
        B, Tc, V = logprobs.shape
        if B != self.B or V != self.V or Tc > self.T_chunk:
            raise ValueError("chunk shape does not fit this stream")
        rc = int(load().fltop_ctc_stream_decode(
            _ptr(logprobs), _ptr(lengths), B, Tc, V, ctypes.byref(self.params),
            _ptr(self.workspace), self.workspace.numel(), _ptr(self.state), self.state.numel(),
            self.T_total, _ptr(self.tokens), _ptr(self.lengths), _ptr(self.scores),
            _ptr(self.stats), _stream_handle(stream)))
        if rc != 0:
            raise FltopError(rc, "fltop_ctc_stream_decode")


def log_add(a: torch.Tensor, b: torch.Tensor, stream=None) -> torch.Tensor:
    """fltop_ctc_log_add on two float64 device tensors of equal size."""
    if not (a.is_cuda and b.is_cuda and a.dtype == torch.float64 and b.dtype == torch.float64
            and a.is_contiguous() and b.is_contiguous() and a.numel() == b.numel()):
        raise ValueError("a and b must be contiguous float64 device tensors of one size")
    out = torch.empty_like(a)
    rc = int(load().fltop_ctc_log_add(_ptr(a), _ptr(b), _ptr(out), a.numel(),
                                      _stream_handle(stream)))
    if rc != 0:
        raise FltopError(rc, "fltop_ctc_log_add")
    return out


def stats_dict(stats: torch.Tensor) -> dict:
    vals = stats.cpu().tolist()
    out = dict(zip(STATS_FIELDS, vals))
    out.update({f"clk{i}": v for i, v in enumerate(vals[len(STATS_FIELDS):])})
    return out
