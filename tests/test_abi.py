"""Host-side checks of the C ABI: the library loads, exports what the header declares,
and rejects bad arguments before anything is enqueued (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2510_09085_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fltop_ctc.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2510_09085_amd import build
        build.build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fltop_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_header_constants_match_binding():
    text = open(HEADER).read()
    assert int(re.search(r"#define FLTOP_MAX_BEAM\s+(\d+)", text).group(1)) == binding.MAX_BEAM
    assert int(re.search(r"#define FLTOP_MAX_VOCAB\s+(\d+)", text).group(1)) == binding.MAX_VOCAB
    codes = dict(re.findall(r"#define (FLTOP_(?:OK|ERR_[A-Z_]+))\s+(-?\d+)", text))
    assert codes["FLTOP_OK"] == "0"
    assert sorted(int(v) for v in codes.values()) == list(range(-10, 1))
    assert int(re.search(r"#define FLTOP_STATIC_SCRATCH_BYTES\s+\((\d+)u << 20\)", text).group(1)) << 20 \
        == binding.STATIC_SCRATCH_BYTES


def test_status_strings(lib):
    seen = set()
    for code in range(-10, 1):
        s = binding.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 11
    assert binding.status_string(-99) == "unknown status"


def test_workspace_bytes(lib):
    assert binding.workspace_bytes(0, 10, 32, 8) == 0
    assert binding.workspace_bytes(1, 0, 32, 8) == 0
    assert binding.workspace_bytes(1, 10, 1, 8) == 0
    assert binding.workspace_bytes(1, 10, binding.MAX_VOCAB + 1, 8) == 0
    assert binding.workspace_bytes(1, 10, 32, 0) == 0
    assert binding.workspace_bytes(1, 10, 32, binding.MAX_BEAM + 1) == 0
    small = binding.workspace_bytes(1, 200, 32, 8)
    big = binding.workspace_bytes(64, 500, 32, 32)
    assert 0 < small < big
    assert small % 256 == 0
    # worst case: every frame keeps every token, six in its header, the others as 8-byte records;
    # a budget gets some slack on top (the record array is handed out in 64 slices, and each may
    # end on a stretch shorter than one wavefront's request: 8 frames x 26 records at V = 32)
    fixed = binding.workspace_bytes(64, 500, 32, 32, max_records=0)
    assert 0 < fixed < big and fixed % 256 == 0
    slack = 64 * 8 * (32 - 6)
    assert big - fixed == (64 * 500 * (32 - 6) + slack) * 8
    # a record budget in between; more than the shapes can need changes nothing
    mid = binding.workspace_bytes(64, 500, 32, 32, max_records=1000)
    assert fixed + (1000 + slack) * 8 <= mid <= fixed + (1000 + slack + 64) * 8 + 256
    assert binding.workspace_bytes(64, 500, 32, 32, max_records=10 ** 12) == big
    # six tokens or fewer never need a record
    assert binding.workspace_bytes(3, 50, 6, 4) == binding.workspace_bytes(3, 50, 6, 4, max_records=0)


def test_argument_errors_are_reported_before_any_launch(lib):
    """Fake non-null addresses are safe here: every call must fail in validation."""
    fake = ctypes.c_void_p(256 * 4096)
    p = binding.FltopParams()
    p.beam = 8
    p.rel_threshold = 0.01
    need = binding.workspace_bytes(2, 10, 32, 8)
    least = binding.workspace_bytes(2, 10, 32, 8, max_records=0)  # smaller ones are refused

    def call(lp=fake, ln=fake, B=2, T=10, V=32, params=p, ws=fake, nbytes=need, tok=fake,
             olen=fake, sc=fake):
        return lib.fltop_ctc_decode(lp, ln, B, T, V, ctypes.byref(params) if params else None,
                                    ws, nbytes, tok, olen, sc, None, None)

    assert call(lp=None) == -1
    assert call(ln=None) == -1
    assert call(params=None) == -1
    assert call(tok=None) == -1
    assert call(olen=None) == -1
    assert call(sc=None) == -1
    assert call(ws=None) == -1
    assert call(B=0) == -2
    assert call(T=0) == -2
    assert call(V=1) == -2
    assert call(V=binding.MAX_VOCAB + 1) == -6
    assert call(nbytes=least - 1) == -5
    assert call(ws=ctypes.c_void_p(256 * 4096 + 8)) == -8
    for bad_beam in (0, -3, binding.MAX_BEAM + 1):
        q = binding.FltopParams()
        q.beam = bad_beam
        q.rel_threshold = 0.01
        assert call(params=q) == -3
    wide = binding.FltopParams()  # a beam beyond 512 entries takes vocabularies up to 2048 only
    wide.beam = 600
    wide.rel_threshold = 0.01
    assert call(params=wide, V=binding.MAX_VOCAB_WIDE_BEAM + 1,
                nbytes=1 << 40) == -3
    assert binding.workspace_bytes(2, 10, binding.MAX_VOCAB_WIDE_BEAM + 1, 600) == 0
    assert binding.workspace_bytes(2, 10, binding.MAX_VOCAB_WIDE_BEAM, 600) > \
        binding.workspace_bytes(2, 10, binding.MAX_VOCAB_WIDE_BEAM, 512)
    for bad_r in (-0.1, 1.5, float("nan")):
        q = binding.FltopParams()
        q.beam = 8
        q.rel_threshold = bad_r
        assert call(params=q) == -4
    q = binding.FltopParams()
    q.beam = 8
    q.rel_threshold = 0.5
    q.nbest_count = 4096  # some but not all n-best pointers
    assert call(params=q) == -1
    # the stand-alone prune stage validates the same way
    assert lib.fltop_ctc_prune(None, fake, 2, 10, 32, 8, 0.01, 0, fake, need, None) == -1
    assert lib.fltop_ctc_prune(fake, fake, 2, 10, 32, 8, 2.0, 0, fake, need, None) == -4
    assert lib.fltop_ctc_prune(fake, fake, 2, 10, 32, 8, 0.01, 0, fake, 16, None) == -5
    assert lib.fltop_ctc_prune(fake, fake, 2, 10, 32, 8, 0.01, -1, fake, need, None) == -9
    for field, bad in (("top_n", -2), ("beam_threshold", float("nan"))):
        q = binding.FltopParams()
        q.beam = 8
        q.rel_threshold = 0.5
        setattr(q, field, bad)
        assert call(params=q) == -9
    # the entry point with the workspace inside the library: shapes beyond it, and a missing
    # params block, are refused before anything touches the GPU
    big = binding.FltopParams()
    big.beam = 100
    big.rel_threshold = 0.01
    assert binding.workspace_bytes(256, 1500, 32, 100, max_records=0) > binding.STATIC_SCRATCH_BYTES
    assert lib.fltop_ctc_decode_static(fake, fake, 256, 1500, 32, ctypes.byref(big), fake, fake,
                                       fake, None, None) == -10
    assert lib.fltop_ctc_decode_static(fake, fake, 2, 10, 32, None, fake, fake, fake, None,
                                       None) == -1
    assert lib.fltop_ctc_token_ranks(None, 2, 10, 32, fake, fake, fake, None, None, None,
                                     None) == -1
    assert lib.fltop_ctc_token_ranks(fake, 2, 10, 1, fake, fake, fake, None, None, None,
                                     None) == -2
    assert lib.fltop_ctc_unpack_survivors(fake, need, fake, 2, 10, 32, 8, None, fake, fake, None,
                                          None) == -1
    assert lib.fltop_ctc_unpack_survivors(fake, need, None, 2, 10, 32, 8, fake, fake, fake, None,
                                          None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()


def test_stream_entry_points_validate_before_any_launch(lib):
    fake = ctypes.c_void_p(256 * 4096)
    p = binding.FltopParams()
    p.beam = 8
    p.rel_threshold = 0.01
    B, Tc, Ttot, V = 2, 10, 100, 32
    ws_need = binding.workspace_bytes(B, Tc, V, 8)
    st_need = lib.fltop_ctc_stream_state_bytes(B, Ttot, 8)
    assert st_need > 0 and st_need % 256 == 0
    # the state holds the trie for T_total frames: 16 bytes per (frame, beam slot)
    assert st_need >= B * Ttot * 8 * 16
    assert lib.fltop_ctc_stream_state_bytes(B, Ttot, 8) < lib.fltop_ctc_stream_state_bytes(B, 2 * Ttot, 8)
    assert lib.fltop_ctc_stream_state_bytes(0, Ttot, 8) == 0
    assert lib.fltop_ctc_stream_state_bytes(B, 0, 8) == 0
    assert lib.fltop_ctc_stream_state_bytes(B, Ttot, binding.MAX_BEAM_STREAMING + 1) == 0

    assert lib.fltop_ctc_stream_begin(None, st_need, B, Ttot, 8, None) == -1
    assert lib.fltop_ctc_stream_begin(fake, st_need - 1, B, Ttot, 8, None) == -5
    assert lib.fltop_ctc_stream_begin(ctypes.c_void_p(256 * 4096 + 16), st_need, B, Ttot, 8, None) == -8
    assert lib.fltop_ctc_stream_begin(fake, st_need, B, Ttot, 0, None) == -3

    def call(lp=fake, ln=fake, Tchunk=Tc, params=p, ws=fake, ws_bytes=ws_need, st=fake,
             st_bytes=st_need, total=Ttot, tok=fake):
        return lib.fltop_ctc_stream_decode(lp, ln, B, Tchunk, V,
                                           ctypes.byref(params) if params else None, ws, ws_bytes,
                                           st, st_bytes, total, tok, fake, fake, None, None)

    assert call(lp=None) == -1
    assert call(ln=None) == -1
    assert call(params=None) == -1
    assert call(tok=None) == -1
    assert call(ws=None) == -1
    assert call(st=None) == -1
    assert call(Tchunk=0) == -2
    assert call(total=Tc - 1) == -2          # a chunk longer than the whole stream
    assert call(ws_bytes=binding.workspace_bytes(B, Tc, V, 8, max_records=0) - 1) == -5
    assert call(st_bytes=st_need - 1) == -5
    assert call(st=ctypes.c_void_p(256 * 4096 + 64)) == -8
    q = binding.FltopParams()
    q.beam = 8
    q.rel_threshold = 1.5
    assert call(params=q) == -4
    q.rel_threshold = 0.5
    q.top_n = -1
    assert call(params=q) == -9


def test_header_is_plain_c_and_the_struct_layout_matches_the_binding(tmp_path):
    """The boundary is a C ABI: the header must compile as C99, and the ctypes mirror of
    fltop_params / fltop_stats must have the C compiler's sizes and field offsets."""
    import subprocess
    fields = [name for name, _ in binding.FltopParams._fields_]
    prog = ['#include <stddef.h>', '#include <stdio.h>', '#include "fltop_ctc.h"',
            'int main(void) {', '  printf("%zu %zu\\n", sizeof(fltop_params), sizeof(fltop_stats));']
    for name in fields:
        prog.append(f'  printf("{name} %zu\\n", offsetof(fltop_params, {name}));')
    prog += ['  return 0;', '}']
    src = tmp_path / "abi_probe.c"
    src.write_text("\n".join(prog) + "\n")
    exe = tmp_path / "abi_probe"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I",
                    os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split("\n")
    size_params, size_stats = (int(x) for x in out[0].split())
    assert size_params == ctypes.sizeof(binding.FltopParams)
    assert size_stats == 8 * len(binding.STATS_FIELDS)
    for line in out[1:]:
        if line:
            name, off = line.split()
            assert getattr(binding.FltopParams, name).offset == int(off), name
