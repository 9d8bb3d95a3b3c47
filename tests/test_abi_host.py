"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol include/dart.h declares, mirrors the descriptor layout, sizes the
workspace and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re
import subprocess
import tempfile

import pytest

import paper_2502_11494_amd as D
from paper_2502_11494_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dart.h")


def declared_functions():
    text = open(HEADER).read()
    return re.findall(r"DART_API\s+[\w\s\*]+?\b(dart_\w+)\s*\(", text)


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS) and len(names) == len(binding.EXPORTS)
    L = binding.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_descriptor_layout_matches_the_header():
    src = '#include <stdio.h>\n#include <stddef.h>\n#include "dart.h"\nint main(){printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu", sizeof(dart_desc), offsetof(dart_desc, cu_seqlens), offsetof(dart_desc, ld), offsetof(dart_desc, K), offsetof(dart_desc, score_mode), offsetof(dart_desc, P_ext), offsetof(dart_desc, ext_ld), offsetof(dart_desc, ext_pivots), offsetof(dart_desc, span_start), offsetof(dart_desc, X_rows), offsetof(dart_desc, seed), sizeof(dart_row_tensor));return 0;}\n'
    with tempfile.TemporaryDirectory() as td:
        c = os.path.join(td, "t.c")
        open(c, "w").write(src)
        exe = os.path.join(td, "t")
        subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), c, "-o", exe],
                       check=True)
        out = subprocess.run([exe], capture_output=True, text=True, check=True).stdout.split()
    T = D.DartDesc
    assert list(map(int, out)) == [C.sizeof(T), T.cu_seqlens.offset, T.ld.offset, T.K.offset,
                                   T.score_mode.offset, T.P_ext.offset, T.ext_ld.offset,
                                   T.ext_pivots.offset, T.span_start.offset, T.X_rows.offset,
                                   T.seed.offset, C.sizeof(binding.DartRowTensor)]


def test_workspace_grows_with_the_problem():
    small = D.dart_workspace_bytes(D.make_desc(1, 4096, 8, D.DART_F32, N=576, K=64))
    big = D.dart_workspace_bytes(D.make_desc(8, 4096, 16, D.DART_BF16, N=2880, K=320))
    assert 0 < small < big
    assert small % 256 == 0 and big % 256 == 0
    assert D.dart_workspace_bytes(D.make_desc(0, 4096, 8, D.DART_F32, N=576, K=64)) > 0


BAD = [
    (dict(B=1, D=4096, P=0, dtype=D.DART_BF16, N=576, K=64), D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=65, dtype=D.DART_BF16, N=576, K=70), D.DART_ERR_SHAPE),
    (dict(B=-1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64), D.DART_ERR_SHAPE),
    (dict(B=1, D=0, P=8, dtype=D.DART_BF16, N=576, K=64), D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=16385, K=64), D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, ld=4000), D.DART_ERR_SHAPE),
    (dict(B=2, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, total_N=1000), D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=8, dtype=7, N=576, K=64), D.DART_ERR_DTYPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, pivot_mode=5), D.DART_ERR_DTYPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, pivot_mode=4), D.DART_ERR_DTYPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, pivot_mode=-1), D.DART_ERR_DTYPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=7), D.DART_ERR_BUDGET),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=577), D.DART_ERR_BUDGET),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=4, K=4), D.DART_ERR_BUDGET),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=0, keep_num=1, keep_den=0),
     D.DART_ERR_BUDGET),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=0, keep_num=3, keep_den=2),
     D.DART_ERR_BUDGET),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=0, keep_num=1, keep_den=1000),
     D.DART_ERR_BUDGET),  # floor(0.576) = 0 < P
    # pivots from outside the samples
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, P_ext=9, ext_pivots=4096),
     D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, P_ext=-1), D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, P_ext=4), D.DART_ERR_NULL),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, P_ext=4, ext_pivots=4096,
          ext_ld=4000), D.DART_ERR_SHAPE),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=64, P_ext=4, ext_pivots=4100),
     D.DART_ERR_ALIGN),
    (dict(B=1, D=4096, P=8, dtype=D.DART_F32, N=576, K=64, P_ext=4, ext_pivots=4096,
          ext_ld=4098), D.DART_ERR_ALIGN),
    (dict(B=1, D=4096, P=8, dtype=D.DART_BF16, N=576, K=3, P_ext=4, ext_pivots=4096),
     D.DART_ERR_BUDGET),  # K < P - P_ext
    (dict(B=1, D=4100, P=8, dtype=D.DART_BF16, N=576, K=64), D.DART_ERR_ALIGN),
    (dict(B=1, D=4096, P=8, dtype=D.DART_F32, N=576, K=64, ld=4098), D.DART_ERR_ALIGN),
]


@pytest.mark.parametrize("kw,code", BAD)
def test_bad_descriptors_are_rejected_on_the_host(kw, code):
    kw = dict(kw)
    d = D.make_desc(kw.pop("B"), kw.pop("D"), kw.pop("P"), kw.pop("dtype"), **kw)
    assert D.dart_workspace_bytes(d) == 0
    L = binding.lib()
    fake = C.c_void_p(4096)  # never dereferenced: the descriptor is rejected first
    rc = L.dart_reduce(C.byref(d), fake, None, 0, 0, None, fake, None, fake, None, None, None,
                       fake, 1 << 40, None)
    assert rc == code, D.strerror(rc)


def test_null_and_workspace_errors_need_no_device():
    d = D.make_desc(1, 4096, 8, D.DART_BF16, N=576, K=64)
    L = binding.lib()
    fake = C.c_void_p(4096)
    need = D.dart_workspace_bytes(d)
    call = lambda X, Y, keep, ws, nbytes: L.dart_reduce(C.byref(d), X, None, 0, 0, None, Y, None,
                                                        keep, None, None, None, ws, nbytes, None)
    assert call(None, fake, fake, fake, need) == D.DART_ERR_NULL
    # Y == NULL is allowed (the compaction step is skipped): the next check is reached
    assert call(fake, None, fake, None, need) == D.DART_ERR_WORKSPACE
    assert call(fake, fake, None, fake, need) == D.DART_ERR_NULL
    assert call(fake, fake, fake, None, need) == D.DART_ERR_WORKSPACE
    assert call(fake, fake, fake, fake, need - 1) == D.DART_ERR_WORKSPACE
    assert call(fake, fake, fake, C.c_void_p(4096 + 8), need) == D.DART_ERR_WORKSPACE
    assert call(C.c_void_p(4100), fake, fake, fake, need) == D.DART_ERR_ALIGN
    # position ids come in pairs
    rc = L.dart_reduce(C.byref(d), fake, None, 0, 0, fake, fake, None, fake, None, None, None,
                       fake, need, None)
    assert rc == D.DART_ERR_NULL
    # caller-supplied pivots: the pivot list is required, and there is nothing to select
    dg = D.make_desc(1, 4096, 8, D.DART_BF16, N=576, K=64, pivot_mode=D.DART_PIVOT_GIVEN)
    assert D.dart_workspace_bytes(dg) == need
    rc = L.dart_reduce(C.byref(dg), fake, None, 0, 0, None, fake, None, fake, None, None, None,
                       fake, need, None)
    assert rc == D.DART_ERR_NULL
    rc = L.dart_select_pivots(C.byref(dg), fake, None, 0, 0, fake, None, fake, need, None)
    assert rc == D.DART_ERR_DTYPE
    # pivots drawn at random: a valid descriptor whatever the seed, the same workspace
    dr = D.make_desc(1, 4096, 8, D.DART_BF16, N=576, K=64, pivot_mode=D.DART_PIVOT_RANDOM,
                     seed=2**64 - 1)
    assert D.dart_workspace_bytes(dr) == need
    assert L.dart_select_pivots(C.byref(dr), fake, None, 0, 0, None, None, fake, need,
                                None) == D.DART_ERR_NULL  # the list it would write is missing
    # caller-supplied criterion norms: the norms are required, the error bound must be one,
    # and only the modes that rank norms take them
    wn = L.dart_reduce_with_norms
    assert wn(C.byref(d), fake, None, 0, 0, None, 1e-6, None, fake, None, fake, None, None, None,
              fake, need, None) == D.DART_ERR_NULL
    for bad_err in (-1e-9, 0.11, float("nan"), float("inf")):
        assert wn(C.byref(d), fake, None, 0, 0, fake, bad_err, None, fake, None, fake, None, None,
                  None, fake, need, None) == D.DART_ERR_SHAPE
    for dm in (dg, dr):
        assert wn(C.byref(dm), fake, None, 0, 0, fake, 1e-6, None, fake, None, fake, None, fake,
                  None, fake, need, None) == D.DART_ERR_DTYPE
    assert wn(C.byref(d), None, None, 0, 0, fake, 1e-6, None, fake, None, fake, None, None, None,
              fake, need, None) == D.DART_ERR_NULL  # X
    # an empty batch is a valid no-op and needs nothing else
    d0 = D.make_desc(0, 4096, 8, D.DART_BF16, N=576, K=64)
    assert L.dart_reduce(C.byref(d0), None, None, 0, 0, None, None, None, None, None, None,
                         None, None, 0, None) == D.DART_OK


def test_outside_pivots_relax_the_budget_check():
    """With P_ext pivots from outside, P - P_ext <= K suffices (they hold no slot), and the
    workspace does not depend on where the pivots come from."""
    base = D.dart_workspace_bytes(D.make_desc(1, 4096, 8, D.DART_BF16, N=576, K=64))
    d = D.make_desc(1, 4096, 8, D.DART_BF16, N=576, K=5, P_ext=4, ext_pivots=4096)
    assert D.dart_workspace_bytes(d) == base
    d = D.make_desc(1, 4096, 8, D.DART_BF16, N=576, K=1, P_ext=8, ext_pivots=4096)
    assert D.dart_workspace_bytes(d) == base


def test_spans_need_the_packed_lengths_and_the_row_count():
    fake = 4096
    ok = D.make_desc(2, 4096, 8, D.DART_BF16, keep_num=1, keep_den=9, cu_seqlens=None,
                     total_N=1000, max_N=600, span_start=fake, X_rows=1200)
    assert D.dart_workspace_bytes(ok) == 0          # dense layout: spans are refused
    ok.cu_seqlens = fake
    assert D.dart_workspace_bytes(ok) > 0
    ok.X_rows = 999                                  # fewer rows than scored tokens
    assert D.dart_workspace_bytes(ok) == 0
    # sequences exist only around spans
    L = binding.lib()
    d = D.make_desc(2, 4096, 8, D.DART_BF16, keep_num=1, keep_den=9, total_N=1000, max_N=600)
    d.cu_seqlens = fake
    p = C.c_void_p(fake)
    rc = L.dart_compact_sequences(C.byref(d), p, p, 0, None, None, 0, 0, None, 0, p, p, p,
                                  1 << 40, None)
    assert rc == D.DART_ERR_NULL
    d.span_start, d.X_rows = fake, 1200
    need = D.dart_workspace_bytes(d)
    t = (binding.DartRowTensor * 1)(binding.DartRowTensor(fake, fake, 100, 128, 128))
    rc = L.dart_compact_sequences(C.byref(d), p, p, 1, t, None, 0, 0, None, 0, p, p, p, need, None)
    assert rc == D.DART_ERR_ALIGN                    # rows must be multiples of 16 bytes
    t[0].row_bytes, t[0].src_ld_bytes = 128, 64
    rc = L.dart_compact_sequences(C.byref(d), p, p, 1, t, None, 0, 0, None, 0, p, p, p, need, None)
    assert rc == D.DART_ERR_SHAPE
    rc = L.dart_compact_sequences(C.byref(d), p, p, 0, None, None, 0, 0, None, 0, p, None, p,
                                  need, None)
    assert rc == D.DART_ERR_NULL                     # the row map is required


def test_status_strings():
    texts = [D.strerror(code) for code in range(0, -9, -1)]
    assert all(texts) and len(set(texts)) == 9
    assert D.strerror(-99) not in texts
    assert 0 < D.score_tolerance(D.DART_F32) < D.score_tolerance(D.DART_BF16) < 1e-4


def test_static_entry_refuses_what_its_buffer_cannot_hold():
    """dart_reduce_static checks the descriptor against the built-in buffer on the host, before
    anything touches a device."""
    limit = D.dart_static_scratch_bytes()
    assert limit == 32 << 20
    fits = D.make_desc(8, 4096, 16, D.DART_BF16, N=2880, K=320)
    assert D.dart_workspace_bytes(fits) <= limit
    video = D.make_desc(4, 3584, 32, D.DART_BF16, N=9216, K=1024)
    assert D.dart_workspace_bytes(video) <= limit
    big = D.make_desc(32, 3584, 16, D.DART_BF16, keep_num=111, keep_den=1000, total_N=250000,
                      max_N=16384)
    big.cu_seqlens = 0x1000  # never dereferenced on the host
    assert D.dart_workspace_bytes(big) > limit
    L = binding.lib()
    rc = L.dart_reduce_static(C.byref(big), 0x1000, None, 0, 0, None, 0x1000, None, 0x1000, None,
                              None, None, None)
    assert rc == D.DART_ERR_STATIC_LIMIT
    assert "built-in buffer" in D.strerror(rc)
    bad = D.make_desc(1, 4096, 0, D.DART_BF16, N=576, K=64)
    assert L.dart_reduce_static(C.byref(bad), 0x1000, None, 0, 0, None, 0x1000, None, 0x1000,
                                None, None, None, None) == D.DART_ERR_SHAPE


def _built_tile_shapes(P):
    """Every (waves, groups) the library accepts from DART_SCORE_TILE for P pivots."""
    desc = D.make_desc(4, 1024, P, D.DART_BF16, N=600, K=max(P, 64))
    found = []
    try:
        for w in range(1, 17):
            for ks in range(1, 5):
                os.environ["DART_SCORE_TILE"] = f"{w},{ks}"
                try:
                    assert D.dart_score_tile_shape(desc) == (w, ks)
                    found.append((w, ks))
                except D.DartError as e:
                    assert e.status == D.DART_ERR_SHAPE
    finally:
        del os.environ["DART_SCORE_TILE"]
    return found


def test_score_tile_shape_follows_the_batch_and_the_override():
    """The tile chooser is host arithmetic: the benchmark shapes get the tiles that spread
    their rows evenly over 256 compute units, fp32 has no choice, and the environment override
    is honoured for built shapes and refused (by every entry point) for anything else."""
    assert "DART_SCORE_TILE" not in os.environ
    # 8 x 2880 rows: 96-row tiles = 240 tiles, every unit at most one
    assert D.dart_score_tile_shape(D.make_desc(8, 4096, 16, D.DART_BF16, N=2880, K=320)) == (6, 1)
    # 4 x 9216 rows: 144-row tiles = 256 tiles, one per unit
    assert D.dart_score_tile_shape(D.make_desc(4, 3584, 32, D.DART_BF16, N=9216, K=1024)) == (9, 1)
    # 16 x 576 rows: 48-row tiles, the hidden dimension split over four groups of waves
    assert D.dart_score_tile_shape(D.make_desc(16, 4096, 8, D.DART_BF16, N=576, K=64)) == (12, 4)
    # a first read of X (no norm pass before the score pass) changes small dense batches only:
    # the headline shape goes to four groups of waves on tiles that load no unit more ...
    head = D.make_desc(8, 4096, 16, D.DART_BF16, N=2880, K=320)
    w, ks = D.dart_score_tile_shape_first_read(head)
    assert (w, ks) == (8, 4)
    for mode in (D.DART_PIVOT_GIVEN, D.DART_PIVOT_RANDOM):  # (no norm pass exists for these)
        assert D.dart_score_tile_shape(D.make_desc(8, 4096, 16, D.DART_BF16, N=2880, K=320,
                                                   pivot_mode=mode)) == (w, ks)
    # ... while 32 pivots, or a ragged batch with thousands of tiles, keep their single group
    video = D.make_desc(4, 3584, 32, D.DART_BF16, N=9216, K=1024)
    assert D.dart_score_tile_shape_first_read(video) == (9, 1)
    ragged = D.make_desc(32, 3584, 16, D.DART_BF16, keep_num=111, keep_den=1000,
                         total_N=234356, max_N=16384)
    ragged.cu_seqlens = 0x1000  # never dereferenced on the host
    assert D.dart_score_tile_shape_first_read(ragged) == D.dart_score_tile_shape(ragged)
    assert D.dart_score_tile_shape_first_read(D.make_desc(1, 4096, 8, D.DART_F32, N=576,
                                                          K=64)) == (0, 0)
    assert D.dart_score_tile_shape(D.make_desc(1, 4096, 8, D.DART_F32, N=576, K=64)) == (0, 0)
    shapes = _built_tile_shapes(8)
    assert len(shapes) >= 15 and (6, 1) in shapes and (9, 1) in shapes and (1, 1) not in shapes
    assert all(w % ks == 0 for w, ks in shapes)
    # with 64 pivots the widest split shapes do not fit the LDS and are refused
    assert set(_built_tile_shapes(64)) < set(shapes)
    desc = D.make_desc(2, 1024, 8, D.DART_BF16, N=300, K=32)
    os.environ["DART_SCORE_TILE"] = "7,5"
    try:
        assert D.dart_workspace_bytes(desc) == 0
        with pytest.raises(D.DartError) as e:
            D.dart_score_tile_shape(desc)
        assert e.value.status == D.DART_ERR_SHAPE
    finally:
        del os.environ["DART_SCORE_TILE"]
    assert D.dart_workspace_bytes(desc) > 0
    L = binding.lib()
    w = C.c_int32(7)
    assert L.dart_score_tile_shape(C.byref(desc), None, C.byref(w)) == D.DART_ERR_NULL
    assert L.dart_score_tile_shape(C.byref(desc), C.byref(w), None) == D.DART_ERR_NULL
    assert L.dart_score_tile_shape(None, C.byref(w), C.byref(w)) == D.DART_ERR_NULL
    assert w.value == 7  # nothing is written on an error
