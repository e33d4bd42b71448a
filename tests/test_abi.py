"""The C ABI library loads, exports every symbol include/goq.h declares, and rejects bad
arguments on the host before any launch.  No GPU, no compute calls."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def goq():
    import paper_2605_26092_amd as g
    from paper_2605_26092_amd import build
    build.build(force=False)
    g.lib()
    return g


def test_every_declared_symbol_is_exported(goq):
    hdr = open(os.path.join(ROOT, "include", "goq.h")).read()
    declared = set(re.findall(r"\b(goq_[a-z_0-9]+)\s*\(", hdr))
    from paper_2605_26092_amd import binding
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(goq.lib(), name), name


def test_version_and_packed_bytes(goq):
    assert goq.version() >= 1000
    # 4.0 / 5.0 bits per weight, rows padded to 64
    assert goq.packed_bytes(3, 4096, 4096) == 4096 * 4096 // 2
    assert goq.packed_bytes(4, 4096, 4096) == 4096 * 4096 * 5 // 8
    assert goq.packed_bytes(3, 65, 128) == 128 * 128 // 2
    assert goq.packed_bytes(3, 11008, 4096) == 11008 * 4096 // 2


def test_host_side_argument_errors(goq):
    from paper_2605_26092_amd import binding as b
    L = goq.lib()
    n = ctypes.c_size_t()
    assert L.goq_packed_bytes(5, 64, 128, ctypes.byref(n)) == b.EINVAL
    assert "bw" in goq.last_error()
    assert L.goq_packed_bytes(3, 64, 4100, ctypes.byref(n)) == b.ESHAPE
    assert L.goq_packed_bytes(3, 0, 128, ctypes.byref(n)) == b.ESHAPE
    assert L.goq_packed_bytes(3, 64, 128, None) == b.EINVAL
    fake = 0x1000   # never dereferenced: validation fails first
    assert L.goq_pack(None, 3, 64, 128, None, fake, fake, fake, fake, fake) == b.EINVAL
    assert L.goq_pack(None, 3, 64, 128, fake, fake, fake, fake, fake, fake + 4) == b.EINVAL
    assert L.goq_gemv(None, 3, 0, 64, 100, fake, fake, None, fake, 1) == b.ESHAPE
    assert L.goq_gemv(None, 3, 7, 64, 128, fake, fake, None, fake, 1) == b.EINVAL
    assert L.goq_gemv(None, 3, 0, 64, 128, fake, fake, None, fake, 9) == b.EINVAL
    assert L.goq_gemv(None, 3, 1, 64, 128, fake, fake, None, fake, 1) == b.EINVAL      # A8 needs sx
    assert L.goq_gemv(None, 4, 2, 64, 128, fake, fake, None, fake, 1) == b.EINVAL      # A4 needs sx
    assert L.goq_gemm(None, 3, 5, 4, 64, 128, fake, fake, fake, fake, 1, None) == b.EINVAL   # no such activation type
    assert L.goq_gemv(None, 3, 4, 64, 128, fake, fake, None, fake, 1) == b.EINVAL      # A3 needs sx
    assert L.goq_gemv(None, 3, 3, 64, 128, fake, fake, None, fake, 1) == b.EINVAL      # A6 needs sx
    assert L.goq_gemv(None, 3, 0, 64, 128, fake, fake, fake, fake, 1) == b.EINVAL      # A16 forbids sx
    assert L.goq_gemm_batch(None, 3, 0, 0, None) == b.EINVAL
    assert L.goq_gemm_batch(None, 3, 0, 9, (b._GemmDesc * 9)()) == b.ESHAPE
    assert L.goq_gemm_batch(None, 3, 0, 1, (b._GemmDesc * 1)()) == b.ESHAPE             # out = in = 0
    assert L.goq_gemm_folded(None, 3, 4, 64, 100, fake, fake, fake, 1) == b.ESHAPE
    assert L.goq_gemm_folded(None, 3, 4, 64, 128, fake, None, fake, 1) == b.EINVAL
    assert L.goq_gemv_select(3) == b.EINVAL and "goq_gemv_select" in goq.last_error()
    assert L.goq_gemv_select(b.GEMV_ROWS) == b.OK and L.goq_gemv_select(b.GEMV_AUTO) == b.OK
    assert L.goq_gemv(None, 3, 0, 64, 128, fake, fake + 2, None, fake, 1) == b.EINVAL  # misaligned x
    assert L.goq_gemm(None, 3, 0, 0, 64, 128, fake, fake, None, fake, 1, None) == b.ESHAPE
    assert L.goq_gemm(None, 3, 0, 4, 64, 128, fake, fake, None, fake, 1, fake) == b.EINVAL
    assert L.goq_gemv_batch(None, 3, 0, 0, None) == b.EINVAL
    with pytest.raises(goq.GoqError):
        goq.packed_bytes(3, 64, 64)


def test_gemv_plan_follows_the_documented_choice(goq):
    """Host logic of the automatic kernel choice (include/goq.h): at most 512 tiles of 16 rows and
    24576 (tile, macro-block) pairs -> row-owner kernel, one workgroup per tile; else the streaming
    kernel with min(units, 512) workgroups, a unit being 512 rows x one macro-block."""
    b3 = lambda shapes: goq.gemv_plan(3, goq.A16, shapes)
    assert b3([(4096, 4096)]) == (goq.GEMV_ROWS, 256)
    assert b3([(8192, 4096)]) == (goq.GEMV_ROWS, 512)
    assert b3([(8208, 128)]) == (goq.GEMV_STREAM, 17)                   # 513 tiles
    assert b3([(8192, 8192)]) == (goq.GEMV_STREAM, 512)                 # 512 tiles x 64 = 32768 pairs
    assert b3([(4096, 11008)]) == (goq.GEMV_ROWS, 256)                  # 256 x 86 = 22016 pairs
    assert b3([(17, 128), (33, 256)]) == (goq.GEMV_ROWS, 2 + 3)
    block = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    assert b3(block) == (goq.GEMV_STREAM, 512)
    assert goq.gemv_plan(4, goq.A8, [(4096, 4096)]) == (goq.GEMV_ROWS, 256)
    try:
        goq.gemv_select(goq.GEMV_STREAM)
        assert b3([(4096, 4096)]) == (goq.GEMV_STREAM, 256)             # 8 row groups x 32 macro-blocks
        assert b3([(100, 256)]) == (goq.GEMV_STREAM, 2)
        goq.gemv_select(goq.GEMV_ROWS)
        assert b3(block) == (goq.GEMV_ROWS, 4 * 256 + 2 * 688 + 256)
    finally:
        goq.gemv_select(goq.GEMV_AUTO)
    with pytest.raises(goq.GoqError):
        goq.gemv_plan(3, goq.A16, [(64, 100)])


def _table_words(goq, bw, act, shapes):
    """goq_gemv_stream_table on descriptors with made-up (aligned, never dereferenced) pointers ->
    (header int32 view, problems as int32 rows of 16)."""
    import numpy as np
    from paper_2605_26092_amd import binding as b
    arr = (b._Desc * len(shapes))()
    for i, (d, (out, inn)) in enumerate(zip(arr, shapes)):
        d.out, d.in_ = out, inn
        d.packed, d.x, d.y = 0x100000 * (i + 1), 0x100000 * (i + 1) + 0x1000, 0x100000 * (i + 1) + 0x2000
        d.sx = None if act == goq.A16 else 0x100000 * (i + 1) + 0x3000
        d.ytype = goq.F32
    th, nbytes = goq.gemv_stream_table(bw, act, arr)
    raw = np.frombuffer((ctypes.c_ubyte * nbytes).from_address(ctypes.addressof(th)), dtype=np.uint8).copy()
    words = raw.view(np.int32)
    nprob = words[3]
    return words, words[len(words) - 16 * nprob:].reshape(nprob, 16)


def test_stream_table_cuts_the_unit_sequence_into_pieces(goq):
    """Host logic of goq_gemv_stream_table: units = row groups (512 rows) x macro-blocks of all
    problems in order; min(units, 512) pieces whose sizes differ by at most one, the larger first;
    first[b] = the problem that holds the first unit of piece b."""
    block = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    for shapes in ([(100, 256)], block, block * 32, [(1, 128), (700, 512), (64, 4096), (3000, 128)] * 5):
        words, probs = _table_words(goq, 3, goq.A16, shapes)
        magic, bw, act, n, total, nwg, pq, pr = (int(v) for v in words[:8])
        assert magic == 0x51544247 and bw == 3 and act == goq.A16 and n == len(shapes)
        units = [((out + 511) // 512) * (inn // 128) for out, inn in shapes]
        begins = [sum(units[:i]) for i in range(n)]
        assert total == sum(units) and nwg == min(total, 512)
        assert (pq, pr) == (total // nwg, total % nwg)
        # problem fields: gn at dword 9, rbn 11, rgroups 12, begin 13 (after four pointers and `out`)
        for i, (out, inn) in enumerate(shapes):
            assert int(probs[i][8]) == out and int(probs[i][9]) == inn // 128
            assert int(probs[i][11]) == (out + 63) // 64 and int(probs[i][12]) == (out + 511) // 512
            assert int(probs[i][13]) == begins[i]
        first = words[16:16 + 512]
        for piece in range(nwg):
            i0 = piece * pq + min(piece, pr)
            holder = max(i for i in range(n) if begins[i] <= i0)
            assert int(first[piece]) == holder, (piece, i0)


def test_stream_entry_points_reject_bad_arguments_on_the_host(goq):
    from paper_2605_26092_amd import binding as b
    L = goq.lib()
    n = ctypes.c_size_t()
    assert L.goq_gemv_stream_table_bytes(0, ctypes.byref(n)) == b.ESHAPE
    assert L.goq_gemv_stream_table_bytes(65537, ctypes.byref(n)) == b.ESHAPE
    assert L.goq_gemv_stream_table_bytes(7, None) == b.EINVAL
    assert L.goq_gemv_stream_table_bytes(224, ctypes.byref(n)) == b.OK and n.value == 2112 + 224 * 64
    arr = (b._Desc * 1)()
    arr[0].out, arr[0].in_, arr[0].packed, arr[0].x, arr[0].y, arr[0].ytype = 64, 128, 0x1000, 0x2000, 0x3000, goq.F32
    buf = (ctypes.c_uint64 * 512)()
    assert L.goq_gemv_stream_table(3, goq.A16, 1, arr, None) == b.EINVAL
    assert L.goq_gemv_stream_table(3, goq.A16, 1, arr, ctypes.addressof(buf) + 4) == b.EINVAL
    assert L.goq_gemv_stream_table(3, goq.A16, 0, arr, ctypes.addressof(buf)) == b.ESHAPE
    assert L.goq_gemv_stream_table(5, goq.A16, 1, arr, ctypes.addressof(buf)) == b.EINVAL
    assert L.goq_gemv_stream_table(3, goq.A8, 1, arr, ctypes.addressof(buf)) == b.EINVAL       # A8 needs sx
    arr[0].in_ = 100
    assert L.goq_gemv_stream_table(3, goq.A16, 1, arr, ctypes.addressof(buf)) == b.ESHAPE
    arr[0].in_ = 128
    assert L.goq_gemv_stream_table(3, goq.A16, 1, arr, ctypes.addressof(buf)) == b.OK
    fake = 0x10000
    # a host table that goq_gemv_stream_table did not write is refused before any launch
    junk = (ctypes.c_uint64 * 512)()
    assert L.goq_gemv_stream(None, ctypes.addressof(junk), fake, fake) == b.EINVAL
    assert L.goq_gemv_stream(None, None, fake, fake) == b.EINVAL
    assert L.goq_gemv_stream(None, ctypes.addressof(buf), fake + 8, fake) == b.EINVAL           # table_dev misaligned
    assert L.goq_gemv_stream(None, ctypes.addressof(buf), fake, fake + 16) == b.EINVAL          # workspace misaligned
    assert L.goq_gemv_workspace_bytes(None) == b.EINVAL
    assert L.goq_gemv_workspace_bytes(ctypes.byref(n)) == b.OK and n.value > 2 * 512 * 512 * 4
    assert L.goq_gemv_batch_ws(None, 3, goq.A16, 1, arr, None) == b.EINVAL
    assert L.goq_gemv_batch_ws(None, 3, goq.A16, 1, arr, fake + 16) == b.EINVAL
