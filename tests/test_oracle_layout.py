"""Pins for oracle/layout.py: hand-derived bit positions (tests/golden), word-walking
pure-Python decoders written in the opposite direction, and round trips."""
import numpy as np
import pytest

from oracle import layout
from tests import pyref
from tests.golden_io import read_cases


def _run_case(kind, prm, sets, expect):
    if kind == "q4":
        rows, K, KT = prm["rows"], prm["K"], prm["KT"]
        codes = np.zeros((rows, K), np.uint8)
        for o, i, c in sets:
            codes[o, i] = c
        words = layout.pack_q4(codes, KT)
        back = layout.unpack_q4(words, rows, K, KT)
    elif kind == "q3":
        rows, K = prm["rows"], prm["K"]
        codes = np.zeros((rows, K), np.uint8)
        for o, i, c in sets:
            codes[o, i] = c
        words = layout.pack_q3(codes)
        back = layout.unpack_q3(words, rows, K)
    elif kind == "q2":
        rows, K = prm["rows"], prm["K"]
        codes = np.zeros((rows, K), np.uint8)
        for o, i, c in sets:
            codes[o, i] = c
        words = layout.pack_q2(codes)
        back = layout.unpack_q2(words, rows, K)
    elif kind == "zeros":
        rows, NG = prm["rows"], prm["NG"]
        codes = np.zeros((rows, NG), np.uint8)
        for o, q, c in sets:
            codes[o, q] = c
        words = layout.pack_zeros(codes)
        back = layout.unpack_zeros(words, rows, NG)
    elif kind == "sp24":
        rows, K = prm["rows"], prm["K"]
        codes = np.tile(np.array([0, 1], np.uint8), (rows, K // 4))
        for o, u, c in sets:
            codes[o, u] = c
        vals = np.arange(rows * K // 2, dtype=np.float32).reshape(rows, K // 2).astype(np.float16)
        _, words = layout.pack_sp24(vals, codes)
        _, back = layout.unpack_sp24(*layout.pack_sp24(vals, codes), rows, K)
        default = 0x44444444
    elif kind == "sp24q4":
        rows, K = prm["rows"], prm["K"]
        pos = np.tile(np.array([0, 1], np.uint8), (rows, K // 4))
        codes = np.zeros((rows, K // 2), np.uint8)
        for o, u, c in sets:
            codes[o, u] = c
        z1, s1 = np.zeros((rows, K // 128), np.uint8), np.ones((rows, K // 128), np.float16)
        words, _ = layout.pack_sp24q4(codes, pos, z1, s1, 128)
        back = layout.unpack_sp24q4(*layout.pack_sp24q4(codes, pos, z1, s1, 128), rows, K)[0]
    else:
        raise AssertionError(kind)
    default = 0x44444444 if kind == "sp24" else 0
    want = np.full(words.shape, default, np.uint32)
    if kind == "sp24q4":
        want[2::3] = 0x44444444                      # the index word of every lane
    for w, v in expect.items():
        want[w] = v
    assert np.array_equal(words, want), [(i, hex(a), hex(b)) for i, (a, b) in enumerate(zip(words, want)) if a != b][:8]
    assert np.array_equal(back, codes)


@pytest.mark.parametrize("name", ["layout_q4.txt", "layout_q3.txt", "layout_q2.txt", "layout_misc.txt"])
def test_golden_bit_positions(name):
    cases = read_cases(name)
    assert cases
    for kind, prm, sets, expect in cases:
        _run_case(kind, prm, sets, expect)


def test_sp24_value_positions_by_hand():
    # o=3 u=37 -> value element 512 + 3*8 + 2*2 + 1 = 541 ; o=0 u=1 -> element 1 (derivation in layout_misc.txt)
    rows, K = 16, 128
    pos = np.tile(np.array([0, 1], np.uint8), (rows, K // 4))
    vals = np.zeros((rows, K // 2), np.float16)
    vals[3, 37] = 2.5
    vals[0, 1] = -1.0
    # o=9 u=63: group 31, value 1, dense col 124: s=1 c2=60 j=3 q=3, lane 57 -> 512 + 57*8 + 7 = 975
    vals[9, 63] = 7.0
    values, _ = layout.pack_sp24(vals, pos)
    nz = {int(i): float(values[i]) for i in np.nonzero(values)[0]}
    assert nz == {541: 2.5, 1: -1.0, 975: 7.0}


def test_scales_and_f16_positions_by_hand():
    s = np.zeros((32, 2), np.float16)
    s[20, 1] = 3.0          # row-major: 20*2+1 = 41
    s[0, 0] = 1.5           # element 0
    s[15, 1] = 0.25         # 31
    flat = layout.pack_scales(s)
    assert {int(i): float(flat[i]) for i in np.nonzero(flat)[0]} == {41: 3.0, 0: 1.5, 31: 0.25}
    assert np.array_equal(layout.unpack_scales(flat, 32, 2), s)
    m = np.zeros((16, 64), np.float16)
    m[2, 45] = 9.0          # tile 1, j=1, i=5 -> (64 + 18)*8 + 5 = 661
    m[0, 0] = 1.0
    m[15, 31] = 2.0         # tile 0, j=3, i=7, lane 63 -> 63*8+7 = 511
    flat = layout.pack_f16(m)
    assert {int(i): float(flat[i]) for i in np.nonzero(flat)[0]} == {661: 9.0, 0: 1.0, 511: 2.0}
    assert np.array_equal(layout.unpack_f16(flat, 16, 64), m)


@pytest.mark.parametrize("rows,K,KT", [(16, 128, 128), (48, 384, 128), (32, 64, 64), (16, 512, 128)])
def test_q4_roundtrip_and_word_walk(rows, K, KT):
    rng = np.random.default_rng(rows * 1000 + K)
    codes = rng.integers(0, 16, (rows, K), dtype=np.uint8)
    words = layout.pack_q4(codes, KT)
    assert words.dtype == np.uint32 and words.size == rows * K // 8
    assert np.array_equal(layout.unpack_q4(words, rows, K, KT), codes)
    assert np.array_equal(np.array(pyref.decode_q4(words, rows, K, KT), dtype=np.uint8), codes)


@pytest.mark.parametrize("rows,K", [(16, 128), (32, 256), (48, 384)])
def test_q3_roundtrip_and_word_walk(rows, K):
    rng = np.random.default_rng(rows * 77 + K)
    codes = rng.integers(0, 8, (rows, K), dtype=np.uint8)
    words = layout.pack_q3(codes)
    assert words.size == rows * K * 3 // 32          # exactly 3.0 bits per weight
    assert np.array_equal(layout.unpack_q3(words, rows, K), codes)
    assert np.array_equal(np.array(pyref.decode_q3(words, rows, K), dtype=np.uint8), codes)


@pytest.mark.parametrize("rows,K", [(16, 128), (48, 384)])
def test_q2_roundtrip_and_word_walk(rows, K):
    rng = np.random.default_rng(rows + K + 2)
    codes = rng.integers(0, 4, (rows, K), dtype=np.uint8)
    words = layout.pack_q2(codes)
    assert words.size == rows * K // 16                     # 2.0 bits per weight, no padding
    assert np.array_equal(layout.unpack_q2(words, rows, K), codes)
    assert np.array_equal(np.array(pyref.decode_q2(words, rows, K), dtype=np.uint8), codes)
    assert np.all(layout.pack_q2(np.full((16, 128), 3, np.uint8)) == 0xFFFFFFFF)
    with pytest.raises(ValueError):
        layout.pack_q2(np.full((16, 128), 4, np.uint8))


def test_q3_all_ones_and_all_zero():
    ones = np.full((16, 128), 7, np.uint8)
    assert np.all(layout.pack_q3(ones) == 0xFFFFFFFF)      # every bit is used: no padding
    assert np.all(layout.pack_q3(np.zeros((16, 128), np.uint8)) == 0)
    assert np.all(layout.pack_q4(np.full((16, 128), 15, np.uint8)) == 0xFFFFFFFF)


def test_zeros_scales_roundtrip():
    rng = np.random.default_rng(5)
    z = rng.integers(0, 16, (48, 3), dtype=np.uint8)
    w = layout.pack_zeros(z)
    assert w.size == 48                                   # one (padded) word per row when NG <= 8
    assert layout.pack_zeros(np.zeros((48, 32), np.uint8)).nbytes == 48 * 32 // 2    # no padding when NG % 8 == 0
    assert np.array_equal(layout.unpack_zeros(w, 48, 3), z)
    assert np.array_equal(np.array(pyref.decode_zeros(w, 48, 3), dtype=np.uint8), z)
    s = rng.standard_normal((48, 3)).astype(np.float16)
    f = layout.pack_scales(s)
    assert np.array_equal(layout.unpack_scales(f, 48, 3), s)
    assert np.array_equal(np.array(pyref.decode_scales(f, 48, 3), dtype=np.float64), s.astype(np.float64))


def test_sp24_roundtrip_and_word_walk():
    from synth import prune_24
    rng = np.random.default_rng(11)
    W = rng.standard_normal((32, 256)).astype(np.float16)
    vals, pos = prune_24(W)
    values, indices = layout.pack_sp24(vals, pos)
    assert values.size == 32 * 128 and indices.size == 32 * 256 // 32   # 1.125 B per dense weight
    v2, p2 = layout.unpack_sp24(values, indices, 32, 256)
    assert np.array_equal(v2, vals) and np.array_equal(p2, pos)
    dense = np.array(pyref.decode_sp24(values, indices, 32, 256), dtype=np.float64)
    mask = np.zeros((32, 256), bool)
    mask[np.arange(32)[:, None], 4 * (np.arange(128) // 2)[None, :] + pos] = True
    assert np.array_equal(dense, np.where(mask, W.astype(np.float64), 0.0))
    assert np.all(mask.reshape(32, 64, 4).sum(axis=2) == 2)


def test_sp24q4_code_positions_by_hand():
    # Same (row, kept index) cases as the SP24 test above; derivation in layout_misc.txt.
    # o=3 u=37: group 18, v=1, dense col 72: tile 0, s=1, c2=8, j=0, q=2, lane 3, e=5 -> half 1 of lane 3, nibble 4*1+2=6
    # o=0 u=1:  group 0, v=1: s=0, j=0, q=0, lane 0, e=1 -> half 0 of lane 0, nibble 4
    # o=9 u=63: group 31, v=1, dense col 124: s=1, c2=60, j=3, q=3, lane 57, e=7 -> half 1 of lane 57, nibble 7
    rows, K = 16, 128
    pos = np.tile(np.array([0, 1], np.uint8), (rows, K // 4))
    codes = np.zeros((rows, K // 2), np.uint8)
    codes[3, 37] = 0xB
    codes[0, 1] = 0x5
    codes[9, 63] = 0xF
    zeros = np.zeros((rows, 1), np.uint8)
    scales = np.ones((rows, 1), np.float16)
    zeros[9, 0], scales[9, 0] = 7, 0.5                  # fp16 0.5 = 0x3800: meta word of (tile 0, row 9) = 0x00073800
    tiles, meta = layout.pack_sp24q4(codes, pos, zeros, scales, 128)
    cw = np.concatenate([tiles[0::3], tiles[1::3]])       # the code words: half 0 of every lane, then half 1
    nz = {int(i): int(cw[i]) for i in np.nonzero(cw)[0]}
    assert nz == {64 + 3: 0xB << 24, 0: 0x5 << 16, 64 + 57: 0xF << 28}
    # the index words are those of the fp16 format
    _, ref_idx = layout.pack_sp24(np.zeros((rows, K // 2), np.float16), pos)
    assert np.array_equal(tiles[2::3], ref_idx)
    assert int(meta[9]) == 0x00073800 and int(meta[0]) == 0x00003C00 and meta.size == 16


def test_sp24q4_roundtrip_word_walk_and_size():
    import synth
    rng = np.random.default_rng(12)
    W = rng.standard_normal((32, 512)).astype(np.float16)
    vals, pos = synth.prune_24(W)
    from oracle import linear
    for group in (128, 256):
        codes, zeros, scales = synth.quantize_kept_rtn(vals, pos, group)
        tiles, meta = layout.pack_sp24q4(codes, pos, zeros, scales, group)
        assert tiles.size * 4 == 32 * 512 * 3 // 8 and meta.size * 4 == 32 * 512 // 32     # 0.375 + 0.031 B per dense weight
        c2, p2, z2, s2 = layout.unpack_sp24q4(tiles, meta, 32, 512)
        assert np.array_equal(c2, codes) and np.array_equal(p2, pos)
        assert np.array_equal(z2, np.repeat(zeros, group // 128, axis=1))
        assert np.array_equal(s2.view(np.uint16), np.repeat(scales, group // 128, axis=1).view(np.uint16))
        dense = linear.dequant_sp24q4(codes, pos, zeros, scales, group)
        assert np.array_equal(linear.dequant_sp24q4_packed(tiles, meta, 512, 32), dense)
        walked = pyref.decode_sp24q4(tiles, meta, 32, 512)
        assert np.array_equal(np.array(walked, dtype=np.float64), dense)
    # exactly two non-pruned positions per group of four (a kept value may still dequantise to zero)
    mask = np.zeros((32, 512), bool)
    mask[np.arange(32)[:, None], 4 * (np.arange(256) // 2)[None, :] + pos] = True
    assert np.all(dense[~mask] == 0) and np.all(mask.reshape(32, 128, 4).sum(axis=2) == 2)


def test_sp24q4_with_unit_scale_is_the_fp16_format():
    """Scale 1 and zero-point 0 make the codes the kept values themselves: the dequantised matrix must be
    the expansion of the fp16 2:4 format holding the same numbers (which has its own pins)."""
    import synth
    from oracle import linear
    rng = np.random.default_rng(13)
    W = rng.standard_normal((16, 256)).astype(np.float16)
    _, pos = synth.prune_24(W)
    codes = rng.integers(0, 16, (16, 128)).astype(np.uint8)
    dense = linear.dequant_sp24q4(codes, pos, np.zeros((16, 2), np.uint8), np.ones((16, 2), np.float16), 128)
    assert np.array_equal(dense, linear.expand_sp24(codes.astype(np.float16), pos))


def test_pack_rejects_bad_input():
    with pytest.raises(ValueError):
        layout.pack_q4(np.full((16, 128), 16, np.uint8))
    with pytest.raises(ValueError):
        layout.pack_q3(np.full((16, 128), 8, np.uint8))
    with pytest.raises(ValueError):
        layout.pack_q4(np.zeros((8, 128), np.uint8))
    with pytest.raises(ValueError):
        layout.pack_sp24(np.zeros((16, 64), np.float16), np.zeros((16, 64), np.uint8))  # not ascending
