"""Bit-level layouts of the stored operands, written out independently of the GPU code.

The paper fixes only the logical content of the formats ("3/4-bit", "group size
128", "asymmetric", Sec. 4.1 and App. A.11; "2:4", Sec. 1; "quantise EoRA to
4-bit", Sec. 4.5).  The byte placement below is this project's own and is
restated here from its specification, not shared with the HIP sources.

All weight-like operands (a matrix with `rows` output rows and `K` contraction
columns) are stored TILE-MAJOR.  A tile covers 16 consecutive rows and KT
consecutive columns and belongs to a 64-lane wavefront: lane l = 16*j + n owns
row n of the tile and the j-th quarter of its columns.  Tiles are ordered
row-block first:  tile index = R * (K / KT) + g,  R = row // 16, g = col // KT.

Q4  (4-bit codes, KT = 128 for the backbone, min(128, K) for a factor)
    lane owns columns  c = (KT/4)*j + 8*t + kk  (t = word of the lane, kk = 0..7)
    word index in the array = tile*(64*KT/32) + l*(KT/32) + t
    the code of column kk sits in nibble e = 4*(kk % 2) + kk // 2 of that word
    (even columns fill nibbles 0..3, odd columns nibbles 4..7)

Q3  (3-bit codes, KT = 128): three words per lane, word index = tile*192 + 3*l + d.
    The lane owns 32 columns cc = 0..31 of its quarter.  Columns 0..29 form 15
    pairs p = cc // 2 (h = cc % 2 is the 16-bit half: 0 low, 1 high); pair p
    sits in word d = p // 5 at bits 16*h + 3*(p % 5) .. +2.  Bit 15 of each
    half is spare; the spare bits carry the last two codes: bit b of the code
    of column 30 + h is bit 16*h + 15 of word b.

Q2  (2-bit codes, KT = 128): two words per lane, word index = tile*128 + 2*l + u.
    The lane owns 32 columns cc = 0..31 of its quarter; column cc sits in word u = cc // 16 at bits
    16*h + 2*p .. +1 with h = cc % 2 (the 16-bit half) and p = (cc % 16) // 2 (eight pairs of adjacent
    columns per word, even column in the low half, odd column in the high half, same bit offset).
    Zero-points (< 4) use the common nibble array.

zeros   one nibble per (row, quantisation group), row-major, eight groups per
        32-bit word: word row*NGW + q // 8, nibble q % 8
        (NG = K / group, q = col // group, NGW = ceil(NG / 8))
scales  fp16, row-major: element row*NG + q

F16 (fp16 factor, KT = 32): element index = (tile*64 + l)*8 + i for column
    32*g + 8*j + i.

SP24 (2:4 sparse fp16 backbone, tile = 16 rows x 128 dense columns)
    the lane owns dense columns 64*s + 16*j + 4*q + p  (s = 0,1 half of the
    tile, q = 0..3 group of four, p = 0..3 position).  Each group keeps two
    values v = 0,1 at positions p_0 < p_1.
    values:  element tile*1024 + s*512 + l*8 + 2*q + v
    indices: one uint32 per (tile, lane): bits 16*s + 4*q + 2*v .. +1 = p_v

SP24Q4 (2:4 sparse backbone whose kept values are 4-bit codes, tile = 16 rows x 128 dense columns)
    tiles: three uint32 per (tile, lane), words (tile*64 + l)*3 + 0, 1, 2:
        word s = 0, 1: the lane's eight kept values of half s, element e = 2*q + v in nibble
        4*(e % 2) + e // 2 (the Q4 nibble order); word 2: the SP24 index word.
    meta: one uint32 per (tile, row n), word tile*16 + n: bits 0..15 the fp16 scale, bits 16..19 the
        zero-point of the quantisation group that holds the tile's columns (a group of `group` DENSE
        columns, group a multiple of 128, covers group/128 tiles, which repeat its scale and zero).
"""
import numpy as np

ROWS = 16          # rows of a tile
LANES = 64


def _check(rows, K, KT):
    if rows % ROWS or K % KT or KT % 32:
        raise ValueError("rows must be a multiple of 16 and K of the k-tile")


# ----------------------------------------------------------------------------
# 4-bit codes
# ----------------------------------------------------------------------------
def q4_locate(o, i, K, KT):
    """(word index, bit shift) of the code of row o, column i."""
    R, n = o // ROWS, o % ROWS
    g, c = i // KT, i % KT
    per_lane = KT // 4
    j, cc = c // per_lane, c % per_lane
    t, kk = cc // 8, cc % 8
    e = 4 * (kk % 2) + kk // 2
    wpl = KT // 32
    lane = 16 * j + n
    tile = R * (K // KT) + g
    return tile * (LANES * wpl) + lane * wpl + t, 4 * e


def pack_q4(codes, KT=128):
    """Word-walk direction: every output word gathers the eight codes it holds."""
    codes = np.asarray(codes)
    rows, K = codes.shape
    _check(rows, K, KT)
    if codes.min(initial=0) < 0 or codes.max(initial=0) > 15:
        raise ValueError("4-bit code out of range")
    wpl, ntk = KT // 32, K // KT
    w = np.arange(rows * K // 8)
    tile, rem = w // (LANES * wpl), w % (LANES * wpl)
    lane, t = rem // wpl, rem % wpl
    R, g = tile // ntk, tile % ntk
    j, n = lane // 16, lane % 16
    row = 16 * R + n
    col0 = g * KT + j * (KT // 4) + 8 * t
    out = np.zeros(w.size, dtype=np.uint32)
    for kk in range(8):
        e = 4 * (kk % 2) + kk // 2
        out |= codes[row, col0 + kk].astype(np.uint32) << np.uint32(4 * e)
    return out


def unpack_q4(words, rows, K, KT=128):
    words = np.asarray(words, dtype=np.uint32)
    _check(rows, K, KT)
    if words.size != rows * K // 8:
        raise ValueError("wrong number of words")
    o, i = np.meshgrid(np.arange(rows), np.arange(K), indexing="ij")
    word, shift = q4_locate(o, i, K, KT)
    return ((words[word] >> shift.astype(np.uint32)) & 0xF).astype(np.uint8)


# ----------------------------------------------------------------------------
# 3-bit codes
# ----------------------------------------------------------------------------
def _q3_lane(o, i, K):
    R, n = o // ROWS, o % ROWS
    g, c = i // 128, i % 128
    j, cc = c // 32, c % 32
    lane = 16 * j + n
    tile = R * (K // 128) + g
    return tile * 192 + 3 * lane, cc


def pack_q3(codes):
    """Word-walk direction: every lane gathers its 32 codes and lays them into its three words."""
    codes = np.asarray(codes)
    rows, K = codes.shape
    _check(rows, K, 128)
    if codes.min(initial=0) < 0 or codes.max(initial=0) > 7:
        raise ValueError("3-bit code out of range")
    ntk = K // 128
    L = np.arange(rows * K // 32)                   # global (tile, lane)
    tile, lane = L // LANES, L % LANES
    R, g = tile // ntk, tile % ntk
    j, n = lane // 16, lane % 16
    row = 16 * R + n
    col0 = 128 * g + 32 * j
    d = [np.zeros(L.size, dtype=np.uint32) for _ in range(3)]
    for cc in range(30):                            # the fifteen in-place pairs
        p, h = cc // 2, cc % 2
        d[p // 5] |= codes[row, col0 + cc].astype(np.uint32) << np.uint32(16 * h + 3 * (p % 5))
    for h in range(2):                              # the two codes spread over the spare bits
        q = codes[row, col0 + 30 + h].astype(np.uint32)
        for b in range(3):
            d[b] |= ((q >> np.uint32(b)) & np.uint32(1)) << np.uint32(16 * h + 15)
    return np.stack(d, axis=1).reshape(-1)


def unpack_q3(words, rows, K):
    words = np.asarray(words, dtype=np.uint32)
    _check(rows, K, 128)
    if words.size != rows * K * 3 // 32:
        raise ValueError("wrong number of words")
    o, i = np.meshgrid(np.arange(rows), np.arange(K), indexing="ij")
    base, cc = _q3_lane(o, i, K)
    p, h = cc // 2, cc % 2
    pc = np.minimum(p, 14)                      # clamp so the gather below stays in range
    s = (16 * h + 3 * (pc % 5)).astype(np.uint32)
    inplace = (words[base + pc // 5] >> s) & 7
    hs = np.clip(cc - 30, 0, 1)
    s15 = (16 * hs + 15).astype(np.uint32)
    spread = np.zeros_like(inplace)
    for b in range(3):
        spread |= ((words[base + b] >> s15) & 1) << np.uint32(b)
    return np.where(cc < 30, inplace, spread).astype(np.uint8)


# ----------------------------------------------------------------------------
# 2-bit codes
# ----------------------------------------------------------------------------
def q2_locate(o, i, K):
    """(word index, bit shift) of the code of row o, column i."""
    R, n = o // ROWS, o % ROWS
    g, c = i // 128, i % 128
    j, cc = c // 32, c % 32
    u, p, h = cc // 16, (cc % 16) // 2, cc % 2
    lane = 16 * j + n
    tile = R * (K // 128) + g
    return tile * 128 + 2 * lane + u, 16 * h + 2 * p


def pack_q2(codes):
    """Word-walk direction: every output word gathers the sixteen codes it holds."""
    codes = np.asarray(codes)
    rows, K = codes.shape
    _check(rows, K, 128)
    if codes.min(initial=0) < 0 or codes.max(initial=0) > 3:
        raise ValueError("2-bit code out of range")
    ntk = K // 128
    w = np.arange(rows * K // 16)
    tile, rem = w // 128, w % 128
    lane, u = rem // 2, rem % 2
    R, g = tile // ntk, tile % ntk
    j, n = lane // 16, lane % 16
    row = 16 * R + n
    col0 = 128 * g + 32 * j + 16 * u
    out = np.zeros(w.size, dtype=np.uint32)
    for p in range(8):
        for h in range(2):
            out |= codes[row, col0 + 2 * p + h].astype(np.uint32) << np.uint32(16 * h + 2 * p)
    return out


def unpack_q2(words, rows, K):
    words = np.asarray(words, dtype=np.uint32)
    _check(rows, K, 128)
    if words.size != rows * K // 16:
        raise ValueError("wrong number of words")
    o, i = np.meshgrid(np.arange(rows), np.arange(K), indexing="ij")
    word, shift = q2_locate(o, i, K)
    return ((words[word] >> shift.astype(np.uint32)) & 3).astype(np.uint8)


# ----------------------------------------------------------------------------
# zero-points and scales of the quantisation groups
# ----------------------------------------------------------------------------
def pack_zeros(zeros):
    """rows x NG zero-points -> uint32 words, row-major, eight groups per word."""
    zeros = np.asarray(zeros)
    rows, NG = zeros.shape
    if zeros.min(initial=0) < 0 or zeros.max(initial=0) > 15:
        raise ValueError("zero-point out of range")
    NGW = (NG + 7) // 8
    out = np.zeros((rows, NGW), dtype=np.uint32)
    for q in range(NG):
        out[:, q // 8] |= zeros[:, q].astype(np.uint32) << np.uint32(4 * (q % 8))
    return out.reshape(-1)


def unpack_zeros(words, rows, NG):
    NGW = (NG + 7) // 8
    words = np.asarray(words, dtype=np.uint32).reshape(rows, NGW)
    q = np.arange(NG)
    return ((words[:, q // 8] >> (4 * (q % 8)).astype(np.uint32)[None, :]) & 0xF).astype(np.uint8)


def pack_scales(scales):
    """fp16 scales are stored as they are: row-major rows x NG."""
    return np.ascontiguousarray(scales, dtype=np.float16).reshape(-1)


def unpack_scales(flat, rows, NG):
    return np.asarray(flat, dtype=np.float16).reshape(rows, NG)


# ----------------------------------------------------------------------------
# fp16 factor
# ----------------------------------------------------------------------------
def _f16_index(o, i, K):
    R, n = o // ROWS, o % ROWS
    g, c = i // 32, i % 32
    j, ii = c // 8, c % 8
    tile = R * (K // 32) + g
    return (tile * LANES + 16 * j + n) * 8 + ii


def pack_f16(mat):
    mat = np.asarray(mat, dtype=np.float16)
    rows, K = mat.shape
    _check(rows, K, 32)
    o, i = np.meshgrid(np.arange(rows), np.arange(K), indexing="ij")
    out = np.empty(rows * K, dtype=np.float16)
    out[_f16_index(o, i, K).ravel()] = mat.ravel()
    return out


def unpack_f16(flat, rows, K):
    flat = np.asarray(flat, dtype=np.float16)
    o, i = np.meshgrid(np.arange(rows), np.arange(K), indexing="ij")
    return flat[_f16_index(o, i, K)]


# ----------------------------------------------------------------------------
# 2:4 sparse fp16 backbone
# ----------------------------------------------------------------------------
def _sp24_locate(o, u, K):
    """o: row, u: index of the kept value along the row (0 .. K/2-1).
    Returns (value element index, index-word index, bit shift)."""
    grp, v = u // 2, u % 2          # group of four dense columns, which of its two values
    dense0 = 4 * grp                # first dense column of the group
    R, n = o // ROWS, o % ROWS
    g, c = dense0 // 128, dense0 % 128
    s, c2 = c // 64, c % 64
    j, q = c2 // 16, (c2 % 16) // 4
    lane = 16 * j + n
    tile = R * (K // 128) + g
    return tile * 1024 + s * 512 + lane * 8 + 2 * q + v, tile * LANES + lane, 16 * s + 4 * q + 2 * v


def pack_sp24(vals, pos):
    """vals: fp16 rows x K/2 kept values; pos: their positions 0..3 in the group of
    four, strictly ascending within each pair."""
    vals = np.asarray(vals, dtype=np.float16)
    pos = np.asarray(pos)
    rows, half = vals.shape
    K = 2 * half
    _check(rows, K, 128)
    if pos.shape != vals.shape or pos.min(initial=0) < 0 or pos.max(initial=0) > 3:
        raise ValueError("bad positions")
    if np.any(pos[:, 0::2] >= pos[:, 1::2]):
        raise ValueError("positions of a pair must be strictly ascending")
    o, u = np.meshgrid(np.arange(rows), np.arange(half), indexing="ij")
    ve, iw, sh = _sp24_locate(o, u, K)
    values = np.empty(rows * half, dtype=np.float16)
    values[ve.ravel()] = vals.ravel()
    indices = np.zeros(rows * K // 128 * 4, dtype=np.uint32)  # 64 words per tile of 16 rows
    np.bitwise_or.at(indices, iw.ravel(), (pos.astype(np.uint32) << sh.astype(np.uint32)).ravel())
    return values, indices


def unpack_sp24(values, indices, rows, K):
    values = np.asarray(values, dtype=np.float16)
    indices = np.asarray(indices, dtype=np.uint32)
    _check(rows, K, 128)
    o, u = np.meshgrid(np.arange(rows), np.arange(K // 2), indexing="ij")
    ve, iw, sh = _sp24_locate(o, u, K)
    return values[ve], ((indices[iw] >> sh.astype(np.uint32)) & 3).astype(np.uint8)


# ----------------------------------------------------------------------------
# 2:4 sparse backbone with 4-bit kept values
# ----------------------------------------------------------------------------
def _sp24q4_locate(o, u, K):
    """o: row, u: index of the kept value along the row (0 .. K/2-1).
    Returns (code word index, code bit shift, index-word index, index bit shift)."""
    grp, v = u // 2, u % 2
    dense0 = 4 * grp
    R, n = o // ROWS, o % ROWS
    g, c = dense0 // 128, dense0 % 128
    s, c2 = c // 64, c % 64
    j, q = c2 // 16, (c2 % 16) // 4
    lane = 16 * j + n
    tile = R * (K // 128) + g
    e = 2 * q + v
    base = (tile * LANES + lane) * 3
    return base + s, 4 * (4 * (e % 2) + e // 2), base + 2, 16 * s + 4 * q + 2 * v


def pack_sp24q4(codes, pos, zeros, scales, group):
    """codes: uint8 rows x K/2 (4-bit codes of the kept values); pos: their positions 0..3, strictly
    ascending within each pair; zeros uint8 / scales fp16: rows x K/group.
    Returns (tile words uint32, meta words uint32)."""
    codes = np.asarray(codes)
    pos = np.asarray(pos)
    zeros = np.asarray(zeros)
    scales = np.asarray(scales, dtype=np.float16)
    rows, half = codes.shape
    K = 2 * half
    _check(rows, K, 128)
    if group % 128 or K % group or zeros.shape != (rows, K // group) or scales.shape != zeros.shape:
        raise ValueError("bad quantisation groups")
    if codes.min(initial=0) < 0 or codes.max(initial=0) > 15 or zeros.min(initial=0) < 0 or zeros.max(initial=0) > 15:
        raise ValueError("codes and zero-points must be 4-bit")
    if pos.shape != codes.shape or pos.min(initial=0) < 0 or pos.max(initial=0) > 3:
        raise ValueError("bad positions")
    if np.any(pos[:, 0::2] >= pos[:, 1::2]):
        raise ValueError("positions of a pair must be strictly ascending")
    o, u = np.meshgrid(np.arange(rows), np.arange(half), indexing="ij")
    cw, csh, iw, ish = _sp24q4_locate(o, u, K)
    tiles = np.zeros(rows * K // 128 * 12, dtype=np.uint32)        # 192 words per tile of 16 rows
    np.bitwise_or.at(tiles, cw.ravel(), (codes.astype(np.uint32) << csh.astype(np.uint32)).ravel())
    np.bitwise_or.at(tiles, iw.ravel(), (pos.astype(np.uint32) << ish.astype(np.uint32)).ravel())
    ntk = K // 128
    meta = np.zeros(rows // ROWS * ntk * ROWS, dtype=np.uint32)
    oo, gg = np.meshgrid(np.arange(rows), np.arange(ntk), indexing="ij")
    q = (gg * 128) // group
    word = scales.view(np.uint16)[oo, q].astype(np.uint32) | (zeros[oo, q].astype(np.uint32) << 16)
    meta[((oo // ROWS) * ntk + gg) * ROWS + oo % ROWS] = word
    return tiles, meta


def unpack_sp24q4(tiles, meta, rows, K):
    """-> (codes, positions, zeros per (row, tile), scales per (row, tile))."""
    tiles = np.asarray(tiles, dtype=np.uint32)
    meta = np.asarray(meta, dtype=np.uint32)
    _check(rows, K, 128)
    o, u = np.meshgrid(np.arange(rows), np.arange(K // 2), indexing="ij")
    cw, csh, iw, ish = _sp24q4_locate(o, u, K)
    ntk = K // 128
    oo, gg = np.meshgrid(np.arange(rows), np.arange(ntk), indexing="ij")
    m = meta[((oo // ROWS) * ntk + gg) * ROWS + oo % ROWS]
    return (((tiles[cw] >> csh.astype(np.uint32)) & 15).astype(np.uint8),
            ((tiles[iw] >> ish.astype(np.uint32)) & 3).astype(np.uint8),
            ((m >> 16) & 15).astype(np.uint8), (m & 0xFFFF).astype(np.uint16).view(np.float16))
