"""Pure-Python, word-by-word decoders of the stored formats, written in the
opposite direction from oracle/layout.py (they walk the words and scatter the
codes to (row, column)), plus an exact-rational forward pass.  Used only to pin
the oracle on tiny shapes."""
from fractions import Fraction

import numpy as np


def decode_q4(words, rows, K, KT=128):
    out = [[None] * K for _ in range(rows)]
    wpl = KT // 32
    ntk = K // KT
    for w, word in enumerate(int(v) for v in words):
        tile, rem = divmod(w, 64 * wpl)
        lane, t = divmod(rem, wpl)
        R, g = divmod(tile, ntk)
        j, n = divmod(lane, 16)
        for e in range(8):
            kk = 2 * (e % 4) + e // 4
            col = g * KT + j * (KT // 4) + 8 * t + kk
            out[16 * R + n][col] = (word >> (4 * e)) & 0xF
    return out


def decode_q2(words, rows, K):
    out = [[None] * K for _ in range(rows)]
    ntk = K // 128
    for w, word in enumerate(int(v) for v in words):
        lane_global, u = divmod(w, 2)
        tile, lane = divmod(lane_global, 64)
        R, g = divmod(tile, ntk)
        j, n = divmod(lane, 16)
        for h in range(2):
            half = (word >> (16 * h)) & 0xFFFF
            for p in range(8):
                out[16 * R + n][g * 128 + 32 * j + 16 * u + 2 * p + h] = (half >> (2 * p)) & 3
    return out


def decode_q3(words, rows, K):
    out = [[None] * K for _ in range(rows)]
    ntk = K // 128
    words = [int(v) for v in words]
    for lane_global in range(len(words) // 3):
        d0, d1, d2 = words[3 * lane_global: 3 * lane_global + 3]
        tile, lane = divmod(lane_global, 64)
        R, g = divmod(tile, ntk)
        j, n = divmod(lane, 16)
        base = g * 128 + 32 * j
        ws = (d0, d1, d2)
        for d in range(3):
            for h in range(2):
                half = (ws[d] >> (16 * h)) & 0xFFFF
                for u in range(5):
                    p = 5 * d + u
                    out[16 * R + n][base + 2 * p + h] = (half >> (3 * u)) & 7
        for h in range(2):
            code = 0
            for b in range(3):
                code |= ((ws[b] >> (16 * h + 15)) & 1) << b
            out[16 * R + n][base + 30 + h] = code
    return out


def decode_zeros(words, rows, NG):
    NGW = (NG + 7) // 8
    out = [[None] * NG for _ in range(rows)]
    for w, word in enumerate(int(v) for v in words):
        row, wq = divmod(w, NGW)
        for e in range(8):
            if 8 * wq + e < NG:
                out[row][8 * wq + e] = (word >> (4 * e)) & 0xF
    return out


def decode_scales(flat, rows, NG):
    return [[Fraction(float(flat[r * NG + q])) for q in range(NG)] for r in range(rows)]


def decode_f16(flat, rows, K):
    out = [[None] * K for _ in range(rows)]
    ntk = K // 32
    for idx, v in enumerate(flat):
        tl, i = divmod(idx, 8)
        tile, lane = divmod(tl, 64)
        R, g = divmod(tile, ntk)
        j, n = divmod(lane, 16)
        out[16 * R + n][32 * g + 8 * j + i] = Fraction(float(v))
    return out


def decode_sp24(values, indices, rows, K):
    """-> dense rows x K matrix of Fractions."""
    out = [[Fraction(0)] * K for _ in range(rows)]
    ntk = K // 128
    for w, word in enumerate(int(v) for v in indices):
        tile, lane = divmod(w, 64)
        R, g = divmod(tile, ntk)
        j, n = divmod(lane, 16)
        for s in range(2):
            for q in range(4):
                for v in range(2):
                    p = (word >> (16 * s + 4 * q + 2 * v)) & 3
                    val = values[tile * 1024 + s * 512 + lane * 8 + 2 * q + v]
                    out[16 * R + n][128 * g + 64 * s + 16 * j + 4 * q + p] = Fraction(float(val))
    return out


def decode_sp24q4(tiles, meta, rows, K):
    """-> dense rows x K matrix of Fractions, walking the stored words: the third word of a lane names the
    dense columns of its sixteen kept values, the first two hold their nibbles, the tile's meta word of
    the lane's row the scale and the zero-point."""
    import numpy as np
    out = [[Fraction(0)] * K for _ in range(rows)]
    ntk = K // 128
    for tl in range(len(tiles) // 3):
        tile, lane = divmod(tl, 64)
        R, g = divmod(tile, ntk)
        j, n = divmod(lane, 16)
        o = 16 * R + n
        m = int(meta[tile * 16 + n])
        scale = Fraction(float(np.array([m & 0xFFFF], dtype=np.uint16).view(np.float16)[0]))
        zero = (m >> 16) & 0xF
        word = int(tiles[3 * tl + 2])
        for s in range(2):
            cw = int(tiles[3 * tl + s])
            for q in range(4):
                for v in range(2):
                    p = (word >> (16 * s + 4 * q + 2 * v)) & 3
                    e = 2 * q + v
                    code = (cw >> (4 * (4 * (e % 2) + e // 2))) & 0xF
                    out[o][128 * g + 64 * s + 16 * j + 4 * q + p] = scale * (code - zero)
    return out


def exact_forward(x, What, A=None, B=None):
    """Exact rational y = x What^T + (x A^T) B^T; inputs are lists of Fractions."""
    M, K = len(x), len(x[0])
    N = len(What)
    y = [[sum(x[m][i] * What[o][i] for i in range(K)) for o in range(N)] for m in range(M)]
    if A is not None:
        r = len(A)
        t = [[sum(x[m][i] * A[p][i] for i in range(K)) for p in range(r)] for m in range(M)]
        for m in range(M):
            for o in range(N):
                y[m][o] += sum(t[m][p] * B[o][p] for p in range(r))
    return y


def frac_matrix(a):
    a = np.asarray(a)
    return [[Fraction(float(v)) for v in row] for row in a]
