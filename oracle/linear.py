"""Float64 forward pass of the compensated compressed linear layer.

Everything is computed in float64 with no intermediate rounding.  All stored
inputs (fp16 scales and values, small integers) are dyadic rationals, so the
dequantised weights are exact and the only rounding is float64 accumulation.

Row convention: x is M x d_in, What is d_out x d_in, A is r x d_in, B is
d_out x r, y is M x d_out.  The paper writes the same product in column
convention, What X + B' A X with X of shape d_in x M (Sec. 3, forward equation).
"""
import numpy as np

from . import layout


def dequant(codes, zeros, scales, group):
    """What[o][i] = s[o][i // group] * (q[o][i] - z[o][i // group]).

    Asymmetric uniform quantisation with an integer zero-point (Sec. 4.1:
    "asymmetric quantisation"; App. A.11: groups of 128 along the input dim).
    """
    q = np.asarray(codes).astype(np.float64)
    z = np.repeat(np.asarray(zeros).astype(np.float64), group, axis=1)
    s = np.repeat(np.asarray(scales, dtype=np.float16).astype(np.float64), group, axis=1)
    if q.shape != z.shape:
        raise ValueError("codes / zeros / group mismatch")
    return s * (q - z)


def dequant_q(qweight, qzeros, scales_packed, d_in, d_out, bits, group):
    """Packed quantised backbone -> float64 d_out x d_in."""
    NG = d_in // group
    if bits == 4:
        codes = layout.unpack_q4(qweight, d_out, d_in, 128)
    elif bits == 3:
        codes = layout.unpack_q3(qweight, d_out, d_in)
    elif bits == 2:
        codes = layout.unpack_q2(qweight, d_out, d_in)
    else:
        raise ValueError("bits must be 2, 3 or 4")
    zeros = layout.unpack_zeros(qzeros, d_out, NG)
    scales = layout.unpack_scales(scales_packed, d_out, NG)
    return dequant(codes, zeros, scales, group)


def dequant_factor_q4(qcodes_packed, scales_packed, rows, K):
    """4-bit EoRA factor (Sec. 4.5, quantised EoRA).  Symmetric: the zero-point
    is the constant 8; one fp16 scale per row and per group of min(128, K)
    columns along the contraction dimension."""
    KT = min(128, K)
    codes = layout.unpack_q4(qcodes_packed, rows, K, KT)
    scales = layout.unpack_scales(scales_packed, rows, K // KT)
    zeros = np.full((rows, K // KT), 8, dtype=np.uint8)
    return dequant(codes, zeros, scales, KT)


def dequant_factor_q3(qcodes_packed, scales_packed, rows, K):
    """3-bit EoRA factor (App. A.9 quantises the factors to 3 and 4 bits).  Symmetric: the zero-point is
    the constant 4; one fp16 scale per row and per group of 128 columns along the contraction dimension."""
    codes = layout.unpack_q3(qcodes_packed, rows, K)
    scales = layout.unpack_scales(scales_packed, rows, K // 128)
    zeros = np.full((rows, K // 128), 4, dtype=np.uint8)
    return dequant(codes, zeros, scales, 128)


def expand_sp24(vals, pos):
    """2:4 sparse -> dense float64: of every four consecutive input columns two
    are kept (Sec. 1), value v at column 4*group + position, the others zero."""
    vals = np.asarray(vals, dtype=np.float16).astype(np.float64)
    pos = np.asarray(pos).astype(np.int64)
    rows, half = vals.shape
    dense = np.zeros((rows, 2 * half), dtype=np.float64)
    col = 4 * (np.arange(half) // 2)[None, :] + pos
    dense[np.arange(rows)[:, None], col] = vals
    return dense


def expand_sp24_packed(values, indices, d_in, d_out):
    vals, pos = layout.unpack_sp24(values, indices, d_out, d_in)
    return expand_sp24(vals, pos)


def dequant_sp24q4(codes, pos, zeros, scales, group):
    """2:4 pruned, then quantised (the combined compression of Sec. 4.2): kept value u of row o lies at
    dense column c = 4*(u // 2) + pos and is s[o][c // group] * (q - z[o][c // group]); the pruned
    columns are zero."""
    q = np.asarray(codes).astype(np.float64)
    pos = np.asarray(pos).astype(np.int64)
    rows, half = q.shape
    col = 4 * (np.arange(half) // 2)[None, :] + pos
    grp = col // group
    r_idx = np.arange(rows)[:, None]
    z = np.asarray(zeros).astype(np.float64)[r_idx, grp]
    s = np.asarray(scales, dtype=np.float16).astype(np.float64)[r_idx, grp]
    dense = np.zeros((rows, 2 * half), dtype=np.float64)
    dense[r_idx, col] = s * (q - z)
    return dense


def dequant_sp24q4_packed(tiles, meta, d_in, d_out):
    """From the stored bytes: every tile carries its rows' scale and zero-point, i.e. groups of 128."""
    codes, pos, zeros, scales = layout.unpack_sp24q4(tiles, meta, d_out, d_in)
    return dequant_sp24q4(codes, pos, zeros, scales, 128)


def eora_linear(x, W_hat, A=None, B=None):
    """y = x What^T + (x A^T) B^T  (Sec. 3 forward equation; Alg. 1 step 7).

    A = B = None is the bare compressed layer (adapter switched off).
    """
    x = np.asarray(x).astype(np.float64)
    W_hat = np.asarray(W_hat, dtype=np.float64)
    y = x @ W_hat.T
    if A is not None:
        A = np.asarray(A).astype(np.float64)
        B = np.asarray(B).astype(np.float64)
        t = x @ A.T                      # M x r  down-projection
        y = y + t @ B.T                  # up-projection into the same output
    return y


def eora_linear_q(x, qweight, scales, qzeros, A, B, A_scales, B_scales,
                  M, d_in, d_out, r, w_bits, group, ab_bits):
    """Forward pass straight from the stored bytes (quantised backbone)."""
    x = np.asarray(x, dtype=np.float16).reshape(M, d_in)
    W_hat = dequant_q(qweight, qzeros, scales, d_in, d_out, w_bits, group)
    if r == 0:
        return eora_linear(x, W_hat)
    Ad, Bd = _factors(A, B, A_scales, B_scales, d_in, d_out, r, ab_bits)
    return eora_linear(x, W_hat, Ad, Bd)


def eora_linear_sp24(x, values, indices, A, B, M, d_in, d_out, r):
    """Forward pass straight from the stored bytes (2:4 sparse backbone)."""
    x = np.asarray(x, dtype=np.float16).reshape(M, d_in)
    W_hat = expand_sp24_packed(values, indices, d_in, d_out)
    if r == 0:
        return eora_linear(x, W_hat)
    Ad, Bd = _factors(A, B, None, None, d_in, d_out, r, 16)
    return eora_linear(x, W_hat, Ad, Bd)


def eora_linear_sp24q4(x, tiles, meta, A, B, M, d_in, d_out, r):
    """Forward pass straight from the stored bytes (2:4 sparse backbone with 4-bit kept values)."""
    x = np.asarray(x, dtype=np.float16).reshape(M, d_in)
    W_hat = dequant_sp24q4_packed(tiles, meta, d_in, d_out)
    if r == 0:
        return eora_linear(x, W_hat)
    Ad, Bd = _factors(A, B, None, None, d_in, d_out, r, 16)
    return eora_linear(x, W_hat, Ad, Bd)


def eora_linear_multi(x, W_hat, adapters, adapter_of_row):
    """One compressed backbone, several compensations: token row m gets
    y[m] = x[m] What^T + (x[m] A_a^T) B_a^T with a = adapter_of_row[m], and the bare
    y[m] = x[m] What^T for a = -1.

    The compensation is a separate residual path that never alters What (Sec. 1, Sec. 3), so
    requests with different (B', A) pairs, or none, can share one batch; row by row this is the
    forward equation of Sec. 3 with that row's pair.  adapters: list of (A, B).
    """
    x = np.asarray(x).astype(np.float64)
    W_hat = np.asarray(W_hat, dtype=np.float64)
    y = np.empty((x.shape[0], W_hat.shape[0]), dtype=np.float64)
    for m in range(x.shape[0]):
        a = int(adapter_of_row[m])
        if a < -1 or a >= len(adapters):
            raise ValueError("adapter index out of range")
        y[m] = W_hat @ x[m]
        if a >= 0:
            A = np.asarray(adapters[a][0]).astype(np.float64)
            B = np.asarray(adapters[a][1]).astype(np.float64)
            y[m] += B @ (A @ x[m])
    return y


def eora_linear_q_multi(x, qweight, scales, qzeros, A_all, B_all, A_scales, B_scales, adapter_of_row,
                        M, d_in, d_out, r, n_adapters, w_bits, group, ab_bits):
    """The same from stored bytes: A_all holds the adapters' A stacked by rows (n_adapters*r x d_in),
    B_all their B side by side (d_out x n_adapters*r), each packed as one factor."""
    x = np.asarray(x, dtype=np.float16).reshape(M, d_in)
    W_hat = dequant_q(qweight, qzeros, scales, d_in, d_out, w_bits, group)
    R = n_adapters * r
    Ad, Bd = _factors(A_all, B_all, A_scales, B_scales, d_in, d_out, R, ab_bits)
    adapters = [(Ad[a * r:(a + 1) * r], Bd[:, a * r:(a + 1) * r]) for a in range(n_adapters)]
    return eora_linear_multi(x, W_hat, adapters, adapter_of_row)


def _factors(A, B, A_scales, B_scales, d_in, d_out, r, ab_bits):
    if ab_bits == 16:
        return layout.unpack_f16(A, r, d_in), layout.unpack_f16(B, d_out, r)
    if ab_bits == 4:
        return (dequant_factor_q4(A, A_scales, r, d_in),
                dequant_factor_q4(B, B_scales, d_out, r))
    if ab_bits == 3:
        return (dequant_factor_q3(A, A_scales, r, d_in),
                dequant_factor_q3(B, B_scales, d_out, r))
    raise ValueError("ab_bits must be 16, 4 or 3")


def y_error(y_test, y_ref):
    """The comparison rule for y: max |y_test - y_ref| / max(|y_ref|, rms(y_ref)).

    Pure element-wise relative error is undefined where a sum of thousands of
    signed terms cancels to ~0, so the denominator is floored at the rms of the
    reference output."""
    y_ref = np.asarray(y_ref, dtype=np.float64)
    y_test = np.asarray(y_test).astype(np.float64)
    rms = np.sqrt(np.mean(y_ref ** 2)) if y_ref.size else 0.0
    den = np.maximum(np.abs(y_ref), rms)
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(y_test - y_ref) / den)) if y_ref.size else 0.0
