"""Pins for oracle/linear.py (forward pass of Sec. 3 / Alg. 1 step 7)."""
from fractions import Fraction

import numpy as np
import pytest

import synth
from oracle import layout, linear
from tests import pyref
from tests.golden_io import read_dequant


def test_dequant_hand_values():
    # values written out by hand in tests/golden/dequant.txt
    for s, z, codes, want in read_dequant():
        n = len(codes)
        pad = 128 - n
        q = np.array([codes + [z] * pad], np.uint8)
        got = linear.dequant(q, np.array([[z]], np.uint8), np.array([[s]], np.float16), 128)
        assert np.array_equal(got[0, :n], np.array(want))
        assert np.all(got[0, n:] == 0.0)


def _tiny_q(bits, rows=16, K=256, M=3, r=32, seed=0, ab_bits=16):
    W, A, B, x = synth.draw_layer(seed, K, rows, M, r)
    codes, zeros, scales = synth.quantize_rtn(W, bits, 128)
    qw = {4: layout.pack_q4, 3: layout.pack_q3, 2: layout.pack_q2}[bits](codes)
    qz, sc = layout.pack_zeros(zeros), layout.pack_scales(scales)
    if ab_bits == 16:
        Ap, Bp, As, Bs = layout.pack_f16(A), layout.pack_f16(B), None, None
    elif ab_bits == 3:
        ca, sa = synth.quantize_sym3(A)
        cb, sb = synth.quantize_sym3(B)
        Ap, As = layout.pack_q3(ca), layout.pack_scales(sa)
        Bp, Bs = layout.pack_q3(cb), layout.pack_scales(sb)
    else:
        KTb = min(128, r)
        ca, sa = synth.quantize_sym4(A, 128)
        cb, sb = synth.quantize_sym4(B, KTb)
        Ap, As = layout.pack_q4(ca, 128), layout.pack_scales(sa)
        Bp, Bs = layout.pack_q4(cb, KTb), layout.pack_scales(sb)
    return dict(x=x, qw=qw, qz=qz, sc=sc, A=Ap, B=Bp, As=As, Bs=Bs, rows=rows, K=K, M=M, r=r, bits=bits,
                ab_bits=ab_bits, logical=(codes, zeros, scales, A, B))


@pytest.mark.parametrize("bits,ab_bits,r", [(4, 16, 32), (3, 16, 32), (4, 4, 64), (3, 4, 128), (2, 16, 32), (4, 3, 128)])
def test_forward_exact_rational(bits, ab_bits, r):
    """All stored inputs are dyadic rationals, so y is computable exactly with
    Fractions from the raw words, by decoders that share nothing with the oracle."""
    d = _tiny_q(bits, rows=16, K=128 if r != 128 else 256, M=2, r=r, seed=bits * 10 + r, ab_bits=ab_bits)
    rows, K, M = d["rows"], d["K"], d["M"]
    y = linear.eora_linear_q(d["x"], d["qw"], d["sc"], d["qz"], d["A"], d["B"], d["As"], d["Bs"],
                             M, K, rows, r, bits, 128, ab_bits)
    NG = K // 128
    q = {4: pyref.decode_q4, 3: pyref.decode_q3, 2: pyref.decode_q2}[bits](d["qw"], rows, K)
    z = pyref.decode_zeros(d["qz"], rows, NG)
    s = pyref.decode_scales(d["sc"], rows, NG)
    What = [[s[o][i // 128] * (q[o][i] - z[o][i // 128]) for i in range(K)] for o in range(rows)]
    if ab_bits == 16:
        Af, Bf = pyref.decode_f16(d["A"], r, K), pyref.decode_f16(d["B"], rows, r)
    elif ab_bits == 3:
        qa, sa = pyref.decode_q3(d["A"], r, K), pyref.decode_scales(d["As"], r, K // 128)
        qb, sb = pyref.decode_q3(d["B"], rows, r), pyref.decode_scales(d["Bs"], rows, r // 128)
        Af = [[sa[p][i // 128] * (qa[p][i] - 4) for i in range(K)] for p in range(r)]
        Bf = [[sb[o][p // 128] * (qb[o][p] - 4) for p in range(r)] for o in range(rows)]
    else:
        KTb = min(128, r)
        qa, sa = pyref.decode_q4(d["A"], r, K), pyref.decode_scales(d["As"], r, K // 128)
        qb, sb = pyref.decode_q4(d["B"], rows, r, KTb), pyref.decode_scales(d["Bs"], rows, r // KTb)
        Af = [[sa[p][i // 128] * (qa[p][i] - 8) for i in range(K)] for p in range(r)]
        Bf = [[sb[o][p // KTb] * (qb[o][p] - 8) for p in range(r)] for o in range(rows)]
    exact = pyref.exact_forward(pyref.frac_matrix(d["x"]), What, Af, Bf)
    for m in range(M):
        for o in range(rows):
            e = exact[m][o]
            assert abs(Fraction(float(y[m, o])) - e) <= abs(e) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 15)


def test_sparse_forward_exact_rational():
    W, A, B, x = synth.draw_layer(3, 128, 16, 2, 32)
    vals, pos = synth.prune_24(W.astype(np.float16))
    values, indices = layout.pack_sp24(vals, pos)
    y = linear.eora_linear_sp24(x, values, indices, layout.pack_f16(A), layout.pack_f16(B), 2, 128, 16, 32)
    What = pyref.decode_sp24(values, indices, 16, 128)
    exact = pyref.exact_forward(pyref.frac_matrix(x), What, pyref.frac_matrix(A), pyref.frac_matrix(B))
    for m in range(2):
        for o in range(16):
            e = exact[m][o]
            assert abs(Fraction(float(y[m, o])) - e) <= abs(e) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 15)


def test_sparse_quantised_forward_exact_rational():
    W, A, B, x = synth.draw_layer(4, 256, 16, 2, 32)
    vals, pos = synth.prune_24(W.astype(np.float16))
    codes, zeros, scales = synth.quantize_kept_rtn(vals, pos, 128)
    tiles, meta = layout.pack_sp24q4(codes, pos, zeros, scales, 128)
    y = linear.eora_linear_sp24q4(x, tiles, meta, layout.pack_f16(A), layout.pack_f16(B), 2, 256, 16, 32)
    What = pyref.decode_sp24q4(tiles, meta, 16, 256)
    exact = pyref.exact_forward(pyref.frac_matrix(x), What, pyref.frac_matrix(A), pyref.frac_matrix(B))
    for m in range(2):
        for o in range(16):
            e = exact[m][o]
            assert abs(Fraction(float(y[m, o])) - e) <= abs(e) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 15)
    # the quantiser keeps every kept value within half a step of its code (a property of the generator)
    Wd = linear.dequant_sp24q4(codes, pos, zeros, scales, 128)
    step = np.repeat(scales.astype(np.float64), 128, axis=1)
    assert np.all(np.abs(Wd - linear.expand_sp24(vals, pos)) <= 0.5 * step + 1e-12)


@pytest.mark.parametrize("bits", [3, 4])
def test_zero_factors_equal_bare_layer(bits):
    d = _tiny_q(bits, rows=32, K=256, M=4, r=32, seed=7)
    z16 = np.zeros(32 * 256, np.float16)
    zB = np.zeros(32 * 32, np.float16)
    y0 = linear.eora_linear_q(d["x"], d["qw"], d["sc"], d["qz"], None, None, None, None, 4, 256, 32, 0, bits, 128, 16)
    y1 = linear.eora_linear_q(d["x"], d["qw"], d["sc"], d["qz"], z16, zB, None, None, 4, 256, 32, 32, bits, 128, 16)
    assert np.array_equal(y0, y1)


def test_planted_exact_rank_r_reproduces_W():
    """Integer-valued What, A, B, x: W = What + B A is an exact integer matrix and
    every product and sum is exact in float64, so the compensated layer must equal
    x W^T bit for bit, computed here with int64 numpy."""
    rng = np.random.default_rng(21)
    rows, K, r, M = 32, 256, 32, 5
    codes = rng.integers(0, 16, (rows, K), dtype=np.uint8)
    zeros = rng.integers(0, 16, (rows, K // 128), dtype=np.uint8)
    scales = np.full((rows, K // 128), 2.0, np.float16)          # integer scale
    A = rng.integers(-3, 4, (r, K)).astype(np.float16)
    B = rng.integers(-3, 4, (rows, r)).astype(np.float16)
    x = rng.integers(-4, 5, (M, K)).astype(np.float16)
    What_i = 2 * (codes.astype(np.int64) - np.repeat(zeros.astype(np.int64), 128, axis=1))
    W_i = What_i + B.astype(np.int64) @ A.astype(np.int64)
    want = x.astype(np.int64) @ W_i.T
    y = linear.eora_linear_q(x, layout.pack_q4(codes), layout.pack_scales(scales), layout.pack_zeros(zeros),
                             layout.pack_f16(A), layout.pack_f16(B), None, None, M, K, rows, r, 4, 128, 16)
    assert np.array_equal(y, want.astype(np.float64))
    # and the bare layer differs by exactly the low-rank term
    y0 = linear.eora_linear_q(x, layout.pack_q4(codes), layout.pack_scales(scales), layout.pack_zeros(zeros),
                              None, None, None, None, M, K, rows, 0, 4, 128, 16)
    assert np.array_equal(y - y0, (x.astype(np.int64) @ A.astype(np.int64).T @ B.astype(np.int64).T).astype(np.float64))


def test_group_identity():
    """x What^T = sum_groups s_g (sum_{i in g} q_i x_i - z_g sum_{i in g} x_i)."""
    d = _tiny_q(4, rows=16, K=384, M=3, r=0, seed=9)
    codes, zeros, scales, _, _ = d["logical"]
    y = linear.eora_linear_q(d["x"], d["qw"], d["sc"], d["qz"], None, None, None, None, 3, 384, 16, 0, 4, 128, 16)
    x = d["x"].astype(np.float64).reshape(3, 3, 128)
    q = codes.astype(np.float64).reshape(16, 3, 128)
    qx = np.einsum("mgi,ogi->mog", x, q)
    sx = x.sum(axis=2)
    alt = np.einsum("og,mog->mo", scales.astype(np.float64), qx - zeros.astype(np.float64)[None] * sx[:, None, :])
    assert np.allclose(y, alt, rtol=1e-12, atol=1e-12)


def test_channelwise_group_equals_replicated_group128():
    """group = d_in (the paper's main-text channel-wise setting, Sec. 4.1) equals
    group 128 with the scale / zero repeated."""
    rng = np.random.default_rng(4)
    rows, K = 16, 256
    codes = rng.integers(0, 16, (rows, K), dtype=np.uint8)
    z1 = rng.integers(0, 16, (rows, 1), dtype=np.uint8)
    s1 = rng.uniform(0.01, 0.1, (rows, 1)).astype(np.float16)
    x = rng.standard_normal((2, K)).astype(np.float16)
    qw = layout.pack_q4(codes)
    ya = linear.eora_linear_q(x, qw, layout.pack_scales(s1), layout.pack_zeros(z1), None, None, None, None,
                              2, K, rows, 0, 4, K, 16)
    yb = linear.eora_linear_q(x, qw, layout.pack_scales(np.repeat(s1, 2, 1)), layout.pack_zeros(np.repeat(z1, 2, 1)),
                              None, None, None, None, 2, K, rows, 0, 4, 128, 16)
    assert np.array_equal(ya, yb)


def test_quantised_factors_equal_their_dequantised_fp_path():
    d = _tiny_q(4, rows=32, K=256, M=2, r=64, seed=13, ab_bits=4)
    y = linear.eora_linear_q(d["x"], d["qw"], d["sc"], d["qz"], d["A"], d["B"], d["As"], d["Bs"],
                             2, 256, 32, 64, 4, 128, 4)
    Ad = linear.dequant_factor_q4(d["A"], d["As"], 64, 256)
    Bd = linear.dequant_factor_q4(d["B"], d["Bs"], 32, 64)
    W_hat = linear.dequant_q(d["qw"], d["qz"], d["sc"], 256, 32, 4, 128)
    assert np.array_equal(y, linear.eora_linear(d["x"], W_hat, Ad, Bd))
    # symmetric: code 8 is exactly zero, range is [-7s, 7s]
    ca, sa = synth.quantize_sym4(d["logical"][3], 128)
    assert ca.min() >= 1 and ca.max() <= 15
    assert np.all(np.abs(Ad) <= 7 * np.repeat(sa.astype(np.float64), 128, axis=1))


def test_linearity_and_row_independence():
    d = _tiny_q(3, rows=16, K=256, M=4, r=32, seed=17)
    f = lambda x, M: linear.eora_linear_q(x, d["qw"], d["sc"], d["qz"], d["A"], d["B"], None, None,
                                          M, 256, 16, 32, 3, 128, 16)
    y = f(d["x"], 4)
    for m in range(4):
        assert np.array_equal(f(d["x"][m:m + 1], 1)[0], y[m])
    assert np.allclose(f((2 * d["x"].astype(np.float32)).astype(np.float16), 4), 2 * y, rtol=1e-13)


def test_y_error_rule():
    ref = np.array([[1.0, -2.0, 0.0, 4.0]])
    rms = np.sqrt(21 / 4)
    got = ref + np.array([[0.1, 0.0, 0.2, 0.0]])
    assert np.isclose(linear.y_error(got, ref), 0.2 / rms)   # the zero entry is floored at rms
    assert linear.y_error(ref, ref) == 0.0


# ---------------------------------------------------------------- several adapters over one backbone
def _multi_setup(seed, d_in=256, d_out=32, M=9, r=32, n=3):
    rng = np.random.default_rng(seed)
    W_hat = rng.integers(-7, 8, (d_out, d_in)).astype(np.float64)
    ads = [(rng.integers(-3, 4, (r, d_in)).astype(np.float64), rng.integers(-3, 4, (d_out, r)).astype(np.float64))
           for _ in range(n)]
    x = rng.integers(-4, 5, (M, d_in)).astype(np.float64)
    sel = rng.integers(-1, n, M)
    sel[0], sel[1] = -1, n - 1                      # both ends of the range are present
    return W_hat, ads, x, sel


def test_multi_adapter_exact_rational_brute_force():
    """Integer-valued operands: every row's result is an exact integer, computed here with Python
    integers element by element from the per-row definition."""
    W_hat, ads, x, sel = _multi_setup(40, d_in=24, d_out=5, M=6, r=3, n=3)
    got = linear.eora_linear_multi(x, W_hat, ads, sel)
    for m in range(x.shape[0]):
        for o in range(W_hat.shape[0]):
            want = sum(int(W_hat[o, i]) * int(x[m, i]) for i in range(x.shape[1]))
            if sel[m] >= 0:
                A, B = ads[sel[m]]
                for k in range(A.shape[0]):
                    t = sum(int(A[k, i]) * int(x[m, i]) for i in range(x.shape[1]))
                    want += int(B[o, k]) * t
            assert got[m, o] == want


def test_multi_adapter_special_cases():
    W_hat, ads, x, sel = _multi_setup(41)
    M, n = x.shape[0], len(ads)
    # one adapter for every row is the single-adapter layer; none is the bare layer
    for a in range(n):
        assert np.array_equal(linear.eora_linear_multi(x, W_hat, ads, np.full(M, a)), linear.eora_linear(x, W_hat, *ads[a]))
    assert np.array_equal(linear.eora_linear_multi(x, W_hat, ads, np.full(M, -1)), linear.eora_linear(x, W_hat))
    # rows are independent: a row's result depends on its own selection only
    full = linear.eora_linear_multi(x, W_hat, ads, sel)
    for m in range(M):
        one = linear.eora_linear_multi(x[m:m + 1], W_hat, ads, sel[m:m + 1])
        assert np.array_equal(one[0], full[m])
    with pytest.raises(ValueError):
        linear.eora_linear_multi(x, W_hat, ads, np.full(M, n))


def test_multi_adapter_equals_masked_stacked_factors():
    """Stacking the A's by rows and the B's side by side, and zeroing in t = x A_all^T every column that
    does not belong to the row's adapter, is the same map (the identity the GPU path is built on)."""
    W_hat, ads, x, sel = _multi_setup(42)
    r = ads[0][0].shape[0]
    A_all = np.vstack([A for A, _ in ads])
    B_all = np.hstack([B for _, B in ads])
    t = x @ A_all.T
    mask = (np.arange(A_all.shape[0])[None, :] // r) == sel[:, None]
    want = x @ W_hat.T + (t * mask) @ B_all.T
    assert np.array_equal(linear.eora_linear_multi(x, W_hat, ads, sel), want)


def test_multi_adapter_from_stored_bytes():
    d_in, d_out, M, r, n = 256, 32, 5, 32, 2
    W, _, _, x = synth.draw_layer(43, d_in, d_out, M, 0)
    codes, zeros, scales = synth.quantize_rtn(W, 4, 128)
    qw, qz, sc = layout.pack_q4(codes), layout.pack_zeros(zeros), layout.pack_scales(scales)
    rng = np.random.default_rng(44)
    As = [(rng.standard_normal((r, d_in)) * 0.01).astype(np.float16) for _ in range(n)]
    Bs = [(rng.standard_normal((d_out, r)) * 0.01).astype(np.float16) for _ in range(n)]
    sel = np.array([1, -1, 0, 0, 1])
    got = linear.eora_linear_q_multi(x, qw, sc, qz, layout.pack_f16(np.vstack(As)), layout.pack_f16(np.hstack(Bs)), None, None,
                                     sel, M, d_in, d_out, r, n, 4, 128, 16)
    W_hat = linear.dequant(codes, zeros, scales, 128)
    for m in range(M):
        want = linear.eora_linear(x[m:m + 1], W_hat, *((As[sel[m]], Bs[sel[m]]) if sel[m] >= 0 else (None, None)))
        assert np.allclose(got[m], want[0], rtol=1e-13, atol=1e-15)
