"""Pins for oracle/calibrate.py (Alg. 1 steps 1-6, Theorem 1)."""
import numpy as np

from oracle import calibrate, linear


def _setup(d=24, k=40, n=200, seed=0):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((d, k))
    W_hat = W + 0.1 * rng.standard_normal((d, k))
    scale = np.exp(rng.uniform(-2, 2, k))              # very uneven channel energies
    Xt = rng.standard_normal((k, n)) * scale[:, None]
    return W, W_hat, Xt


def test_planted_rank_r_error_is_recovered():
    rng = np.random.default_rng(1)
    d, k, r = 24, 40, 5
    W_hat = rng.standard_normal((d, k))
    W = W_hat + rng.standard_normal((d, r)) @ rng.standard_normal((r, k))
    Xt = rng.standard_normal((k, 120))
    Bp, A = calibrate.eora_factors(W, W_hat, Xt, r)
    assert Bp.shape == (d, r) and A.shape == (r, k)
    assert np.linalg.norm(Bp @ A - (W - W_hat)) <= 1e-9 * np.linalg.norm(W - W_hat)
    # forward pass with the compensated layer reproduces the uncompressed layer
    x = rng.standard_normal((7, k))
    assert np.allclose(linear.eora_linear(x, W_hat, A, Bp), x @ W.T, rtol=1e-9, atol=1e-9)


def test_identity_gram_reduces_to_plain_svd():
    """Orthonormal rows of Xt (Xt Xt^T = I) make the projection trivial: the product
    B'A equals the truncated SVD of the raw error (Sec. 2, Eq. 2)."""
    rng = np.random.default_rng(2)
    W, W_hat, _ = _setup(seed=2)
    k = W.shape[1]
    Qo, _ = np.linalg.qr(rng.standard_normal((100, k)))
    Xt = Qo.T                                            # k x 100, Xt Xt^T = I
    Bp, A = calibrate.eora_factors(W, W_hat, Xt, 6)
    Bs, As = calibrate.plain_svd_factors(W, W_hat, 6)
    assert np.allclose(Bp @ A, Bs @ As, atol=1e-10)


def test_residual_loss_closed_form_theorem1():
    """|| dW Xt - B'A Xt ||_F = sqrt(sum_{i>r} sigma'_i^2), sigma' the singular values
    of dW Q' (Theorem 1 with Eckart-Young)."""
    W, W_hat, Xt = _setup(seed=3)
    r = 7
    Bp, A = calibrate.eora_factors(W, W_hat, Xt, r)
    lam, Q = np.linalg.eigh(Xt @ Xt.T)
    sig = np.linalg.svd((W - W_hat) @ (Q * np.sqrt(lam)[None, :]), compute_uv=False)
    want = np.sqrt(np.sum(sig[r:] ** 2))
    assert np.isclose(calibrate.layer_loss(W, W_hat, Bp, A, Xt), want, rtol=1e-9)


def test_not_worse_than_plain_svd_or_activation_scaling():
    """The eigenspace projection minimises the layer-wise loss among rank-r
    compensations (Theorem 1), so it cannot lose to plain SVD (Eq. 2) or to the
    diagonal activation scaling baseline of Sec. 4.1."""
    for seed in range(4):
        W, W_hat, Xt = _setup(seed=10 + seed)
        r = 5
        Bp, A = calibrate.eora_factors(W, W_hat, Xt, r)
        e = calibrate.layer_loss(W, W_hat, Bp, A, Xt)
        Bs, As = calibrate.plain_svd_factors(W, W_hat, r)
        assert e <= calibrate.layer_loss(W, W_hat, Bs, As, Xt) * (1 + 1e-12)
        S = np.sqrt(np.mean(np.abs(Xt), axis=1))
        U, sg, Vt = np.linalg.svd((W - W_hat) * S[None, :], full_matrices=False)
        Ba, Aa = U[:, :r] * sg[None, :r], Vt[:r] / S[None, :]
        assert e <= calibrate.layer_loss(W, W_hat, Ba, Aa, Xt) * (1 + 1e-12)
        # random rank-r perturbation of the optimum is never better
        rng = np.random.default_rng(seed)
        assert e <= calibrate.layer_loss(W, W_hat, Bp + 1e-3 * rng.standard_normal(Bp.shape), A, Xt)


def test_gram_scaling_invariance_and_projection_inverse():
    W, W_hat, Xt = _setup(seed=5)
    B1, A1 = calibrate.eora_factors(W, W_hat, Xt, 6)
    B2, A2 = calibrate.eora_factors(W, W_hat, 37.0 * Xt, 6)
    assert np.allclose(B1 @ A1, B2 @ A2, atol=1e-9)
    lam, Q = np.linalg.eigh(calibrate.gram(Xt))
    Qp = Q * np.sqrt(lam)[None, :]
    Qp_inv = (Q / np.sqrt(lam)[None, :]).T              # sqrt(Lambda)^-1 Q^T
    assert np.allclose(Qp @ Qp_inv, np.eye(Q.shape[0]), atol=1e-9)
    assert np.allclose(Qp @ Qp.T, calibrate.gram(Xt), rtol=1e-9, atol=1e-9)


def test_full_rank_compensation_is_exact():
    W, W_hat, Xt = _setup(d=12, k=20, seed=6)
    Bp, A = calibrate.eora_factors(W, W_hat, Xt, 12)
    assert np.allclose(Bp @ A, W - W_hat, atol=1e-9)


def test_balanced_factors_keep_the_product_and_share_the_norm():
    rng = np.random.default_rng(30)
    B = rng.standard_normal((24, 6)) * np.array([1e3, 1.0, 1e-3, 5.0, 0.0, 2.0])[None, :]
    A = rng.standard_normal((6, 40)) * np.array([1e-2, 1.0, 1e4, 0.1, 1.0, 0.0])[:, None]
    Bb, Ab = calibrate.balance_factors(B, A)
    assert np.abs(Bb @ Ab - B @ A).max() <= 1e-13 * np.abs(B @ A).max()
    nb, na = np.linalg.norm(Bb, axis=0), np.linalg.norm(Ab, axis=1)
    want = np.sqrt(np.linalg.norm(B, axis=0) * np.linalg.norm(A, axis=1))
    live = [0, 1, 2, 3]
    assert np.allclose(nb[live], want[live], rtol=1e-13) and np.allclose(na[live], want[live], rtol=1e-13)
    # a component with a zero factor is left alone
    assert np.array_equal(Bb[:, 4:], B[:, 4:]) and np.array_equal(Ab[4:], A[4:])


def test_stored_factors_are_the_fp16_rounding_in_tile_order():
    from oracle import layout
    rng = np.random.default_rng(31)
    B, A = rng.standard_normal((32, 32)) * 50.0, rng.standard_normal((32, 64)) * 1e-3
    At, Bt = calibrate.store_factors_f16(B, A, balance=False)
    assert np.array_equal(layout.unpack_f16(At, 32, 64), A.astype(np.float16))
    assert np.array_equal(layout.unpack_f16(Bt, 32, 32), B.astype(np.float16))
    At, Bt = calibrate.store_factors_f16(B, A)
    P = layout.unpack_f16(Bt, 32, 32).astype(np.float64) @ layout.unpack_f16(At, 32, 64).astype(np.float64)
    assert np.abs(P - B @ A).max() <= 2e-3 * np.abs(B @ A).max()          # two fp16 roundings per product term
    # without balancing the small factor would sit in fp16's subnormal range; with it both are near 0.2
    assert np.abs(layout.unpack_f16(At, 32, 64)).max() > 0.05


def test_factor_quantiser_hand_values_and_error_bound():
    # fp16(0.7 / 7) = 0.0999755859375: 0.7 -> +7 -> code 15; -0.35 -> -3.5009 -> -4 -> code 4; 0.1 -> +1 -> code 9
    row = np.zeros((1, 128))
    row[0, :3] = [0.7, -0.35, 0.1]
    codes, scales = calibrate.quantize_factor(row, 4)
    assert float(scales[0, 0]) == 0.0999755859375
    assert list(codes[0, :4]) == [15, 4, 9, 8]
    # 3 bits: fp16(0.7 / 3) = 1911 * 2^-13 = 0.2332763671875: 0.7 -> 3.0007 -> +3 -> code 7; -0.35 -> -1.5004 -> -2 -> code 2;
    # 0.1 -> 0.43 -> 0 -> code 4
    codes, scales = calibrate.quantize_factor(row, 3)
    assert float(scales[0, 0]) == 0.2332763671875 and list(codes[0, :4]) == [7, 2, 4, 4]
    # an all-zero group gets scale 1 and the zero-point everywhere
    codes, scales = calibrate.quantize_factor(np.zeros((2, 256)), 4)
    assert np.all(scales == 1) and np.all(codes == 8)
    rng = np.random.default_rng(32)
    for bits, zp in ((4, 8), (3, 4)):
        M = rng.standard_normal((16, 256)) * np.exp(rng.uniform(-3, 3, (16, 1)))
        codes, scales = calibrate.quantize_factor(M, bits)
        assert codes.min() >= 1 and codes.max() <= 2 * zp - 1
        back = (codes.astype(np.float64) - zp) * np.repeat(scales.astype(np.float64), 128, axis=1)
        # half a step, plus the fp16 rounding of the scale on the largest magnitude (qpos steps of 2^-11 each)
        assert np.all(np.abs(back - M) <= np.repeat(scales.astype(np.float64), 128, axis=1) * (0.5 + 0.004))


def test_stored_quantised_factors_dequantise_to_the_quantiser_values():
    from oracle import linear
    rng = np.random.default_rng(33)
    B, A = rng.standard_normal((32, 128)) * 3.0, rng.standard_normal((128, 256)) * 1e-2
    for bits, deq in ((4, linear.dequant_factor_q4), (3, linear.dequant_factor_q3)):
        Aq, As, Bq, Bs = calibrate.store_factors_q(B, A, bits, balance=False)
        ca, sa = calibrate.quantize_factor(A, bits)
        zp = 1 << (bits - 1)
        want = (ca.astype(np.float64) - zp) * np.repeat(sa.astype(np.float64), 128, axis=1)
        assert np.array_equal(deq(Aq, As, 128, 256), want)
        cb, sb = calibrate.quantize_factor(B, bits)
        want_b = (cb.astype(np.float64) - zp) * np.repeat(sb.astype(np.float64), 128, axis=1)
        assert np.array_equal(deq(Bq, Bs, 32, 128), want_b)
        # B is quantised along the rank: its largest entry of a row is hit exactly by the top code (|code - zp| = qpos)
        assert np.all(np.abs(cb.astype(np.int64) - zp).max(axis=1) == zp - 1)
        assert np.max(np.abs(want_b - B)) <= float(sb.max()) * 0.504
    # rank 64 with 4 bits: B's groups are 64 columns wide (one scale per row), stored as 64-column tiles
    B64, A64 = rng.standard_normal((32, 64)) * 0.5, rng.standard_normal((64, 256)) * 0.1
    Aq, As, Bq, Bs = calibrate.store_factors_q(B64, A64, 4, balance=False)
    cb, sb = calibrate.quantize_factor(B64, 4)
    assert sb.shape == (32, 1) and np.asarray(Bs).size == 32
    want_b = (cb.astype(np.float64) - 8) * sb.astype(np.float64)
    assert np.array_equal(linear.dequant_factor_q4(Bq, Bs, 32, 64), want_b)
    # hand value: row of B64 with largest magnitude m gets scale fp16(m / 7) and that entry the code 8 +- 7
    i, j = np.unravel_index(np.argmax(np.abs(B64)), B64.shape)
    assert float(sb[i, 0]) == float(np.float16(abs(B64[i, j]) / 7)) and cb[i, j] == (15 if B64[i, j] > 0 else 1)


def test_any_square_root_of_the_gram_matrix_gives_the_same_factors():
    """What the library's Cholesky route rests on (Alg. 1 steps 2-6): with S S^T = X~ X~^T for ANY square S, not only
    S = Q sqrt(Lambda), the matrix dW S is dW Q sqrt(Lambda) times an orthogonal factor on the right, so its left
    singular vectors and singular values are those of step 5, and step 6's A' (S)^-1 is Sigma'^-1 U'^T dW.  Checked
    with the Cholesky factor and with a randomly rotated square root, against the oracle's own route."""
    for d, k in ((24, 40), (40, 24)):
        W, W_hat, Xt = _setup(d=d, k=k, n=300, seed=3)
        r = 6
        Bo, Ao = calibrate.eora_factors(W, W_hat, Xt, r)
        dW = W - W_hat
        G = calibrate.gram(Xt)
        rot, _ = np.linalg.qr(np.random.default_rng(4).standard_normal((k, k)))
        for S in (np.linalg.cholesky(G), np.linalg.cholesky(G) @ rot):
            assert np.allclose(S @ S.T, G, rtol=1e-10, atol=1e-10 * np.abs(G).max())
            U, sig, _ = np.linalg.svd(dW @ S, full_matrices=False)
            B = U[:, :r] * sig[None, :r]
            A = (U[:, :r] / sig[None, :r]).T @ dW
            assert np.allclose(sig[:r], np.linalg.norm(Bo, axis=0), rtol=1e-9)
            assert np.abs(B @ A - Bo @ Ao).max() <= 1e-9 * np.abs(Bo @ Ao).max()
            sign = np.sign(np.sum(B * Bo, axis=0))
            assert np.abs(B * sign[None, :] - Bo).max() <= 1e-8 * np.abs(Bo).max()
            assert np.abs(A * sign[:, None] - Ao).max() <= 1e-8 * np.abs(Ao).max()


def test_square_factor_of_step5_has_the_same_singular_values_and_left_vectors():
    """What the library's shortening of step 5 rests on: for T (m x n, m <= n, full row rank) and the Cholesky factor
    C of T T^T, the matrix C has T's singular values and left singular vectors w_i, and w_i^T T = sigma_i z_i^T with
    z_i the right singular vectors of T."""
    rng = np.random.default_rng(11)
    m, n, r = 12, 40, 4
    T = rng.standard_normal((m, n)) * np.exp(rng.uniform(-1, 1, m))[:, None]
    C = np.linalg.cholesky(T @ T.T)
    Uc, sc, _ = np.linalg.svd(C)
    Ut, st, Vt = np.linalg.svd(T, full_matrices=False)
    assert np.allclose(sc, st, rtol=1e-10)
    sign = np.sign(np.sum(Uc * Ut, axis=0))
    assert np.allclose(Uc * sign[None, :], Ut, atol=1e-8)
    rows = (Uc[:, :r] * sign[None, :r]).T @ T
    assert np.allclose(rows, st[:r, None] * Vt[:r], atol=1e-9 * st[0])
