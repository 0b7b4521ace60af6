"""Algorithm 1, steps 1-6: eigenspace low-rank approximation of the compression error.

Offline and not part of the GPU hot path; kept in the oracle because (a) it
pins the forward pass on planted errors (What + B'A must reproduce W) and (b) it
is the next step outside the hot path.  float64 numpy throughout.

Paper notation (column convention): W, What are d x k; Xt (X-tilde) is k x n;
Q, Lambda from the eigendecomposition of Xt Xt^T; Q' = Q sqrt(Lambda);
dW' = dW Q'; rank-r SVD of dW' gives B' = U' Sigma', A' = V'^T; A = A' Q'^-1.
"""
import numpy as np


def gram(Xt):
    """Xt Xt^T (k x k), Sec. 3.  Any positive rescaling of it leaves B'A unchanged."""
    Xt = np.asarray(Xt, dtype=np.float64)
    return Xt @ Xt.T


def eora_factors(W, W_hat, Xt, r, eig_floor=1e-12):
    """Return (B', A) with B' of shape d x r and A of shape r x k.

    eig_floor: eigenvalues are clamped to eig_floor * max eigenvalue before the
    inverse square root, since the paper assumes Q' invertible without treating
    zero eigenvalues (Sec. 3); with full-rank calibration activations the clamp
    is inactive.
    """
    W = np.asarray(W, dtype=np.float64)
    W_hat = np.asarray(W_hat, dtype=np.float64)
    dW = W - W_hat                                   # step 1
    lam, Q = np.linalg.eigh(gram(Xt))                # step 2
    lam = np.maximum(lam, eig_floor * lam.max())
    root = np.sqrt(lam)
    Qp = Q * root[None, :]                           # step 3: Q' = Q sqrt(Lambda)
    dWp = dW @ Qp                                    # step 4
    U, sig, Vt = np.linalg.svd(dWp, full_matrices=False)   # step 5
    Bp = U[:, :r] * sig[None, :r]
    Ap = Vt[:r, :]
    A = (Ap / root[None, :]) @ Q.T                   # step 6: A' sqrt(Lambda)^-1 Q^T
    return Bp, A


def balance_factors(Bp, A):
    """Rescale component i of the pair by s_i = sqrt(|B'_i| / |A_i|): (B'_i / s_i, s_i A_i).

    Any invertible r x r matrix between the factors leaves B'A, and with it the compensated
    layer of Sec. 3, unchanged; this diagonal one gives both factors of every component the norm
    sqrt(|B'_i| |A_i|), so that neither leaves fp16's range when they are stored for inference
    (B' = U' Sigma' carries the singular values, A the inverse square roots of Lambda).
    A component with a zero factor is left as it is.
    """
    Bp = np.asarray(Bp, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    nb = np.sqrt(np.sum(Bp * Bp, axis=0))
    na = np.sqrt(np.sum(A * A, axis=1))
    ok = (nb > 0) & (na > 0)
    s = np.where(ok, np.sqrt(np.where(ok, nb, 1.0) / np.where(ok, na, 1.0)), 1.0)
    return Bp / s[None, :], A * s[:, None]


def store_factors_f16(Bp, A, balance=True):
    """The factors as inference reads them: (balanced,) rounded to fp16, in the F16 tile layout.
    Returns (A_tiles, B_tiles)."""
    from . import layout
    if balance:
        Bp, A = balance_factors(Bp, A)
    return layout.pack_f16(np.asarray(A).astype(np.float16)), layout.pack_f16(np.asarray(Bp).astype(np.float16))


def quantize_factor(Mat, bits):
    """Symmetric round-to-nearest quantisation of a factor to `bits` in {4, 3} (Sec. 4.5 and App. A.9
    quantise the factors; the paper names no quantiser, this is the plain one): per row and per group of
    min(128, K) columns, scale = fp16(max |v| / qpos) with qpos = 2^(bits-1) - 1 (1 where the group is all
    zero), code = clip(rint(v / scale) + zp, 1, 2 zp - 1) with the implicit zero-point zp = 2^(bits-1).
    Returns (codes uint8 rows x K, scales fp16 rows x K/KT); the value a code stands for is scale (code - zp)."""
    Mat = np.asarray(Mat, dtype=np.float64)
    rows, K = Mat.shape
    KT = min(128, K)
    zp = 1 << (bits - 1)
    qpos = zp - 1
    codes = np.empty((rows, K), dtype=np.uint8)
    scales = np.empty((rows, K // KT), dtype=np.float16)
    for g in range(K // KT):
        blk = Mat[:, g * KT:(g + 1) * KT]
        s16 = (np.max(np.abs(blk), axis=1) / qpos).astype(np.float16)
        s16[s16 == 0] = np.float16(1.0)
        q = np.rint(blk / s16.astype(np.float64)[:, None]) + zp
        codes[:, g * KT:(g + 1) * KT] = np.clip(q, 1, 2 * zp - 1).astype(np.uint8)
        scales[:, g] = s16
    return codes, scales


def store_factors_q(Bp, A, bits, balance=True):
    """The factors quantised (quantize_factor) and packed as inference reads them.
    Returns (A_q, A_scales, B_q, B_scales)."""
    from . import layout
    if balance:
        Bp, A = balance_factors(Bp, A)
    ca, sa = quantize_factor(A, bits)
    cb, sb = quantize_factor(Bp, bits)
    if bits == 4:
        return (layout.pack_q4(ca, 128), layout.pack_scales(sa),
                layout.pack_q4(cb, min(128, cb.shape[1])), layout.pack_scales(sb))
    if bits == 3:
        return layout.pack_q3(ca), layout.pack_scales(sa), layout.pack_q3(cb), layout.pack_scales(sb)
    raise ValueError("bits must be 4 or 3")


def plain_svd_factors(W, W_hat, r):
    """Rank-r SVD of the raw error (Sec. 2, Eq. 2): the case Xt Xt^T = I of the above."""
    dW = np.asarray(W, dtype=np.float64) - np.asarray(W_hat, dtype=np.float64)
    U, sig, Vt = np.linalg.svd(dW, full_matrices=False)
    return U[:, :r] * sig[None, :r], Vt[:r, :]


def layer_loss(W, W_hat, B, A, Xt):
    """|| (W - What - B A) Xt ||_F : the layer-wise compression loss (Eq. 1) left after compensation."""
    E = np.asarray(W, dtype=np.float64) - np.asarray(W_hat, dtype=np.float64) - B @ A
    return float(np.linalg.norm(E @ np.asarray(Xt, dtype=np.float64)))
