"""GPU parity of Algorithm 1 steps 1-6 (eora_factors, fp64 one-sided Jacobi) against the numpy oracle.

The r components are unique up to sign (distinct singular values), so sigma and the product B'A are
compared directly and the factors after aligning each component's sign.  Tolerances: both sides work
in fp64 (unit roundoff 1.1e-16); the Jacobi sweeps stop at relative orthogonality sqrt(L) * 1.1e-16 and
the eigenvectors of the Gram matrix enter through sqrt(Lambda)^-1 (condition of the synthetic Gram
matrix <= 2e6), so products agree to about 1e-10 relative; the tests allow 1e-8, and 1e-6 on single
components, whose sensitivity is 1 / (relative gap between neighbouring singular values, ~1e-3 here).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2410_21271_amd as eora
    return eora


def _inputs(seed, d_in, d_out, n_tokens, w_bits=4, group=128):
    import synth
    from oracle import linear
    W, _, _, _ = synth.draw_layer(seed, d_in, d_out, 1, 0)
    codes, zeros, scales = synth.quantize_rtn(W, w_bits, group)
    W_hat = linear.dequant(codes, zeros, scales, group).astype(np.float32)      # exact in fp32
    Xt = synth.draw_calibration(seed + 1, d_in, n_tokens)
    return W, W_hat, Xt


def _run(eora, W, W_hat, Xt, r, eig_floor=1e-12, want_route=None):
    """want_route: "cholesky" or "eig": assert (from the call's counters) which route steps 2-4 took."""
    import torch
    d_out, d_in = W.shape
    n = Xt.shape[1]
    Wd, Whd, Xd = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda() for a in (W, W_hat, Xt))
    B = torch.full((d_out, r), float("nan"), dtype=torch.float64, device="cuda")
    A = torch.full((r, d_in), float("nan"), dtype=torch.float64, device="cuda")
    sig = torch.full((r,), float("nan"), dtype=torch.float64, device="cuda")
    ws = torch.empty(eora.factors_workspace_bytes(d_in, d_out, r), dtype=torch.uint8, device="cuda")
    st = eora.factors(Wd, Whd, Xd, B, A, sig, n, d_in, d_out, r, eig_floor, ws, stats=True)
    torch.cuda.synchronize()
    if want_route is not None:
        assert (st["eig_rows"] == 0) == (want_route == "cholesky"), st
        if want_route == "cholesky":
            # step 5's matrix (min x max) is reduced to a square factor when it is at least twice as long as it has rows
            lo, hi = min(d_in, d_out), max(d_in, d_out)
            assert int(st["eig_rotations"]) == (lo if hi >= 2 * lo else hi), st
    return B.cpu().numpy(), A.cpu().numpy(), sig.cpu().numpy()


def _compare(W, W_hat, Xt, r, B, A, sig):
    from oracle import calibrate
    Bo, Ao = calibrate.eora_factors(W, W_hat, Xt, r)
    sig_o = np.linalg.norm(Bo, axis=0)                      # B' = U' Sigma'
    assert np.all(np.isfinite(B)) and np.all(np.isfinite(A))
    assert np.allclose(sig, sig_o, rtol=1e-9, atol=0), np.abs(sig / sig_o - 1).max()
    P, Po = B @ A, Bo @ Ao
    assert np.abs(P - Po).max() <= 1e-8 * np.abs(Po).max(), np.abs(P - Po).max() / np.abs(Po).max()
    sign = np.sign(np.sum(B * Bo, axis=0))
    assert np.all(sign != 0)
    assert np.abs(B * sign[None, :] - Bo).max() <= 1e-6 * np.abs(Bo).max()
    assert np.abs(A * sign[:, None] - Ao).max() <= 1e-6 * np.abs(Ao).max()
    # Theorem 1 with Eckart-Young: the loss left is the tail of the singular values of dW Q'
    lam, Q = np.linalg.eigh(calibrate.gram(Xt))
    tail = np.linalg.svd((W.astype(np.float64) - W_hat) @ (Q * np.sqrt(lam)[None, :]), compute_uv=False)[r:]
    assert np.isclose(calibrate.layer_loss(W, W_hat, B, A, Xt), np.sqrt(np.sum(tail ** 2)), rtol=1e-8)


SHAPES = [
    # d_in, d_out, n_tokens, r
    (128, 64, 300, 16),          # fewer output rows: the rows of dW' are rotated
    (128, 192, 256, 32),         # more output rows: the rows of dW'^T are rotated
    (256, 256, 600, 32),
    (384, 130, 1000, 2),         # ragged tiles of the GEMM, tiny rank
    (640, 256, 1300, 64),        # rows longer than one 64-lane pass
    (128, 320, 300, 16),         # many more output rows: dW'^T reduced to a square factor before the sweeps
]


@pytest.mark.parametrize("route", ["cholesky", "eig"])
@pytest.mark.parametrize("d_in,d_out,n_tokens,r", SHAPES)
def test_factors_match_oracle(gpu, d_in, d_out, n_tokens, r, route):
    """Both ways of steps 2-4 and 6 against the oracle (which takes the paper's steps with LAPACK): the Cholesky
    factor of the Gram matrix (the route a well-conditioned Gram matrix takes) and the eigendecomposition by Jacobi
    sweeps (the route of a nearly singular one, forced here by the test hook)."""
    W, W_hat, Xt = _inputs(7000 + d_in + d_out, d_in, d_out, n_tokens)
    gpu.debug_set_factors_route(1 if route == "eig" else 0)
    try:
        B, A, sig = _run(gpu, W, W_hat, Xt, r, want_route=route)
    finally:
        gpu.debug_set_factors_route(0)
    _compare(W, W_hat, Xt, r, B, A, sig)


def test_planted_rank_r_error_is_recovered_and_served(gpu):
    """W = What + (rank-r term): Algorithm 1 returns that term, and the compensated quantised layer
    (steps 1-6 here, step 7 through eora_linear_q) reproduces x.W^T."""
    import torch
    import synth
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import dev
    d_in, d_out, r, M = 256, 128, 32, 5
    c = QCase(7100, d_in, d_out, M, 0, 4, 128, packer=gpu)
    L = c.logical
    W_hat = linear.dequant(L["codes"], L["zeros"], L["scales"], 128)
    rng = np.random.default_rng(7101)
    low = (rng.standard_normal((d_out, r)) @ rng.standard_normal((r, d_in)) * 0.002).astype(np.float32)
    W = (W_hat + low).astype(np.float32)
    dW = W.astype(np.float64) - W_hat
    Xt = synth.draw_calibration(7102, d_in, 700)
    B, A, _ = _run(gpu, W, W_hat.astype(np.float32), Xt, r)
    # W is rounded to fp32 after the rank-r term was added, so dW is rank r only up to 6e-8 |W|
    assert np.abs(B @ A - dW).max() <= 1e-5 * np.abs(dW).max()
    # rebalance the two factors (any invertible r x r matrix between them leaves B'A unchanged) so that
    # both sit well inside fp16's range, then serve them
    s = np.sqrt(np.linalg.norm(B, axis=0) / np.linalg.norm(A, axis=1))
    A16, B16 = (A * s[:, None]).astype(np.float16), (B / s[None, :]).astype(np.float16)
    qw, sc, qz = dev(c.qw), dev(c.sc), dev(c.qz)
    Ad, Bd = dev(gpu.pack_factor_f16(A16)), dev(gpu.pack_factor_f16(B16))
    y = torch.full((M * d_out,), 777.0, dtype=torch.float16, device="cuda")
    ws = gpu.new_workspace(M, d_in, d_out, r)
    gpu.linear_q(dev(c.x), qw, sc, qz, Ad, Bd, None, None, y, M, d_in, d_out, r, 4, 128, 16, ws)
    torch.cuda.synchronize()
    assert gpu.workspace_error(ws) == 0
    ref = c.x.astype(np.float64) @ W.astype(np.float64).T
    err = linear.y_error(y.cpu().numpy().reshape(M, d_out), ref)
    assert err <= 2e-3, err


@pytest.mark.parametrize("d_in,d_out", [(128, 64), (128, 160)])
def test_error_of_rank_below_r(gpu, d_in, d_out):
    """No compression error at all gives B'A = 0 with finite factors; an error of rank 2 asked for at rank 8
    is returned exactly, the six spare components being zero."""
    import synth
    W, W_hat, _ = _inputs(7400 + d_out, d_in, d_out, 16)
    Xt = synth.draw_calibration(7401, d_in, 300)
    B, A, sig = _run(gpu, W_hat, W_hat, Xt, 8)
    assert np.all(np.isfinite(B)) and np.all(np.isfinite(A)) and np.all(sig == 0)
    assert np.all(B @ A == 0)
    rng = np.random.default_rng(7402)
    low = (rng.standard_normal((d_out, 2)) @ rng.standard_normal((2, d_in)) * 0.01)
    W2 = (W_hat + low).astype(np.float32)
    dW = W2.astype(np.float64) - W_hat
    B, A, sig = _run(gpu, W2, W_hat, Xt, 8)
    assert np.all(np.isfinite(B)) and np.all(np.isfinite(A))
    assert np.abs(B @ A - dW).max() <= 1e-5 * np.abs(dW).max()          # dW is rank 2 up to the fp32 rounding of W2
    assert sig[1] > 0 and np.all(sig[2:] <= 1e-5 * sig[0])


@pytest.mark.parametrize("balance", [False, True])
def test_store_f16_matches_oracle_tiles(gpu, balance):
    """fp64 factors -> fp16 tiles on the GPU against the oracle's rounding and layout.  Without balancing the
    result is one rounding of the same number: bit-exact.  With it the scale s_i comes from sums taken in a
    different order, so a value that sits within 1e-15 of a rounding boundary may fall on the other side: at
    most one fp16 step, on a handful of entries."""
    import torch
    from oracle import calibrate, layout
    rng = np.random.default_rng(7500)
    d_in, d_out, r = 256, 80, 64
    B = rng.standard_normal((d_out, r)) * np.exp(rng.uniform(-6, 6, r))[None, :]
    A = rng.standard_normal((r, d_in)) * np.exp(rng.uniform(-6, 6, r))[:, None]
    Bd, Ad = torch.from_numpy(B).cuda(), torch.from_numpy(A).cuda()
    At = torch.full((r * d_in,), float("nan"), dtype=torch.float16, device="cuda")
    Bt = torch.full((d_out * r,), float("nan"), dtype=torch.float16, device="cuda")
    scratch = torch.empty(r, dtype=torch.float64, device="cuda")
    gpu.factors_store_f16(Bd, Ad, d_in, d_out, r, balance, At, Bt, scratch if balance else None)
    torch.cuda.synchronize()
    oA, oB = calibrate.store_factors_f16(B, A, balance=balance)
    for got, want, rows, K in ((At.cpu().numpy(), oA, r, d_in), (Bt.cpu().numpy(), oB, d_out, r)):
        g, w = layout.unpack_f16(got, rows, K), layout.unpack_f16(want, rows, K)
        if not balance:
            assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
        else:
            diff = np.abs(g.view(np.int16).astype(np.int32) - w.view(np.int16).astype(np.int32))
            assert diff.max() <= 1 and np.count_nonzero(diff) <= 1e-3 * diff.size


@pytest.mark.parametrize("bits,r", [(4, 128), (4, 64), (3, 128), (3, 256)])
def test_store_q_matches_oracle_bytes(gpu, bits, r):
    """Quantised storage without balancing is the same arithmetic on the same numbers (fp64 quotient, rint,
    fp16 scale): codes, their packing and the scales are bit-exact.  With balancing the per-component scale
    comes from sums in another order, which can move a value across a rounding boundary: the dequantised
    factors then agree except on a few entries, by one step."""
    import torch
    from oracle import calibrate, linear
    rng = np.random.default_rng(7700 + bits + r)
    d_in, d_out = 384, 48
    B = rng.standard_normal((d_out, r)) * np.exp(rng.uniform(-4, 4, r))[None, :]
    A = rng.standard_normal((r, d_in)) * np.exp(rng.uniform(-4, 4, r))[:, None]
    A[3, 128:256] = 0.0                                         # an all-zero group
    Bd, Ad = torch.from_numpy(B).cuda(), torch.from_numpy(A).cuda()
    KTb = min(128, r)
    wpl = bits                                                  # 32-bit words per 32 codes
    for balance in (False, True):
        Aq = torch.full((r * d_in * wpl // 32,), -1, dtype=torch.int32, device="cuda")
        Bq = torch.full((d_out * r * wpl // 32,), -1, dtype=torch.int32, device="cuda")
        As = torch.full((r * d_in // 128,), float("nan"), dtype=torch.float16, device="cuda")
        Bs = torch.full((d_out * r // KTb,), float("nan"), dtype=torch.float16, device="cuda")
        scratch = torch.empty(r, dtype=torch.float64, device="cuda")
        gpu.factors_store_q(Bd, Ad, d_in, d_out, r, bits, balance, Aq, As, Bq, Bs, scratch if balance else None)
        torch.cuda.synchronize()
        oAq, oAs, oBq, oBs = calibrate.store_factors_q(B, A, bits, balance=balance)
        gAq, gBq = Aq.cpu().numpy().view(np.uint32), Bq.cpu().numpy().view(np.uint32)
        gAs, gBs = As.cpu().numpy(), Bs.cpu().numpy()
        if not balance:
            assert np.array_equal(gAq, oAq) and np.array_equal(gBq, oBq)
            assert np.array_equal(gAs.view(np.uint16), oAs.view(np.uint16)) and np.array_equal(gBs.view(np.uint16), oBs.view(np.uint16))
        else:
            deq = linear.dequant_factor_q4 if bits == 4 else linear.dequant_factor_q3
            for g, gs, o, os_, rows, K in ((gAq, gAs, oAq, oAs, r, d_in), (gBq, gBs, oBq, oBs, d_out, r)):
                dg, do = deq(g, gs, rows, K), deq(o, os_, rows, K)
                step = np.repeat(layout_scales(os_, rows, K), min(128, K), axis=1)
                assert np.all(np.abs(dg - do) <= 1.001 * step) and np.count_nonzero(dg != do) <= 2e-3 * dg.size


def layout_scales(packed, rows, K):
    from oracle import layout
    return layout.unpack_scales(packed, rows, K // min(128, K)).astype(np.float64)


def test_calibrate_quantise_serve_on_the_gpu(gpu):
    """Algorithm 1, 4-bit storage of its factors and the forward pass, all on the device: y equals the oracle's
    forward pass on the stored bytes (format consistency), and the 4-bit compensation removes most of the
    compression error."""
    import torch
    import synth
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import dev
    d_in, d_out, r, M = 512, 256, 128, 6
    c = QCase(7800, d_in, d_out, M, 0, 3, 128, packer=gpu)
    qw, sc, qz = dev(c.qw), dev(c.sc), dev(c.qz)
    W_hat = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    gpu.dequant_q(qw, sc, qz, W_hat, d_in, d_out, 3, 128)
    rng = np.random.default_rng(7801)
    low = (rng.standard_normal((d_out, r)) @ rng.standard_normal((r, d_in)) * 0.002).astype(np.float32)
    W = W_hat + torch.from_numpy(low).cuda()
    Xt = torch.from_numpy(synth.draw_calibration(7802, d_in, 1100)).cuda()
    B = torch.empty((d_out, r), dtype=torch.float64, device="cuda")
    A = torch.empty((r, d_in), dtype=torch.float64, device="cuda")
    ws = torch.empty(gpu.factors_workspace_bytes(d_in, d_out, r), dtype=torch.uint8, device="cuda")
    gpu.factors(W, W_hat, Xt, B, A, None, 1100, d_in, d_out, r, 1e-12, ws)
    Aq = torch.empty(r * d_in // 8, dtype=torch.int32, device="cuda")
    Bq = torch.empty(d_out * r // 8, dtype=torch.int32, device="cuda")
    As = torch.empty(r * d_in // 128, dtype=torch.float16, device="cuda")
    Bs = torch.empty(d_out * r // 128, dtype=torch.float16, device="cuda")
    gpu.factors_store_q(B, A, d_in, d_out, r, 4, True, Aq, As, Bq, Bs, torch.empty(r, dtype=torch.float64, device="cuda"))
    y = torch.full((M * d_out,), 777.0, dtype=torch.float16, device="cuda")
    lws = gpu.new_workspace(M, d_in, d_out, r)
    gpu.linear_q(dev(c.x), qw, sc, qz, Aq, Bq, As, Bs, y, M, d_in, d_out, r, 3, 128, 4, lws)
    torch.cuda.synchronize()
    assert gpu.workspace_error(lws) == 0
    y = y.cpu().numpy().reshape(M, d_out)
    stored = linear.eora_linear_q(c.x, c.o_qw, c.o_sc, c.o_qz, Aq.cpu().numpy().view(np.uint32), Bq.cpu().numpy().view(np.uint32),
                                  As.cpu().numpy(), Bs.cpu().numpy(), M, d_in, d_out, r, 3, 128, 4)
    assert linear.y_error(y, stored) <= 2e-3
    ref = c.x.astype(np.float64) @ W.cpu().numpy().astype(np.float64).T
    assert linear.y_error(y, ref) < 0.25 * linear.y_error(c.oracle_y(), ref)


def test_calibrate_store_serve_on_the_gpu(gpu):
    """Steps 1-7 without leaving the device: dequantise, eora_factors, eora_factors_store_f16, eora_linear_q.
    The error has rank r, so the served layer reproduces x.W^T up to the fp16 roundings."""
    import torch
    import synth
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import dev
    d_in, d_out, r, M = 512, 256, 64, 7
    c = QCase(7600, d_in, d_out, M, 0, 3, 128, packer=gpu)
    qw, sc, qz = dev(c.qw), dev(c.sc), dev(c.qz)
    W_hat = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    gpu.dequant_q(qw, sc, qz, W_hat, d_in, d_out, 3, 128)
    rng = np.random.default_rng(7601)
    low = (rng.standard_normal((d_out, r)) @ rng.standard_normal((r, d_in)) * 0.002).astype(np.float32)
    W = W_hat + torch.from_numpy(low).cuda()
    Xt = torch.from_numpy(synth.draw_calibration(7602, d_in, 1100)).cuda()
    B = torch.empty((d_out, r), dtype=torch.float64, device="cuda")
    A = torch.empty((r, d_in), dtype=torch.float64, device="cuda")
    ws = torch.empty(gpu.factors_workspace_bytes(d_in, d_out, r), dtype=torch.uint8, device="cuda")
    gpu.factors(W, W_hat, Xt, B, A, None, 1100, d_in, d_out, r, 1e-12, ws)
    At = torch.empty(r * d_in, dtype=torch.float16, device="cuda")
    Bt = torch.empty(d_out * r, dtype=torch.float16, device="cuda")
    gpu.factors_store_f16(B, A, d_in, d_out, r, True, At, Bt, torch.empty(r, dtype=torch.float64, device="cuda"))
    y = torch.full((M * d_out,), 777.0, dtype=torch.float16, device="cuda")
    lws = gpu.new_workspace(M, d_in, d_out, r)
    gpu.linear_q(dev(c.x), qw, sc, qz, At, Bt, None, None, y, M, d_in, d_out, r, 3, 128, 16, lws)
    torch.cuda.synchronize()
    assert gpu.workspace_error(lws) == 0
    ref = c.x.astype(np.float64) @ W.cpu().numpy().astype(np.float64).T
    err = linear.y_error(y.cpu().numpy().reshape(M, d_out), ref)
    assert err <= 2e-3, err
    # and without the compensation the compressed layer is far off
    bare = linear.y_error(c.oracle_y(), ref)
    assert bare > 20 * err


def test_fewer_tokens_than_channels(gpu):
    """Rank-deficient Gram matrix (tokens < d_in): its null space gets the floored eigenvalue on both sides
    (the floor is isotropic there, so the basis chosen inside the null space does not matter).  The inverse
    square root of the floor (1e4 relative to the largest root) amplifies rounding, hence the looser bound."""
    from oracle import calibrate
    d_in, d_out, n_tokens, r = 256, 64, 150, 8
    W, W_hat, Xt = _inputs(7300, d_in, d_out, n_tokens)
    B, A, sig = _run(gpu, W, W_hat, Xt, r, eig_floor=1e-8, want_route="eig")      # the factorisation meets a zero pivot and gives up
    Bo, Ao = calibrate.eora_factors(W, W_hat, Xt, r, eig_floor=1e-8)
    assert np.allclose(sig, np.linalg.norm(Bo, axis=0), rtol=1e-6, atol=0)
    P, Po = B @ A, Bo @ Ao
    assert np.abs(P - Po).max() <= 1e-5 * np.abs(Po).max(), np.abs(P - Po).max() / np.abs(Po).max()
    # on the calibration activations themselves the two compensations act alike
    assert np.abs(P @ Xt - Po @ Xt).max() <= 1e-6 * np.abs(Po @ Xt).max()


def test_identity_gram_reduces_to_plain_svd(gpu):
    """Orthonormal rows of X~ make the projection trivial (Sec. 2, Eq. 2): B'A is the truncated SVD of dW."""
    from oracle import calibrate
    d_in, d_out, r = 128, 96, 8
    W, W_hat, _ = _inputs(7200, d_in, d_out, 16)
    Qo, _ = np.linalg.qr(np.random.default_rng(7201).standard_normal((512, d_in)))
    Xt = np.ascontiguousarray(Qo.T, dtype=np.float32)
    B, A, _ = _run(gpu, W, W_hat, Xt, r)
    Bs, As = calibrate.plain_svd_factors(W, W_hat, r)
    # X~ is orthonormal only up to its rounding to fp32 (1e-7), and so is the match
    assert np.abs(B @ A - Bs @ As).max() <= 1e-4 * np.abs(Bs @ As).max()


def test_factors_validation(gpu):
    import torch
    t = torch.zeros(64, dtype=torch.float64, device="cuda")
    ws = torch.empty(gpu.factors_workspace_bytes(128, 64, 8), dtype=torch.uint8, device="cuda")
    args = lambda **kw: dict(dict(W_f32=t, W_hat_f32=t, Xt_f32=t, B_f64=t, A_f64=t, sigma_f64=None, n_tokens=4, d_in=128,
                                  d_out=64, r=8, eig_floor=1e-12, workspace=ws), **kw)
    for bad, code in ((dict(W_f32=None), -1), (dict(d_in=127), -2), (dict(r=65), -2), (dict(r=0), -2),
                      (dict(n_tokens=0), -2), (dict(d_out=16386), -2), (dict(eig_floor=1.0), -7),
                      (dict(workspace=None), -5), (dict(workspace=ws[:1024]), -5)):
        with pytest.raises(gpu.EoraError) as e:
            gpu.factors(**args(**bad))
        assert e.value.status == code, (bad, e.value.status)
    assert gpu.factors_workspace_bytes(127, 64, 8) == 0
