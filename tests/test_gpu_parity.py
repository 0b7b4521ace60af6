"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-3      # max |y - y_oracle| / max(|y_oracle|, rms(y_oracle)); fp32 accumulate, fp16 output


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2410_21271_amd as eora
    return eora


def _check(y, ref, tol=TOL):
    from oracle import linear
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = linear.y_error(y, ref)
    assert err <= tol, err
    return err


@pytest.mark.parametrize("w_bits", [4, 3, 2])
@pytest.mark.parametrize("group", [128, 384])
def test_unpack_and_dequant_bit_exact(gpu, w_bits, group):
    import torch
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import dev
    c = QCase(11 + w_bits, 768, 80, 1, 0, w_bits, group, packer=gpu)      # 5 row blocks x 6 k-tiles
    qw, sc, qz = dev(c.qw), dev(c.sc), dev(c.qz)
    codes = torch.full((80, 768), 255, dtype=torch.uint8, device="cuda")
    zeros = torch.full((80, 768 // group), 255, dtype=torch.uint8, device="cuda")
    gpu.unpack_q(qw, qz, codes, zeros, 768, 80, w_bits, group)
    W = torch.full((80, 768), float("nan"), dtype=torch.float32, device="cuda")
    gpu.dequant_q(qw, sc, qz, W, 768, 80, w_bits, group)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), c.logical["codes"])
    assert np.array_equal(zeros.cpu().numpy(), c.logical["zeros"])
    ref = linear.dequant_q(c.o_qw, c.o_qz, c.o_sc, 768, 80, w_bits, group)
    got = W.cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref)          # exact, not just close
    assert np.array_equal(got, ref.astype(np.float32))


@pytest.mark.parametrize("w_bits,ab_bits,r,M", [
    (4, 16, 0, 1), (4, 16, 32, 1), (4, 16, 128, 3), (3, 16, 0, 1), (3, 16, 64, 2),
    (4, 4, 64, 1), (4, 4, 128, 5), (3, 4, 256, 16), (4, 16, 96, 16), (4, 16, 64, 17), (3, 16, 32, 37),
    (2, 16, 0, 1), (2, 16, 64, 2), (2, 4, 128, 5), (2, 16, 32, 37),
    (4, 3, 128, 1), (3, 3, 128, 3), (2, 3, 256, 5), (4, 3, 128, 17),
])
def test_linear_q_small_shapes(gpu, w_bits, ab_bits, r, M):
    """Several row blocks and k-tiles, ragged token counts."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(1000 + 7 * r + M + w_bits, 640, 112, M, r, w_bits, 128, ab_bits, packer=gpu)
    _check(run_linear_q(c), c.oracle_y())


def test_adapter_off_equals_rank_zero_and_zero_factors(gpu):
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(5, 512, 64, 4, 32, 4, packer=gpu)
    y0 = run_linear_q(c, r=0)                 # adapter switched off: A and B are not even passed
    _check(y0, c.oracle_y(r=0))
    assert not np.array_equal(y0, run_linear_q(c))
    c.A = np.zeros_like(c.A)
    c.B = np.zeros_like(c.B)
    assert np.array_equal(run_linear_q(c), y0)


def test_row_independence_and_determinism(gpu):
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(9, 1024, 256, 16, 64, 3, packer=gpu)
    y = run_linear_q(c)
    assert np.array_equal(y, run_linear_q(c))                          # fixed reduction order
    ref = c.oracle_y()
    _check(y, ref)
    for m in (0, 7, 15):
        y1 = run_linear_q(c, M=1, x=c.x[m:m + 1])
        _check(y1, ref[m:m + 1])


def test_planted_integers_are_exact_on_gpu(gpu):
    """Small-integer codes, factors and activations: every fp32 partial sum is an exact integer,
    so the GPU result must equal the oracle's bit for bit (after the fp16 store)."""
    from oracle import layout, linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    rng = np.random.default_rng(3)
    c = QCase(3, 256, 32, 4, 32, 4, packer=None)
    codes = rng.integers(0, 16, (32, 256), dtype=np.uint8)
    zeros = rng.integers(0, 16, (32, 2), dtype=np.uint8)
    scales = np.full((32, 2), 0.5, np.float16)
    A = rng.integers(-2, 3, (32, 256)).astype(np.float16)
    B = rng.integers(-2, 3, (32, 32)).astype(np.float16) / 2
    c.x = rng.integers(-3, 4, (4, 256)).astype(np.float16) / 4
    c.logical.update(codes=codes, zeros=zeros, scales=scales, A=A, B=B)
    c.o_qw, c.o_qz, c.o_sc = layout.pack_q4(codes), layout.pack_zeros(zeros), layout.pack_scales(scales)
    c.o_A, c.o_B = layout.pack_f16(A), layout.pack_f16(B)
    c.pack_with(gpu)
    ref = c.oracle_y()
    assert np.array_equal(ref.astype(np.float16).astype(np.float64), ref)      # representable in fp16
    assert np.array_equal(run_linear_q(c).astype(np.float64), ref)


@pytest.mark.parametrize("name,d_in,d_out", [("q", 4096, 4096), ("k", 4096, 1024)])
@pytest.mark.parametrize("w_bits,M", [(4, 1), (4, 16), (3, 1)])
def test_config_shapes_fp16_factors(gpu, name, d_in, d_out, w_bits, M):
    """BASELINE configs 1 and 2 at full size (the oracle needs about a second each)."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(synth.seed_for(1 if w_bits == 4 else 2, 0 if name == "q" else 1), d_in, d_out, M, 128, w_bits,
              packer=gpu)
    _check(run_linear_q(c), c.oracle_y())


@pytest.mark.parametrize("w_bits,ab_bits,r,M,d_in,d_outs", [
    (3, 16, 128, 1, 4096, (4096, 1024, 1024)),      # query / key / value of the 8B layer, config 2
    (3, 16, 128, 1, 4096, (14336, 14336)),          # gate / up: enough row blocks that a workgroup takes two
    (4, 4, 128, 1, 4096, (1024, 2048)),             # 4-bit factors, config 3
    (2, 16, 128, 1, 4096, (4096, 1024, 1024)),      # 2-bit backbone
    (4, 3, 128, 1, 4096, (4096, 1024, 1024)),       # 3-bit factors
    (4, 3, 128, 150, 512, (64, 32)),                # 3-bit factors, many tokens: the members' rows form one GEMM
    (4, 16, 32, 3, 1024, (64, 16, 48, 32)),         # four members, three tokens
    (4, 16, 0, 2, 2048, (128, 64)),                 # adapter off
    (3, 16, 64, 8, 512, (64, 32)),                  # a shape the decode kernel does not take: members run in turn
    (4, 16, 128, 200, 512, (192, 64, 144)),         # many tokens: the members' rows form one GEMM (ragged tiles)
    (3, 16, 0, 130, 256, (16, 128)),                # the same with the adapter off
])
def test_group_of_layers_sharing_x(gpu, w_bits, ab_bits, r, M, d_in, d_outs):
    """Layers that read the same x in one call (query/key/value, gate/up): every member equals the
    oracle on its own weights and factors, and is bit-identical to a separate eora_linear_q call."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q, run_linear_q_group
    cases = [QCase(500 + 7 * i + d_in, d_in, d, M, r, w_bits, ab_bits=ab_bits, packer=gpu) for i, d in enumerate(d_outs)]
    x = cases[0].x
    ys = run_linear_q_group(cases, x)
    for c, y in zip(cases, ys):
        _check(y, c.oracle_y(x=x))
        if M < 128 or r == 0:                        # (with many tokens t is summed in a different split: not bit-identical)
            assert np.array_equal(y, run_linear_q(c, x=x))


@pytest.mark.parametrize("w_bits,ab_bits,r,M,d_in,d_outs", [
    (4, 16, 128, 16, 4096, (4096, 1024, 1024)),     # query / key / value at sixteen tokens
    (3, 4, 64, 37, 2048, (2048, 512)),              # three token blocks (ragged), 4-bit factors of rank 64
    (4, 16, 128, 64, 4096, (14336, 14336)),         # gate / up at 64 tokens
    (2, 16, 0, 9, 2048, (1024, 1024, 1024, 1040)),  # four members, bare, a ragged last row group
    (4, 3, 128, 100, 2048, (4096, 512)),            # seven token blocks: the members' partials share the scratch
    (4, 16, 512, 16, 2048, (1024, 1024, 1024, 1040)),   # four members at the largest rank: every flag of a token block in use
    (3, 16, 128, 127, 2048, (1024, 1024, 1024, 1024)),  # four members x eight token blocks: one k-range each
])
def test_group_of_layers_sharing_x_mid_token_counts(gpu, w_bits, ab_bits, r, M, d_in, d_outs):
    """5 .. 127 tokens: the members' workgroups run in one launch (the split of the sums may differ from a
    separate call's, so members are compared with the oracle, and two runs with each other)."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_group
    cases = [QCase(600 + 7 * i + d_in + M, d_in, d, M, r, w_bits, ab_bits=ab_bits, packer=gpu) for i, d in enumerate(d_outs)]
    x = cases[0].x
    ys = run_linear_q_group(cases, x)
    again = run_linear_q_group(cases, x)
    for c, y, y2 in zip(cases, ys, again):
        _check(y, c.oracle_y(x=x))
        assert np.array_equal(y, y2)


def test_workspace_is_reusable_without_clearing(gpu):
    """Nothing in the workspace is reset between calls: flags are compared with an epoch that each
    low-rank launch advances by one, so one workspace serves any number of calls of any shapes."""
    import torch
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    big = QCase(21, 1024, 512, 16, 128, 4, packer=gpu)
    small = QCase(22, 256, 64, 3, 32, 3, packer=gpu)
    ws = gpu.new_workspace(16, 1024, 512, 128)
    torch.cuda.synchronize()
    e0 = int(ws[:4].view(torch.int32).cpu().numpy()[0])
    assert e0 != 0 and e0 % (1 << 20) == 0        # every initialisation starts its own range of epochs
    y1 = run_linear_q(big, ws=ws)
    y2 = run_linear_q(small, ws=ws)
    y0 = run_linear_q(big, ws=ws, r=0)            # no low-rank path: does not touch the header
    y3 = run_linear_q(big, ws=ws)
    hdr = ws[:256].view(torch.int32).cpu().numpy()
    assert hdr[0] == e0 + 3 and hdr[1] == 0       # epoch after three low-rank launches, no error
    assert not ws[128:128 + 33 * 128].view(torch.int32).cpu().numpy().any()      # arrival counters back at zero
    assert np.array_equal(y1, y3)
    _check(y1, big.oracle_y())
    _check(y2, small.oracle_y())
    _check(y0, big.oracle_y(r=0))
    assert gpu.workspace_error(ws) == 0


@pytest.mark.parametrize("M,d_in,d_out", [(1, 4096, 1024), (16, 2048, 8192), (37, 640, 112)])
def test_bounded_wait_gives_up_cleanly(gpu, M, d_in, d_out):
    """With a negative spin limit every wait for t counts as expired: the kernel still terminates, y lacks the
    low-rank term (so it differs from the oracle), the workspace reports the timeout, and after
    re-initialisation the same workspace works again.  (Decode kernel, the kernel for 5..127 tokens, and the
    general one.)"""
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(23 + M, d_in, d_out, M, 128, 4, packer=gpu)
    ws = gpu.new_workspace(M, d_in, d_out, 128)
    gpu.debug_set_spin_limit(-1)
    try:
        y = run_linear_q(c, ws=ws)
        status = gpu.workspace_error(ws)
    finally:
        gpu.debug_set_spin_limit(1 << 22)
    assert status == -8
    assert linear.y_error(y, c.oracle_y()) > 2e-3            # the result of an expired wait is not the layer's
    _check(y, c.oracle_y(r=0))                               # it is the bare backbone's
    gpu.workspace_init(ws)
    _check(run_linear_q(c, ws=ws), c.oracle_y())
    assert gpu.workspace_error(ws) == 0


def test_spin_limit_zero_never_hangs(gpu):
    """A spin limit of 0 (give up if t is not ready at the first look) ends either way; when it reports no
    timeout the result is the layer's."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(23, 4096, 1024, 1, 128, 4, packer=gpu)
    ws = gpu.new_workspace(1, 4096, 1024, 128)
    gpu.debug_set_spin_limit(0)
    try:
        y = run_linear_q(c, ws=ws)
        status = gpu.workspace_error(ws)
    finally:
        gpu.debug_set_spin_limit(1 << 22)
    assert status in (0, -8)
    if status == 0:
        _check(y, c.oracle_y())


def test_mid_size_token_counts(gpu):
    """Token counts beyond one launch chunk (256) and ragged blocks."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(24, 512, 96, 300, 64, 4, packer=gpu)
    _check(run_linear_q(c), c.oracle_y())


def test_expand_sp24_bit_exact(gpu):
    import torch
    from oracle import linear
    from tests.cases import SparseCase
    from tests.gpu_util import dev
    c = SparseCase(31, 640, 80, 1, 0, packer=gpu)
    W = torch.full((80, 640), float("nan"), dtype=torch.float16, device="cuda")
    gpu.expand_sp24(dev(c.values), dev(c.indices), W, 640, 80)
    torch.cuda.synchronize()
    ref = linear.expand_sp24_packed(c.o_values, c.o_indices, 640, 80)
    assert np.array_equal(W.cpu().numpy().astype(np.float64), ref)


@pytest.mark.parametrize("r,M", [(0, 1), (32, 1), (128, 2), (64, 4), (32, 5), (96, 16), (64, 37)])
def test_linear_sp24_small_shapes(gpu, r, M):
    from tests.cases import SparseCase
    from tests.gpu_util import run_linear_sp24
    c = SparseCase(2000 + 3 * r + M, 1024, 112, M, r, packer=gpu)
    _check(run_linear_sp24(c), c.oracle_y())


def test_linear_sp24_ragged_k_and_determinism(gpu):
    from tests.cases import SparseCase
    from tests.gpu_util import run_linear_sp24
    c = SparseCase(41, 640, 48, 3, 32, packer=gpu)           # d_in not a multiple of 512: fragments from global memory
    y = run_linear_sp24(c)
    _check(y, c.oracle_y())
    assert np.array_equal(y, run_linear_sp24(c))


@pytest.mark.parametrize("w_bits,ab_bits,r,M,d_in,d_out", [
    (3, 16, 128, 1, 14336, 4096),      # config 2, the down projection: the seven-wavefront instantiation
    (3, 16, 128, 2, 14336, 1024),      # the same contraction length with two tokens (fourteen wavefronts)
    (4, 4, 64, 1, 4096, 1024),         # config 3: 4-bit factors, rank 64 (64-column tiles of B)
    (4, 4, 512, 1, 4096, 1024),        # config 3: rank 512 (256 producer units)
    (4, 4, 256, 8, 4096, 1024),        # config 3 at eight tokens
    (4, 16, 128, 1, 8192, 1024),       # 70B-shaped quantised layers: eight wavefronts
    (3, 16, 128, 1, 28672, 512),       # and the 28672-long contraction
    (4, 16, 128, 4, 8192, 256),        # four tokens
    (2, 16, 128, 1, 4096, 4096),       # 2-bit backbone at the 8B shapes
    (2, 16, 128, 1, 14336, 1024),
    (2, 4, 128, 3, 4096, 1024),
    (4, 3, 128, 1, 4096, 4096),        # 3-bit factors at the 8B shapes
    (3, 3, 256, 2, 14336, 1024),
])
def test_more_config_shapes(gpu, w_bits, ab_bits, r, M, d_in, d_out):
    """Full contraction lengths of the configured layers that the other tests do not reach (every
    instantiation of the decode kernel the benchmark workloads launch)."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(synth.seed_for(3, d_in // 512 + r + M), d_in, d_out, M, r, w_bits, ab_bits=ab_bits, packer=gpu)
    _check(run_linear_q(c), c.oracle_y())


@pytest.mark.parametrize("w_bits,ab_bits,r,M,d_in,d_out,group", [
    (4, 16, 128, 16, 2048, 8192, 128),     # 2 row blocks x 4 ranges per workgroup
    (3, 16, 64, 37, 2048, 8208, 128),      # three token blocks (ragged), a ragged last pair of row blocks
    (4, 4, 128, 8, 4096, 4096, 128),       # config 3 at eight tokens: 1 row block x 8 ranges, 4-bit factors
    (4, 4, 64, 16, 4096, 4096, 128),       # 64-column tiles of B
    (3, 16, 0, 16, 14336, 4096, 128),      # the down projection's contraction length: 1 x 4, bare
    (3, 16, 128, 16, 14336, 1024, 128),    # few rows: the finest split, with the low-rank term
    (4, 16, 512, 16, 2048, 4096, 128),     # the largest rank: t fills the LDS of the x slots
    (4, 16, 32, 5, 2048, 4096, 2048),      # channel-wise groups
    (4, 16, 128, 127, 4096, 512, 128),     # eight token blocks, the last one ragged
    (2, 16, 128, 16, 2048, 8192, 128),     # 2-bit backbone
    (2, 16, 64, 37, 2048, 8208, 256),
    (4, 3, 128, 16, 2048, 8192, 128),      # 3-bit factors
    (3, 3, 128, 64, 4096, 4096, 128),
])
def test_linear_q_mid_token_counts(gpu, w_bits, ab_bits, r, M, d_in, d_out, group):
    """The kernel for 5..127 tokens (x shared through LDS), every split of a workgroup it launches."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(synth.seed_for(1, d_in // 512 + r + M + d_out // 16), d_in, d_out, M, r, w_bits, group=group, ab_bits=ab_bits, packer=gpu)
    y = run_linear_q(c)
    _check(y, c.oracle_y())
    assert np.array_equal(y, run_linear_q(c))


@pytest.mark.parametrize("M,r", [(1, 128), (3, 512), (4, 32)])
def test_config5_shape_long_contraction(gpu, M, r):
    """BASELINE config 5, the 28672-long contraction of the 70B-shaped down projection (1024 of its rows): sixteen
    k-ranges of t; with rank 512 every flag of a token block is in use."""
    import synth
    from tests.cases import SparseCase
    from tests.gpu_util import run_linear_sp24
    c = SparseCase(synth.seed_for(5, 6), 28672, 1024, M, r, packer=gpu)
    _check(run_linear_sp24(c), c.oracle_y())


def test_config5_shape_long_contraction_quantised_values(gpu):
    """The same contraction with 4-bit kept values."""
    import synth
    from tests.cases import SparseQCase
    from tests.gpu_util import run_linear_sp24q4
    c = SparseQCase(synth.seed_for(5, 6), 28672, 512, 2, 128, packer=gpu)
    _check(run_linear_sp24q4(c), c.oracle_y())


@pytest.mark.parametrize("M", [1, 64])
def test_config5_shape_k_projection(gpu, M):
    """BASELINE config 5, the 8192 -> 1024 linear of a 70B-shaped layer at full size."""
    import synth
    from tests.cases import SparseCase
    from tests.gpu_util import run_linear_sp24
    c = SparseCase(synth.seed_for(5, 1), 8192, 1024, M, 128, packer=gpu)
    _check(run_linear_sp24(c), c.oracle_y())


@pytest.mark.parametrize("r,M,d_in,d_out", [
    (0, 37, 1024, 5488),       # three token blocks (ragged), a ragged last group of row blocks, no low-rank term
    (32, 37, 1024, 5488),
    (128, 64, 2048, 4096),     # four full token blocks, XCD-aware order of the workgroups
    (512, 16, 512, 16384),     # one token block, one chunk, the largest rank (t fills the x buffers' LDS)
])
def test_linear_sp24_many_tokens_many_rows(gpu, r, M, d_in, d_out):
    """The kernel that shares a token block's x between row blocks through LDS (more than 4 tokens and
    enough rows to fill the chip)."""
    from tests.cases import SparseCase
    from tests.gpu_util import run_linear_sp24
    c = SparseCase(2300 + r + M, d_in, d_out, M, r, packer=gpu)
    y = run_linear_sp24(c)
    _check(y, c.oracle_y())
    assert np.array_equal(y, run_linear_sp24(c))


def test_sparse_many_tokens_different_inputs_on_one_workspace(gpu):
    """The many-token 2:4 kernel hands t over as untagged fp32 partials behind flags: two different activations, then
    a different layer, then the first again, back to back on ONE workspace that is never cleared in between.  A
    partial of an earlier call read in place of this call's would show against the oracle (the inputs differ)."""
    import synth
    from tests.cases import SparseCase
    from tests.gpu_util import run_linear_sp24
    a = SparseCase(2401, 2048, 16384, 64, 128, packer=gpu)
    b = SparseCase(2402, 2048, 16384, 48, 128, packer=gpu)
    ws = gpu.new_workspace(64, 2048, 16384, 128)
    x2 = synth.draw_layer(2403, 2048, 16, 64, 0)[3]
    for c, x in ((a, a.x), (a, x2), (b, b.x), (a, a.x), (b, b.x[::-1].copy())):
        y = run_linear_sp24(c, x=x, ws=ws)
        assert gpu.debug_last_launch().startswith("sparse_wide"), gpu.debug_last_launch()
        _check(y, c.oracle_y(x=x))
    assert gpu.workspace_error(ws) == 0


@pytest.mark.parametrize("w_bits,r,M,d_out", [(4, 0, 128, 128), (4, 128, 200, 192), (3, 256, 333, 144), (4, 128, 129, 16), (2, 128, 200, 192), (2, 0, 130, 48)])
def test_prefill_gemm_small_shapes(gpu, w_bits, r, M, d_out):
    """The many-token GEMM path: ragged token and row tiles, with and without the low-rank extension."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(3000 + r + M, 512, d_out, M, r, w_bits, packer=gpu)
    _check(run_linear_q(c), c.oracle_y())


@pytest.mark.parametrize("w_bits,ab_bits,r,M,d_out", [(4, 4, 128, 200, 192), (3, 4, 256, 333, 144), (4, 3, 128, 129, 16), (2, 3, 256, 200, 272)])
def test_prefill_gemm_quantised_factors(gpu, w_bits, ab_bits, r, M, d_out):
    """The many-token GEMM path with 4-bit and 3-bit factors (quantised EoRA, Sec. 4.5 / App. A.9): A is the weight
    operand of the down-projection launch, B's tiles are decoded in the second segment."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(3100 + r + M, 512, d_out, M, r, w_bits, ab_bits=ab_bits, packer=gpu)
    _check(run_linear_q(c), c.oracle_y())
    assert gpu.debug_last_launch().startswith("prefill FM=%d EXT=1" % {4: 1, 3: 2, 2: 6}[w_bits]), gpu.debug_last_launch()
    assert gpu.debug_last_launch().endswith("FE=%d" % {4: 3, 3: 7}[ab_bits])


def test_prefill_config4_shape_sampled_rows(gpu):
    """BASELINE config 4: M = 2048, 4096 -> 4096, 4-bit backbone, fp16 rank-256 factors, 1 % outlier
    channels scaled by 20.  The oracle is evaluated on a seeded subset of token rows (first and last
    rows of tiles included) over all output columns."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(synth.seed_for(4, 0), 4096, 4096, 2048, 256, 4, outlier_frac=0.01, packer=gpu)
    y = run_linear_q(c)
    rows = np.unique(np.concatenate([np.array([0, 1, 63, 64, 127, 128, 255, 256, 1023, 1024, 2046, 2047]),
                                     np.random.default_rng(0).integers(0, 2048, 52)]))
    _check(y[rows], c.oracle_y(rows=rows))


@pytest.mark.parametrize("w_bits,r,M,d_in,d_out", [
    (4, 128, 2043, 512, 16400),      # 16 token tiles (ragged) x 65 row tiles (ragged): low-rank extension
    (3, 0, 2048, 640, 16384),        # bare, five steps (odd: both LDS buffers end the loop)
])
def test_prefill_gemm_large_row_tiles(gpu, w_bits, r, M, d_in, d_out):
    """The many-token GEMM with many row tiles (as gate+up of a decoder layer at 2048 tokens), ragged in both
    directions.  The oracle is evaluated on a seeded subset of token rows over all output columns."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(3300 + r + w_bits, d_in, d_out, M, r, w_bits, packer=gpu)
    y = run_linear_q(c)
    rows = np.unique(np.concatenate([np.array([0, 31, 32, 127, 128, 1023, 1024, M - 2, M - 1]),
                                     np.random.default_rng(1).integers(0, M, 40)]))
    _check(y[rows], c.oracle_y(rows=rows))


def test_prefill_config4_gate_up_group_sampled_rows(gpu):
    """BASELINE config 4, the gate and up projections (4096 -> 14336 each) as one grouped call at 2048 tokens:
    the launch bench.py times.  Sampled token rows, all output columns of both members."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_group
    cs = [QCase(synth.seed_for(4, 4 + i), 4096, 14336, 2048, 256, 4, outlier_frac=0.01, packer=gpu) for i in range(2)]
    ys = run_linear_q_group(cs, cs[0].x)
    rows = np.unique(np.concatenate([np.array([0, 127, 128, 2047]), np.random.default_rng(2).integers(0, 2048, 12)]))
    for c, y in zip(cs, ys):
        _check(y[rows], c.oracle_y(rows=rows, x=cs[0].x))


def test_expand_sp24q4_bit_exact(gpu):
    """Unpack + dequantise + expand of the 2:4 + 4-bit format: scale*(code - zero) is exact in fp32."""
    import torch
    from tests.cases import SparseQCase
    from tests.gpu_util import dev
    from oracle import linear
    for group in (128, 384):
        c = SparseQCase(31 + group, 768, 80, 1, 0, group=group, packer=gpu)
        W = torch.full((80, 768), 7.0, dtype=torch.float32, device="cuda")
        gpu.expand_sp24q4(dev(c.tiles), dev(c.meta), W, 768, 80)
        torch.cuda.synchronize()
        ref = linear.dequant_sp24q4_packed(c.o_tiles, c.o_meta, 768, 80)
        L = c.logical
        assert np.array_equal(ref, linear.dequant_sp24q4(L["codes"], L["pos"], L["zeros"], L["scales"], group))
        assert np.array_equal(W.cpu().numpy().astype(np.float64), ref)


@pytest.mark.parametrize("r,M,d_in,d_out,group", [
    (0, 1, 1024, 112, 128), (32, 1, 1024, 112, 128), (128, 2, 1024, 112, 256), (64, 4, 640, 48, 128),
    (32, 5, 1024, 112, 128), (96, 16, 1024, 112, 1024), (64, 37, 1024, 5488, 128), (128, 64, 2048, 4096, 128),
])
def test_linear_sp24q4_shapes(gpu, r, M, d_in, d_out, group):
    """The layer on the 2:4 + 4-bit backbone: the decode kernel (x in LDS or from global memory), coarser
    groups, and the kernel for many tokens and rows."""
    from tests.cases import SparseQCase
    from tests.gpu_util import run_linear_sp24q4
    c = SparseQCase(2600 + r + M, d_in, d_out, M, r, group=group, packer=gpu)
    y = run_linear_sp24q4(c)
    _check(y, c.oracle_y())
    assert np.array_equal(y, run_linear_sp24q4(c))


@pytest.mark.parametrize("M", [1, 64])
def test_sp24q4_70b_shape_k_projection(gpu, M):
    """The 8192 -> 1024 linear of a 70B-shaped layer at full size on the 2:4 + 4-bit backbone."""
    import synth
    from tests.cases import SparseQCase
    from tests.gpu_util import run_linear_sp24q4
    c = SparseQCase(synth.seed_for(5, 11), 8192, 1024, M, 128, packer=gpu)
    _check(run_linear_sp24q4(c), c.oracle_y())


@pytest.mark.parametrize("quantised", [False, True])
@pytest.mark.parametrize("r,M,d_in,d_outs", [
    (32, 1, 1024, (256, 64, 64)),          # query / key / value in miniature, one token (x in LDS)
    (0, 3, 1024, (128, 128)),              # bare
    (64, 37, 1024, (192, 64, 48, 16)),     # four members, three token blocks: the kernel without shared x
    (128, 64, 2048, (4096, 1024, 1024)),   # enough rows together for the kernel that shares x through LDS
    (32, 300, 512, (64, 32)),              # more than 256 tokens: the members run one after the other
    (512, 16, 1024, (1024, 1024, 1024, 1040)),   # four members at the largest rank
    (128, 127, 2048, (2048, 1024, 1024, 512)),   # four members x eight token blocks
    (64, 256, 1024, (128, 64)),            # sixteen token blocks: the most one launch takes
])
def test_sparse_group_of_layers_sharing_x(gpu, quantised, r, M, d_in, d_outs):
    """2:4 layers that read the same x in one call: every member equals the oracle on its own weights and
    factors; two runs are identical; for up to four tokens the result is that of a separate call, bit for bit."""
    from tests.cases import SparseCase, SparseQCase
    from tests.gpu_util import run_linear_sp24, run_linear_sp24_group, run_linear_sp24q4
    make = SparseQCase if quantised else SparseCase
    cases = [make(900 + 7 * i + M + d_in, d_in, d, M, r, packer=gpu) for i, d in enumerate(d_outs)]
    for c in cases[1:]:
        c.x = cases[0].x
    ys = run_linear_sp24_group(cases)
    again = run_linear_sp24_group(cases)
    for c, y, y2 in zip(cases, ys, again):
        _check(y, c.oracle_y())
        assert np.array_equal(y, y2)
        if M <= 4:
            assert np.array_equal(y, run_linear_sp24q4(c) if quantised else run_linear_sp24(c))
