"""GPU parity of eora_linear_q_multi (several adapters over one backbone, chosen per token row)
against the per-row oracle, element by element; same tolerance as the single-adapter layer."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2410_21271_amd as eora
    return eora


def _sel(seed, M, n):
    rng = np.random.default_rng(seed)
    sel = rng.integers(-1, n, M).astype(np.int32)
    sel[0] = n - 1
    if M > 1:
        sel[-1] = -1
    return sel


def _oracle(c, sel, r_per, rows=None):
    from oracle import linear
    rows = np.arange(c.M) if rows is None else rows
    return linear.eora_linear_q_multi(c.x[rows], c.o_qw, c.o_sc, c.o_qz, c.o_A, c.o_B, c.o_As, c.o_Bs, sel[rows],
                                      len(rows), c.d_in, c.d_out, r_per, c.r // r_per, c.w_bits, c.group, c.ab_bits)


SHAPES = [
    # M, d_in, d_out, adapters, r per adapter, w_bits, ab_bits
    (1, 512, 64, 2, 32, 4, 16),
    (3, 512, 64, 2, 32, 3, 16),
    (9, 1024, 96, 3, 64, 3, 16),
    (40, 1024, 256, 4, 128, 4, 16),        # three token blocks, the last ragged; rank 512 together
    (17, 512, 80, 2, 128, 4, 4),           # 4-bit factors: a scale group never spans two adapters
    (300, 256, 64, 2, 32, 4, 16),          # two chunks of 256 tokens
    (37, 2048, 2048, 2, 64, 4, 16),        # enough rows for the kernel that shares x through LDS; ragged last block
    (21, 2048, 4096, 2, 128, 3, 4),        # the same with 3-bit backbone and 4-bit factors
    (4, 4096, 1024, 4, 128, 4, 16),        # the decode kernel at an 8B shape: four adapters, four tokens
    (2, 14336, 512, 2, 128, 3, 4),         # the decode kernel's long contraction, 4-bit factors
    (200, 512, 192, 2, 128, 4, 16),        # many tokens: the GEMM path, t masked between its two launches (ragged tiles)
    (333, 1024, 144, 4, 128, 3, 4),        # the same with four adapters of 4-bit factors
    (130, 512, 64, 2, 128, 2, 3),          # 2-bit backbone, 3-bit factors
]


@pytest.mark.parametrize("M,d_in,d_out,n,r,w_bits,ab_bits", SHAPES)
def test_multi_adapter_shapes(gpu, M, d_in, d_out, n, r, w_bits, ab_bits):
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_multi
    c = QCase(8000 + M + d_out, d_in, d_out, M, n * r, w_bits, 128, ab_bits, packer=gpu)
    sel = _sel(8100 + M, M, n)
    y = run_linear_q_multi(c, sel, r)
    ref = _oracle(c, sel, r)
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert linear.y_error(y, ref) <= TOL, linear.y_error(y, ref)
    # the adapters matter: the bare layer is not within tolerance of the compensated one on compensated rows
    bare = c.oracle_y(r=0)
    on = sel >= 0
    if on.any():
        assert linear.y_error(bare[on], ref[on]) > 10 * TOL or ab_bits == 4


@pytest.mark.parametrize("M,d_in,d_out,n,r,w_bits,ab_bits,launch", [
    (16, 4096, 8192, 4, 128, 4, 16, "resident FM=1 FA=5 "),      # 512 row blocks: the kernel with x resident in LDS, rank 512 together
    (9, 2048, 6144, 2, 64, 3, 16, "resident FM=2 FA=5 "),
    (12, 4096, 6144, 2, 128, 4, 4, "resident FM=1 FA=3 "),       # 4-bit factors
    (16, 14336, 4096, 2, 128, 4, 16, "resident FM=1 FA=5 "),     # ranges of the contraction in different workgroups
])
def test_multi_adapter_5_to_16_tokens_many_rows(gpu, M, d_in, d_out, n, r, w_bits, ab_bits, launch):
    """5 .. 16 tokens with enough rows take the kernel that keeps x in LDS; the mask is applied where t goes to LDS."""
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_multi
    c = QCase(8400 + M + d_out, d_in, d_out, M, n * r, w_bits, 128, ab_bits, packer=gpu)
    sel = _sel(8500 + M, M, n)
    y = run_linear_q_multi(c, sel, r)
    assert gpu.debug_last_launch().startswith(launch), gpu.debug_last_launch()
    rows = np.arange(M)
    ref = _oracle(c, sel, r, rows)
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert linear.y_error(y, ref) <= TOL, linear.y_error(y, ref)
    none = run_linear_q_multi(c, np.full(M, -1, np.int32), r)           # no adapter anywhere: the bare layer
    assert linear.y_error(none, c.oracle_y(r=0)) <= TOL


def test_multi_adapter_none_selected_is_the_bare_layer_bit_for_bit(gpu):
    """Rows without an adapter add exact zeros to the backbone's accumulators."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_multi
    c = QCase(8200, 512, 64, 6, 64, 4, 128, 16, packer=gpu)
    y = run_linear_q_multi(c, np.full(6, -1, np.int32), 32)
    ref = c.oracle_y(r=0)
    from oracle import linear
    assert linear.y_error(y, ref) <= TOL
    y2 = run_linear_q_multi(c, np.array([-1, 5, -1, 99, -1, -7], np.int32), 32)     # out of range behaves as none
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))


def test_multi_adapter_8b_q_shape_sampled_rows(gpu):
    """8B q projection, 64 requests over four rank-128 adapters; the oracle on sampled token rows."""
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_multi
    M, n, r = 64, 4, 128
    c = QCase(8300, 4096, 4096, M, n * r, 4, 128, 16, packer=gpu)
    sel = _sel(8301, M, n)
    y = run_linear_q_multi(c, sel, r)
    rows = np.array([0, 1, 15, 16, 37, 62, 63])
    ref = _oracle(c, sel, r, rows)
    assert linear.y_error(y[rows], ref) <= TOL


def test_multi_adapter_validation(gpu):
    import torch
    t = torch.zeros(1 << 16, dtype=torch.float16, device="cuda")
    sel = torch.zeros(8, dtype=torch.int32, device="cuda")
    ws = gpu.new_workspace(4, 256, 32, 64)

    def call(**kw):
        a = dict(x=t, qweight=t, scales=t, qzeros=t, A_all=t, B_all=t, A_scales=None, B_scales=None, adapter_of_row=sel,
                 y=t, M=4, d_in=256, d_out=32, r=32, n_adapters=2, w_bits=4, group=128, ab_bits=16, workspace=ws)
        a.update(kw)
        return gpu.linear_q_multi(**a)

    for bad, code in ((dict(adapter_of_row=None), -1), (dict(n_adapters=0), -2), (dict(r=16), -2), (dict(r=0), -2),
                      (dict(n_adapters=17), -2), (dict(ab_bits=4, r=64, A_scales=t, B_scales=t), -2),
                      (dict(A_all=None), -1), (dict(w_bits=5), -3), (dict(workspace=None), -5)):
        with pytest.raises(gpu.EoraError) as e:
            call(**bad)
        assert e.value.status == code, (bad, e.value.status)
    call(M=0)
