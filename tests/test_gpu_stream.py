"""GPU parity of the kernel that serves 5 .. 16 tokens with x resident in LDS (one workgroup per compute unit, its
sixteen wavefronts as ranges of the contraction x row blocks, partial tiles added in a fixed order inside the
workgroup, t handed over as tagged pairs) against the oracle, element by element: every backbone width, fp16 and
4-bit factors, the bare layer, every split of a workgroup (2, 4 or 8 stored tiles per wavefront; one to four rounds
of row blocks), ragged token counts, groups of up to four members, results that do not depend on timing, a workspace
used by calls of different shapes in a row, and an expired wait."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def gpu():
    """The library, with the kernel under test also taking launches of few rows (by default those go to the kernel
    for 5 .. 127 tokens, which is faster there); the default is restored afterwards."""
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2410_21271_amd as eora
    eora.debug_set_resident_min_blocks(0)
    yield eora
    eora.debug_set_resident_min_blocks(-1)


def _check(y, ref):
    from oracle import linear
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = linear.y_error(y, ref)
    assert err <= TOL, err


@pytest.mark.parametrize("w_bits,ab_bits,M,d_in,d_out,r,ntw", [
    (4, 16, 16, 4096, 1024, 128, 2),       # one row block per workgroup: sixteen ranges
    (4, 16, 5, 1024, 512, 64, 2),          # fewest tokens, shortest contraction (four ranges x four row blocks)
    (3, 16, 13, 2048, 768, 128, 2),        # ragged tokens, 3-bit
    (2, 16, 9, 4096, 256, 32, 2),          # 2-bit, rank 32
    (4, 4, 16, 4096, 1024, 128, 2),        # 4-bit factors
    (3, 4, 7, 2048, 640, 256, 2),          # 4-bit factors, two tiles of B per row block
    (2, 4, 16, 1024, 256, 128, 2),
    (4, 16, 16, 4096, 7680, 128, 4),       # two row blocks per workgroup
    (3, 16, 16, 4096, 28672, 128, 8),      # seven or eight row blocks per workgroup: two rounds of four
    (4, 4, 12, 4096, 57344, 128, 8),       # four rounds (the most), 4-bit factors
    (2, 16, 16, 2048, 16384, 64, 4),       # d_in 2048: four ranges x four row blocks
    (4, 16, 8, 4096, 2048, 512, 2),        # the largest rank: t's pairs beyond the early ones
    (4, 16, 16, 4096, 1024, 0, 2),         # bare layer
    (3, 16, 6, 1024, 256, 0, 2),
    (2, 16, 11, 4096, 12288, 0, 8),
    # contractions longer than 4096: ranges of the contraction in different workgroups, partial tiles of t and of y
    # handed over as tagged pairs and added in the order of the ranges by the range that owns the row block
    (4, 16, 16, 14336, 4096, 128, None),   # the down projection: four ranges of 3584 columns (28 groups: 14 of 16 wavefronts stream)
    (3, 4, 9, 8192, 1024, 128, None),      # two ranges of 4096, 4-bit factors
    (2, 16, 16, 14336, 512, 0, None),      # bare: the launch counter is used for the tiles of y alone
    (4, 16, 12, 6144, 768, 64, None),      # two ranges of 3072 (24 groups)
    (4, 4, 7, 5120, 1280, 128, None),      # two ranges of 2560 (20 groups; A's 20 tiles per range over ten wavefronts)
    (3, 16, 16, 28672, 256, 32, None),     # seven ranges
])
def test_stream_matches_oracle(gpu, w_bits, ab_bits, M, d_in, d_out, r, ntw):
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(5100 + M + d_out + r + w_bits, d_in, d_out, M, r, w_bits, ab_bits=ab_bits, packer=gpu)
    y = run_linear_q(c)
    assert gpu.debug_last_launch().startswith("resident FM=%d " % {4: 1, 3: 2, 2: 6}[w_bits]), gpu.debug_last_launch()
    if ntw is not None:
        assert " NTW=%d " % ntw in gpu.debug_last_launch(), gpu.debug_last_launch()
    else:
        assert " S=%d " % (-(-d_in // 4096)) in gpu.debug_last_launch(), gpu.debug_last_launch()
    _check(y, c.oracle_y())


@pytest.mark.parametrize("w_bits,ab_bits,M,d_in,d_outs,r", [
    (4, 16, 16, 2048, (512, 256, 256), 128),
    (3, 16, 10, 4096, (1024, 1024), 64),
    (4, 4, 12, 2048, (256, 512, 256, 128), 128),
    (2, 16, 16, 1024, (256, 256, 256, 256), 0),
    (4, 16, 16, 14336, (1024, 512), 128),      # two members, four ranges
])
def test_stream_groups(gpu, w_bits, ab_bits, M, d_in, d_outs, r):
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_group
    cases = [QCase(5300 + 11 * i + M, d_in, d, M, r, w_bits, ab_bits=ab_bits, packer=gpu) for i, d in enumerate(d_outs)]
    ys = run_linear_q_group(cases, cases[0].x)
    assert gpu.debug_last_launch().startswith("resident FM=%d " % {4: 1, 3: 2, 2: 6}[w_bits]), gpu.debug_last_launch()
    assert " n=%d " % len(d_outs) in gpu.debug_last_launch()
    for c, y in zip(cases, ys):
        _check(y, c.oracle_y(x=cases[0].x))


@pytest.mark.parametrize("M", list(range(5, 17)))
def test_stream_every_token_count(gpu, M):
    """Every token count the kernel serves, on one small layer with a rank that is not a power of two (rows beyond
    the tokens are not staged; what LDS holds there reaches only accumulator rows that are never stored)."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(6000 + M, 2048, 768, M, 96, 3, packer=gpu)
    y = run_linear_q(c)
    assert gpu.debug_last_launch().startswith("resident FM=2 "), gpu.debug_last_launch()
    _check(y, c.oracle_y())


def test_stream_result_is_independent_of_timing(gpu):
    """The partial tiles are added in the order of the ranges: repeated calls agree bit for bit."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(5501, 4096, 2048, 16, 128, 4, packer=gpu)
    ws = gpu.new_workspace(16, 4096, 2048, 128)
    first = run_linear_q(c, ws=ws)
    for _ in range(5):
        again = run_linear_q(c, ws=ws)
        assert np.array_equal(first.view(np.uint16), again.view(np.uint16))
    assert gpu.workspace_error(ws) == 0


def test_stream_workspace_shared_by_different_calls(gpu):
    """One workspace, never cleared in between: different inputs, shapes, token counts and kernels in a row (a stale
    partial tile or t of an earlier call carries an older tag and is never taken for this call's)."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    a = QCase(5601, 4096, 1024, 16, 128, 4, packer=gpu)
    b = QCase(5602, 2048, 1024, 9, 128, 4, packer=gpu)
    d = QCase(5603, 4096, 1024, 1, 128, 4, packer=gpu)          # the decode kernel, same workspace
    ws = gpu.new_workspace(16, 4096, 1024, 128)
    x2 = synth.draw_layer(5604, 4096, 16, 16, 0)[3]
    for c, x in ((a, a.x), (b, b.x), (a, x2), (d, d.x), (b, b.x[::-1].copy()), (a, a.x)):
        y = run_linear_q(c, x=x, ws=ws)
        _check(y, c.oracle_y(x=x))
    assert gpu.workspace_error(ws) == 0


def test_few_rows_take_the_other_kernel_by_default(gpu):
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(5901, 4096, 2048, 16, 128, 4, packer=gpu)         # 128 row blocks: below the crossover (256)
    gpu.debug_set_resident_min_blocks(-1)
    try:
        y = run_linear_q(c)
        assert gpu.debug_last_launch().startswith("wide_q"), gpu.debug_last_launch()
    finally:
        gpu.debug_set_resident_min_blocks(0)
    _check(y, c.oracle_y())


def test_stream_expired_wait_for_t(gpu):
    """A negative spin limit makes every wait for t count as expired at once: the call reports the timeout, y holds
    the backbone's product alone, and after a re-initialisation the workspace serves the call again."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(5801, 2048, 512, 16, 128, 4, packer=gpu)
    ws = gpu.new_workspace(16, 2048, 512, 128)
    gpu.debug_set_spin_limit(-1)
    try:
        y = run_linear_q(c, ws=ws)
        assert gpu.debug_last_launch().startswith("resident"), gpu.debug_last_launch()
        assert gpu.workspace_error(ws) == -8
        _check(y, c.oracle_y(r=0))
    finally:
        gpu.debug_set_spin_limit(1 << 22)
    gpu.workspace_init(ws)
    _check(run_linear_q(c, ws=ws), c.oracle_y())
    assert gpu.workspace_error(ws) == 0
