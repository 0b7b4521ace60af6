"""eora_linear_q_static (the entry point for callers that cannot allocate: its workspace is an array inside the
library's device code) against eora_linear_q with a caller-provided workspace, through the C ABI: same kernels,
so the outputs must be bit-identical; and against the oracle to the usual bound.  Two calls in a row on the shared
array, the second with a smaller input, then more shapes (every kernel family below 128 tokens)."""
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


def _static(gpu, c):
    import torch
    from tests.gpu_util import dev
    pad = 64
    ybuf = torch.full((c.M * c.d_out + 2 * pad,), 777.0, dtype=torch.float16, device="cuda")
    y = ybuf[pad: pad + c.M * c.d_out]
    fac = (dev(c.A), dev(c.B), dev(c.As), dev(c.Bs)) if c.r > 0 else (None, None, None, None)
    gpu.linear_q_static(dev(c.x), dev(c.qw), dev(c.sc), dev(c.qz), *fac, y, c.M, c.d_in, c.d_out, c.r, c.w_bits, c.group, c.ab_bits)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    assert np.all(out[:pad] == 777.0) and np.all(out[pad + c.M * c.d_out:] == 777.0), "write outside y"
    return out[pad: pad + c.M * c.d_out].reshape(c.M, c.d_out)


def test_static_workspace_entry_point_two_calls_in_a_row(gpu):
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    big = QCase(51, 4096, 1024, 3, 128, 4, packer=gpu)           # decode kernel, low-rank hand-over through the array
    small = QCase(52, 1024, 256, 1, 32, 3, packer=gpu)           # smaller in every size
    y_big, y_small = _static(gpu, big), _static(gpu, small)      # back to back on the one shared array
    assert np.array_equal(y_big, run_linear_q(big))
    assert np.array_equal(y_small, run_linear_q(small))
    assert linear.y_error(y_big, big.oracle_y()) <= TOL and linear.y_error(y_small, small.oracle_y()) <= TOL
    assert np.array_equal(_static(gpu, big), y_big)              # and the larger one again after the smaller


@pytest.mark.parametrize("w_bits,ab_bits,r,M,d_in,d_out", [
    (4, 16, 128, 16, 2048, 8192),      # the kernel for 5..127 tokens
    (3, 4, 64, 37, 640, 112),          # the general kernel (d_in not a multiple of 512), ragged token blocks
    (2, 16, 0, 2, 1024, 64),           # adapter off
    (4, 3, 128, 127, 512, 96),         # the most tokens the entry point takes
])
def test_static_workspace_entry_point_kernel_families(gpu, w_bits, ab_bits, r, M, d_in, d_out):
    from oracle import linear
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(60 + M, d_in, d_out, M, r, w_bits, ab_bits=ab_bits, packer=gpu)
    y = _static(gpu, c)
    assert np.array_equal(y, run_linear_q(c))
    assert linear.y_error(y, c.oracle_y()) <= TOL


def test_static_workspace_entry_point_rejects_what_it_cannot_serve(gpu):
    import torch
    from tests.cases import QCase
    from tests.gpu_util import dev
    c = QCase(70, 512, 64, 128, 0, 4, packer=gpu)                # 128 tokens: beyond the array's limit
    y = torch.full((c.M, c.d_out), 777.0, dtype=torch.float16, device="cuda")
    with pytest.raises(gpu.EoraError) as e:
        gpu.linear_q_static(dev(c.x), dev(c.qw), dev(c.sc), dev(c.qz), None, None, None, None, y, c.M, c.d_in, c.d_out, 0, 4, 128, 16)
    assert e.value.status == -5
    with pytest.raises(gpu.EoraError) as e:                      # the usual validation still applies
        gpu.linear_q_static(dev(c.x), dev(c.qw), dev(c.sc), dev(c.qz), None, None, None, None, y, 4, c.d_in, 60, 0, 4, 128, 16)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert torch.all(y == 777.0)                                 # nothing was enqueued
