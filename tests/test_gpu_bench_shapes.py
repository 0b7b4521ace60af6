"""GPU parity at the shapes bench.py launches, in the launch configuration it times: the full d_out and d_in
of the 70B-shaped 2:4 linears at 64 tokens (so that the many-token kernel's eight-row-block instantiations are
the ones that run), the 8B down projection and the query/key/value group at 2048 tokens.  The kernel each call
chose is asserted through eora_debug_last_launch, so a change of a picker's limits cannot silently leave an
instantiation untested.  The oracle is evaluated on sampled 16-row blocks (rows of a tile-major operand are
stored row block by row block, so the stored bytes of a sample of row blocks are slices of the full operand's)
over all token rows, or on sampled token rows over all outputs."""
import functools

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


@functools.lru_cache(maxsize=2)
def _pruned(seed, d_in, d_out, M, r):
    """Logical 2:4 layer at full size (drawn and pruned once per shape; the fp16 and the 4-bit test share it)."""
    import synth
    W, A, B, x = synth.draw_layer(seed, d_in, d_out, M, r)
    vals, pos = synth.prune_24(W.astype(np.float16))
    return vals, pos, A, B, x


def _sample_blocks(d_out, nw, extra=()):
    """Row blocks to check: first, last, both sides of a workgroup's group of nw row blocks, a few seeded ones."""
    nb = d_out // 16
    rng = np.random.default_rng(d_out + nw)
    pick = {0, 1, nw - 1, nw, nb - nw, nb - 1, *extra, *rng.integers(0, nb, 6).tolist()}
    return sorted(b for b in pick if 0 <= b < nb)


def _rows_of(blocks):
    return np.concatenate([np.arange(16 * b, 16 * b + 16) for b in blocks])


def _check(y, ref):
    from oracle import linear
    assert np.all(np.isfinite(y.astype(np.float32)))
    err = linear.y_error(y, ref)
    assert err <= TOL, err


def _run_sparse(gpu, quantised, seed, d_in, d_out, M, r, want, nw):
    """One 2:4 linear at full size through the C ABI; oracle on sampled row blocks, all tokens."""
    import synth
    import torch
    from oracle import layout, linear
    from tests.gpu_util import dev
    vals, pos, A, B, x = _pruned(seed, d_in, d_out, M, r)
    blocks = _sample_blocks(d_out, nw)
    rows = _rows_of(blocks)
    G = d_in // 128
    A_t, B_t = gpu.pack_factor_f16(A), gpu.pack_factor_f16(B)
    oA, oB = layout.pack_f16(A), layout.pack_f16(B[rows])
    ws = gpu.new_workspace(M, d_in, d_out, r)
    y = torch.full((M, d_out), 777.0, dtype=torch.float16, device="cuda")
    if quantised:
        codes, zeros, scales = synth.quantize_kept_rtn(vals, pos, 128)
        tiles, meta = gpu.pack_sp24q4(codes, pos, zeros, scales, 128)
        o_tiles, o_meta = layout.pack_sp24q4(codes[rows], pos[rows], zeros[rows], scales[rows], 128)
        for i, b in enumerate(blocks):           # the library's stored bytes of the sampled row blocks are the oracle's
            assert np.array_equal(tiles[b * G * 192:(b + 1) * G * 192], o_tiles[i * G * 192:(i + 1) * G * 192])
            assert np.array_equal(meta[b * G * 16:(b + 1) * G * 16], o_meta[i * G * 16:(i + 1) * G * 16])
        gpu.linear_sp24q4(dev(x), dev(tiles), dev(meta), dev(A_t), dev(B_t), y, M, d_in, d_out, r, ws)
        ref = linear.eora_linear_sp24q4(x, o_tiles, o_meta, oA, oB, M, d_in, len(rows), r)
    else:
        values, indices = gpu.pack_sp24(vals, pos)
        o_values, o_indices = layout.pack_sp24(vals[rows], pos[rows])
        for i, b in enumerate(blocks):
            assert np.array_equal(values[b * G * 1024:(b + 1) * G * 1024].view(np.uint16),
                                  o_values[i * G * 1024:(i + 1) * G * 1024].view(np.uint16))
            assert np.array_equal(indices[b * G * 64:(b + 1) * G * 64], o_indices[i * G * 64:(i + 1) * G * 64])
        gpu.linear_sp24(dev(x), dev(values), dev(indices), dev(A_t), dev(B_t), y, M, d_in, d_out, r, ws)
        ref = linear.eora_linear_sp24(x, o_values, o_indices, oA, oB, M, d_in, len(rows), r)
    torch.cuda.synchronize()
    assert gpu.debug_last_launch() == want, gpu.debug_last_launch()
    assert gpu.workspace_error(ws) == 0
    got = y.cpu().numpy()
    _check(got[:, rows], ref)
    # rows outside the sample: written (no canary left), finite
    assert not np.any(got == 777.0) and np.all(np.isfinite(got.astype(np.float32)))


@pytest.mark.parametrize("quantised", [False, True])
@pytest.mark.parametrize("name,d_in,d_out,M,nw,tb,ks", [
    ("gate", 8192, 28672, 64, 8, 4, 1),      # config 5 at 64 tokens: eight row blocks x four token blocks per workgroup
    ("q", 8192, 8192, 64, 4, 2, 1),          # four row blocks x two token blocks
    ("down", 28672, 8192, 64, 8, 4, 4),      # the 28672-long contraction: four ranges of it in different workgroups
    ("down48", 28672, 8192, 48, 8, 2, 2),    # three token blocks, two ranges
    ("long", 16384, 4096, 37, 8, 2, 4),      # the shortest contraction that is split; ragged tokens
    ("mid", 8192, 14336, 64, 8, 2, 1),       # a row count that selects eight row blocks x two token blocks
    ("gate48", 8192, 28672, 48, 8, 2, 1),    # three token blocks (two per workgroup, the last group ragged)
])
def test_sparse_many_tokens_at_bench_shapes(gpu, quantised, name, d_in, d_out, M, nw, tb, ks):
    import synth
    want = "sparse_wide FA=5 NW=%d TB=%d VQ=%d n=1 ksplit=%d" % (nw, tb, int(quantised), ks)
    _run_sparse(gpu, quantised, synth.seed_for(5, {"gate": 4, "q": 0, "down": 6, "down48": 6, "long": 8, "mid": 7, "gate48": 4}[name]),
                d_in, d_out, M, 128, want, nw)


@pytest.mark.parametrize("quantised", [False, True])
def test_sparse_group_gate_up_at_bench_shape(gpu, quantised):
    """The gate + up launch of the grouped 70B workload at 64 tokens (both members 8192 -> 28672)."""
    import synth
    import torch
    from oracle import layout, linear
    from tests.gpu_util import dev
    d_in, d_out, M, r = 8192, 28672, 64, 128
    vals, pos, A, B, x = _pruned(synth.seed_for(5, 4), d_in, d_out, M, r)
    blocks = _sample_blocks(d_out, 8)
    rows = _rows_of(blocks)
    A_t, B_t = dev(gpu.pack_factor_f16(A)), dev(gpu.pack_factor_f16(B))
    oA, oB = layout.pack_f16(A), layout.pack_f16(B[rows])
    if quantised:
        codes, zeros, scales = synth.quantize_kept_rtn(vals, pos, 128)
        tiles, meta = gpu.pack_sp24q4(codes, pos, zeros, scales, 128)
        stored = (None, None, dev(tiles), dev(meta))
        o_tiles, o_meta = layout.pack_sp24q4(codes[rows], pos[rows], zeros[rows], scales[rows], 128)
        ref = linear.eora_linear_sp24q4(x, o_tiles, o_meta, oA, oB, M, d_in, len(rows), r)
    else:
        values, indices = gpu.pack_sp24(vals, pos)
        stored = (dev(values), dev(indices), None, None)
        o_values, o_indices = layout.pack_sp24(vals[rows], pos[rows])
        ref = linear.eora_linear_sp24(x, o_values, o_indices, oA, oB, M, d_in, len(rows), r)
    # both members read the same stored operands (the launch is what is under test) into outputs of their own
    ys = [torch.full((M, d_out), 777.0, dtype=torch.float16, device="cuda") for _ in range(2)]
    ws = gpu.new_workspace(M, d_in, d_out, r)
    gpu.linear_sp24_group(dev(x), [stored + (A_t, B_t, y, d_out) for y in ys], M, d_in, r, ws)
    torch.cuda.synchronize()
    assert gpu.debug_last_launch() == "sparse_wide FA=5 NW=16 TB=4 VQ=%d n=2 ksplit=1" % int(quantised), gpu.debug_last_launch()
    assert gpu.workspace_error(ws) == 0
    for y in ys:
        _check(y.cpu().numpy()[:, rows], ref)
    assert torch.equal(ys[0], ys[1])


def _token_rows(M, seed, n):
    fixed = np.array([0, 1, 127, 128, 255, 256, M // 2 - 1, M // 2, M - 2, M - 1])
    return np.unique(np.concatenate([fixed, np.random.default_rng(seed).integers(0, M, n)]))


def test_prefill_config4_down_projection(gpu):
    """BASELINE config 4, the down projection: 14336 -> 4096 at 2048 tokens (112 k-steps), 4-bit backbone, fp16
    rank-256 factors, 1 % outlier channels scaled by 20.  Sampled token rows, all outputs."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q
    c = QCase(synth.seed_for(4, 6), 14336, 4096, 2048, 256, 4, outlier_frac=0.01, packer=gpu)
    y = run_linear_q(c)
    assert gpu.debug_last_launch().startswith("prefill FM=1 EXT=1"), gpu.debug_last_launch()
    rows = _token_rows(2048, 3, 22)
    _check(y[rows], c.oracle_y(rows=rows))


def test_prefill_config4_qkv_group(gpu):
    """BASELINE config 4, query + key + value (4096 -> 4096, 1024, 1024) as one grouped call at 2048 tokens:
    the launch bench.py times.  Sampled token rows, all outputs of the three members."""
    import synth
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_group
    cs = [QCase(synth.seed_for(4, i), 4096, d, 2048, 256, 4, outlier_frac=0.01, packer=gpu) for i, d in enumerate((4096, 1024, 1024))]
    ys = run_linear_q_group(cs, cs[0].x)
    assert gpu.debug_last_launch() == "prefill FM=1 EXT=1 ksplit=1 n=3 FE=5", gpu.debug_last_launch()
    rows = _token_rows(2048, 4, 14)
    for c, y in zip(cs, ys):
        _check(y[rows], c.oracle_y(rows=rows, x=cs[0].x))


@pytest.mark.parametrize("w_bits,ab_bits,M,d_in,d_outs,want", [
    (3, 16, 1, 4096, (14336, 14336), "small FM=2 FA=5 NW=4 NQ=2 RB=2 n=2 c2=768"),     # default workload: gate + up, strips of two then single row blocks
    (3, 16, 1, 4096, (4096, 1024, 1024), "small FM=2 FA=5 NW=4 NQ=2 RB=1 n=3 c2=-1"),  # query + key + value
    (3, 16, 1, 4096, (28672,), "small FM=2 FA=5 NW=4 NQ=2 RB=2 n=1 c2=768"),           # mixed strips, one member
    (3, 4, 1, 4096, (13312, 13312), "small FM=2 FA=3 NW=4 NQ=2 RB=2 n=2 c2=768"),      # fewest single row blocks a mixed launch takes (128), 4-bit factors
    (2, 16, 1, 4096, (16384, 8192, 8192), "small FM=6 FA=5 NW=4 NQ=2 RB=2 n=3 c2=768"),  # most (512), three members, 2-bit backbone
    (3, 16, 1, 4096, (16384, 16416), "small FM=2 FA=5 NW=4 NQ=2 RB=2 n=2 c2=-1"),      # too many row blocks for mixed strips: strips of two throughout
    (4, 16, 1, 4096, (14336, 14336), "small FM=1 FA=5 NW=4 NQ=2 RB=2 n=2 c2=-1"),      # 4-bit backbone, fp16 factors: no kernel with both strip lengths (registers)
    (4, 4, 1, 4096, (14336, 14336), "small FM=1 FA=3 NW=4 NQ=2 RB=2 n=2 c2=768"),      # 4-bit backbone, 4-bit factors: mixed strips without the early look at t
    (4, 16, 16, 4096, (14336, 14336), "resident FM=1 FA=5 NTW=8 n=2 wgs=232 q=8"),      # config 1 shapes at 16 tokens, grouped
    (4, 16, 64, 4096, (14336, 14336), "wide_q FM=1 FA=5 NWR=4 NWK=2 TB=4 n=2"),  # four token blocks per workgroup
    (4, 16, 16, 4096, (4096,), None),                                             # 256 row blocks: the smallest launch the resident kernel takes
    (4, 16, 16, 4096, (4080,), None),                                             # one row block fewer: the kernel for 5..127 tokens
])
def test_quantised_groups_reach_their_kernels(gpu, w_bits, ab_bits, M, d_in, d_outs, want):
    """The grouped launches of the decode workloads choose the instantiations the profiles name."""
    from tests.cases import QCase
    from tests.gpu_util import run_linear_q_group
    cases = [QCase(700 + 7 * i + M, d_in, d, M, 128, w_bits, ab_bits=ab_bits, packer=gpu) for i, d in enumerate(d_outs)]
    ys = run_linear_q_group(cases, cases[0].x)
    if want is None:
        want_resident = sum(d_outs) // 16 >= 256
        assert gpu.debug_last_launch().startswith("resident ") == want_resident, gpu.debug_last_launch()
    else:
        assert gpu.debug_last_launch() == want, gpu.debug_last_launch()
    for c, y in zip(cases, ys):
        _check(y, c.oracle_y(x=cases[0].x))
