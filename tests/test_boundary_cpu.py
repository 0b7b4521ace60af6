"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, its host packers emit exactly the oracle's bytes, and argument validation returns the
documented codes before anything touches a device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2410_21271_amd as eora
from paper_2410_21271_amd import binding
from tests.cases import QCase, SparseCase

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "eora.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(eora_[a-z0-9_]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(binding.EXPORTS)
    raw = ctypes.CDLL(eora.lib_path())
    for name in declared:
        assert getattr(raw, name) is not None


@pytest.mark.parametrize("w_bits,ab_bits,r", [(4, 16, 32), (3, 16, 64), (4, 4, 64), (3, 4, 128), (4, 16, 0), (2, 16, 32), (4, 3, 128)])
def test_host_packers_match_oracle_bytes(w_bits, ab_bits, r):
    QCase(100 + w_bits + r, 256, 48, 2, r, w_bits, 128, ab_bits, packer=eora)      # asserts inside
    QCase(200 + w_bits + r, 256, 32, 1, r, w_bits, 256, ab_bits, packer=eora)      # channel-wise group


def test_sparse_packer_matches_oracle_bytes():
    SparseCase(7, 256, 32, 1, 32, packer=eora)
    from tests.cases import SparseQCase
    SparseQCase(8, 512, 32, 1, 32, packer=eora)             # host packer = oracle layout, word for word
    SparseQCase(9, 512, 32, 1, 0, group=256, packer=eora)


def test_sizes():
    assert eora.qweight_bytes(4096, 4096, 4) == 4096 * 4096 // 2
    assert eora.qweight_bytes(4096, 4096, 3) == 4096 * 4096 * 3 // 8
    assert eora.qweight_bytes(4096, 4096, 2) == 4096 * 4096 // 4 and eora.qweight_bytes(4096, 4096, 1) == 0
    assert eora.qzeros_bytes(4096, 4096, 128) == 4096 * 32 // 2
    assert eora.qzeros_bytes(4096, 4096, 4096) == 4096 * 4          # channel-wise: one padded word per row
    assert eora.scales_bytes(4096, 4096, 128) == 4096 * 32 * 2
    assert eora.sp24_values_bytes(8192, 1024) == 8192 * 1024
    assert eora.sp24_indices_bytes(8192, 1024) == 8192 * 1024 // 8
    assert eora.sp24q4_tiles_bytes(8192, 1024) == 8192 * 1024 * 3 // 8 and eora.sp24q4_tiles_bytes(8192, 1000) == 0
    assert eora.sp24q4_meta_bytes(8192, 1024) == 1024 * 64 * 4
    assert eora.qweight_bytes(4096, 4100, 4) == 0 and eora.qweight_bytes(4096, 4096, 5) == 0
    assert eora.workspace_bytes(1, 4096, 4096, 128) >= 4 * 128
    assert eora.workspace_bytes(1, 4096, 4096, 1024) == 0


def test_packers_reject_bad_values():
    codes = np.zeros((16, 128), np.uint8)
    zeros = np.zeros((16, 1), np.uint8)
    scales = np.ones((16, 1), np.float16)
    codes[3, 5] = 8
    with pytest.raises(eora.EoraError) as ei:
        eora.pack_q(codes, zeros, scales, 3, 128)
    assert ei.value.status == -7
    eora.pack_q(codes, zeros, scales, 4, 128)
    zeros[0, 0] = 16
    with pytest.raises(eora.EoraError):
        eora.pack_q(codes, zeros, scales, 4, 128)
    with pytest.raises(eora.EoraError):
        eora.pack_sp24(np.zeros((16, 64), np.float16), np.zeros((16, 64), np.uint8))
    with pytest.raises(eora.EoraError):
        eora.pack_factor_f16(np.zeros((8, 32), np.float16))
    pos = np.tile(np.array([0, 1], np.uint8), (16, 32))
    c4 = np.zeros((16, 64), np.uint8)
    eora.pack_sp24q4(c4, pos, np.zeros((16, 1), np.uint8), np.ones((16, 1), np.float16), 128)
    c4[2, 7] = 16
    with pytest.raises(eora.EoraError) as ei:
        eora.pack_sp24q4(c4, pos, np.zeros((16, 1), np.uint8), np.ones((16, 1), np.float16), 128)
    assert ei.value.status == -7


def test_linear_q_validation_codes():
    """Every error path returns before a launch, so these calls are safe without a GPU: the
    pointers are never dereferenced."""
    L = eora.lib
    good = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    null = ctypes.c_void_p(0)

    def call(x=good, qw=good, sc=good, qz=good, A=good, B=good, As=null, Bs=null, y=good, M=1, d_in=256, d_out=32,
             r=32, w_bits=4, group=128, ab_bits=16, ws=good, ws_bytes=1 << 24):
        return L.eora_linear_q(x, qw, sc, qz, A, B, As, Bs, y, M, d_in, d_out, r, w_bits, group, ab_bits, ws,
                               ws_bytes, null)

    assert call(x=null) == -1 and call(y=null) == -1 and call(A=null) == -1
    assert call(d_out=40) == -2 and call(d_in=200) == -2 and call(group=64) == -2 and call(group=384) == -2
    assert call(r=48) == -2 and call(r=1024) == -2 and call(M=-1) == -2
    assert call(w_bits=1) == -3 and call(w_bits=5) == -3 and call(ab_bits=8) == -3
    assert call(ab_bits=4, As=good, Bs=good, r=96) == -2 and call(ab_bits=4, r=64) == -1
    assert call(ab_bits=3, As=good, Bs=good, r=64) == -2 and call(ab_bits=3, r=128) == -1
    assert call(qw=odd) == -4 and call(y=odd) == -4 and call(ws=odd) == -4
    assert call(ws=null) == -5 and call(ws_bytes=16) == -5
    assert call(M=0) == 0                                   # empty input: nothing to do, nothing launched
    assert L.eora_linear_sp24(null, good, good, good, good, good, 1, 256, 32, 32, good, 1 << 24, null) == -1
    assert L.eora_linear_sp24(good, good, good, good, good, good, 1, 256, 32, 48, good, 1 << 24, null) == -2
    assert L.eora_linear_sp24(good, good, odd, good, good, good, 1, 256, 32, 32, good, 1 << 24, null) == -4
    assert L.eora_linear_sp24(good, good, good, good, good, good, 1, 256, 32, 32, good, 16, null) == -5
    # a group of layers that share x: validated member by member before anything is enqueued
    Q = eora.binding.QMember
    g, n0 = 0x1000, None

    def group(members, n=None, M=1, d_in=512, r=32, w_bits=4, group_=128, ab_bits=16, ws=good, ws_bytes=1 << 24, x=good):
        arr = (Q * max(1, len(members)))(*members)
        return L.eora_linear_q_group(x, arr, len(members) if n is None else n, M, d_in, r, w_bits, group_, ab_bits, ws,
                                     ws_bytes, null)

    ok = Q(g, g, g, g, g, n0, n0, g, 32)
    assert group([ok], n=0) == -2 and group([ok] * 5) == -2 and group([ok], x=null) == -1
    assert group([ok, Q(g, g, g, g, g, n0, n0, n0, 32)]) == -1            # second member without y
    assert group([ok, Q(g, g, g, g, g, n0, n0, g, 40)]) == -2             # d_out not a multiple of 16
    assert group([ok, Q(g, 0x1008, g, g, g, n0, n0, g, 32)]) == -4
    assert group([ok, ok], w_bits=5) == -3 and group([ok, ok], ws_bytes=16) == -5 and group([ok, ok], ws=null) == -5
    assert group([ok, ok], M=8, d_in=256, ws_bytes=16) == -5              # the member-by-member path validates too
    assert group([ok, ok], M=0) == 0
    assert L.eora_unpack_q(good, good, good, good, 256, 32, 5, 128, null) == -3
    assert L.eora_dequant_q(good, good, good, null, 256, 32, 4, 128, null) == -1
    assert L.eora_expand_sp24(good, odd, good, 256, 32, null) == -4
    sq = L.eora_linear_sp24q4
    assert sq(good, null, good, good, good, good, 1, 256, 32, 32, good, 1 << 24, null) == -1
    assert sq(good, good, good, good, good, good, 1, 200, 32, 32, good, 1 << 24, null) == -2
    assert sq(good, good, good, good, good, good, 1, 256, 32, 48, good, 1 << 24, null) == -2
    assert sq(good, odd, good, good, good, good, 1, 256, 32, 32, good, 1 << 24, null) == -4
    assert sq(good, good, good, good, good, good, 1, 256, 32, 32, good, 16, null) == -5
    assert sq(good, good, good, good, good, good, 0, 256, 32, 32, good, 1 << 24, null) == 0
    assert L.eora_expand_sp24q4(good, good, null, 256, 32, null) == -1
    assert L.eora_expand_sp24q4(good, good, good, 256, 40, null) == -2
    assert eora.status_string(-4) == "misaligned pointer"


def test_factors_validation_codes_and_sizes():
    """eora_factors validates before its first launch (no pointer is dereferenced on these paths)."""
    L = eora.lib
    good, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_void_p(0)

    def call(W=good, Wh=good, Xt=good, n=8, d_in=128, d_out=64, r=8, floor=1e-12, B=good, A=good, ws=good, ws_bytes=1 << 30):
        return L.eora_factors(W, Wh, Xt, n, d_in, d_out, r, floor, B, A, null, ws, ws_bytes, null, None)

    assert call(W=null) == -1 and call(Xt=null) == -1 and call(A=null) == -1
    assert call(d_in=127) == -2 and call(d_out=16386) == -2 and call(r=0) == -2 and call(r=65) == -2 and call(n=0) == -2
    assert call(floor=1.0) == -7 and call(floor=-1e-3) == -7 and call(floor=float("nan")) == -7
    assert call(ws=null) == -5 and call(ws_bytes=1 << 10) == -5 and call(ws=odd) == -4
    # five fp64 matrices (dW, G, V, dW', its copy) plus vectors and the r-row staging buffers
    n = eora.factors_workspace_bytes(4096, 4096, 128)
    assert 5 * 8 * 4096 * 4096 <= n <= 5 * 8 * 4096 * 4096 + (1 << 24)
    assert eora.factors_workspace_bytes(4096, 4097, 128) == 0 and eora.factors_workspace_bytes(64, 64, 65) == 0
    assert eora.status_string(-9) == "Jacobi sweeps did not converge"


def test_linear_q_multi_validation_codes():
    L = eora.lib
    good, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1002), ctypes.c_void_p(0)

    def call(sel=good, A=good, M=4, r=32, n=2, w_bits=4, ab_bits=16, As=null, Bs=null, ws=good, ws_bytes=1 << 24):
        return L.eora_linear_q_multi(good, good, good, good, A, good, As, Bs, sel, good, M, 256, 32, r, n, w_bits, 128, ab_bits,
                                     ws, ws_bytes, null)

    assert call(sel=null) == -1 and call(A=null) == -1 and call(sel=odd) == -4
    assert call(n=0) == -2 and call(r=16) == -2 and call(r=0) == -2 and call(n=17) == -2
    assert call(ab_bits=4, r=64, As=good, Bs=good) == -2 and call(ab_bits=4, r=128, n=2) == -1
    assert call(w_bits=5) == -3 and call(ws=null) == -5 and call(ws_bytes=16) == -5
    assert call(M=0) == 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's share; asking for more ends with a message and a non-zero status
    before anything touches a GPU."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "not supported" in p.stderr and p.stdout.strip() == ""


def test_factors_store_f16_validation_codes():
    L = eora.lib
    good, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_void_p(0)

    def call(B=good, A=good, d_in=256, d_out=32, r=32, balance=1, At=good, Bt=good, scratch=good, nbytes=8 * 32):
        return L.eora_factors_store_f16(B, A, d_in, d_out, r, balance, At, Bt, scratch, nbytes, null)

    assert call(B=null) == -1 and call(At=null) == -1
    assert call(d_in=250) == -2 and call(d_out=24) == -2 and call(r=16) == -2 and call(r=0) == -2
    assert call(At=odd) == -4 and call(scratch=odd) == -4
    assert call(scratch=null) == -5 and call(nbytes=8 * 31) == -5


def test_factors_store_q_validation_codes():
    L = eora.lib
    good, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_void_p(0)

    def call(B=good, A=good, d_in=256, d_out=32, r=128, bits=4, balance=1, Aq=good, As=good, Bq=good, Bs=good, scratch=good,
             nbytes=8 * 128):
        return L.eora_factors_store_q(B, A, d_in, d_out, r, bits, balance, Aq, As, Bq, Bs, scratch, nbytes, null)

    assert call(B=null) == -1 and call(As=null) == -1 and call(bits=16) == -3 and call(bits=2) == -3
    assert call(d_in=192) == -2 and call(d_out=24) == -2 and call(r=96) == -2 and call(r=64, bits=3) == -2
    assert call(Bq=odd) == -4 and call(scratch=null) == -5 and call(nbytes=8) == -5


def test_linear_sp24_group_validation_codes():
    L = eora.lib
    S = eora.binding.SpMember
    g, null = 0x1000, ctypes.c_void_p(0)
    good = ctypes.c_void_p(g)

    def call(members, n=None, M=1, d_in=256, r=32, ws=good, ws_bytes=1 << 24, x=good):
        arr = (S * max(1, len(members)))(*members)
        return L.eora_linear_sp24_group(x, arr, len(members) if n is None else n, M, d_in, r, ws, ws_bytes, null)

    fp = S(g, g, None, None, g, g, g, 32)
    q4 = S(None, None, g, g, g, g, g, 32)
    # (only error paths and the empty batch are called: nothing here may reach a launch)
    assert call([fp], n=0) == -2 and call([fp] * 5) == -2 and call([fp], x=null) == -1
    assert call([fp, q4]) == -1                                   # members of different kinds
    assert call([fp, S(g, g, None, None, g, g, None, 32)]) == -1  # no y
    assert call([q4, S(None, None, g, g, g, g, g, 40)]) == -2
    assert call([fp, S(g, 0x1008, None, None, g, g, g, 32)]) == -4
    assert call([fp, fp], r=48) == -2 and call([fp, fp], ws=null) == -5 and call([fp, fp], ws_bytes=16) == -5
    assert call([fp, fp], M=0) == 0
