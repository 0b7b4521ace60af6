"""Builds one layer's inputs for the parity tests: logical arrays from the seeded generators,
stored bytes from BOTH packers (the oracle's, fed to the oracle; the library's host packer, fed
to the GPU), with the two byte streams asserted identical."""
import numpy as np

import synth
from oracle import layout


class QCase:
    """Quantised-backbone layer.  ab_bits: 16 or 4; r = 0 for the bare layer."""

    def __init__(self, seed, d_in, d_out, M, r, w_bits, group=128, ab_bits=16, outlier_frac=0.0, packer=None):
        self.d_in, self.d_out, self.M, self.r = d_in, d_out, M, r
        self.w_bits, self.group, self.ab_bits = w_bits, group, ab_bits
        W, A, B, x = synth.draw_layer(seed, d_in, d_out, M, r, outlier_frac)
        codes, zeros, scales = synth.quantize_rtn(W, w_bits, group)
        self.logical = dict(codes=codes, zeros=zeros, scales=scales, A=A, B=B)
        self.x = x
        # oracle side
        self.o_qw = {4: layout.pack_q4, 3: layout.pack_q3, 2: layout.pack_q2}[w_bits](codes)
        self.o_qz, self.o_sc = layout.pack_zeros(zeros), layout.pack_scales(scales)
        self.o_A = self.o_B = self.o_As = self.o_Bs = None
        if r > 0 and ab_bits == 16:
            self.o_A, self.o_B = layout.pack_f16(A), layout.pack_f16(B)
        elif r > 0 and ab_bits == 3:
            ca, sa = synth.quantize_sym3(A)
            cb, sb = synth.quantize_sym3(B)
            self.logical.update(ca=ca, sa=sa, cb=cb, sb=sb)
            self.o_A, self.o_As = layout.pack_q3(ca), layout.pack_scales(sa)
            self.o_B, self.o_Bs = layout.pack_q3(cb), layout.pack_scales(sb)
        elif r > 0:
            KTb = min(128, r)
            ca, sa = synth.quantize_sym4(A, 128)
            cb, sb = synth.quantize_sym4(B, KTb)
            self.logical.update(ca=ca, sa=sa, cb=cb, sb=sb)
            self.o_A, self.o_As = layout.pack_q4(ca, 128), layout.pack_scales(sa)
            self.o_B, self.o_Bs = layout.pack_q4(cb, KTb), layout.pack_scales(sb)
        # library side
        if packer is not None:
            self.pack_with(packer)

    def pack_with(self, e):
        L = self.logical
        self.qw, self.qz, self.sc = e.pack_q(L["codes"], L["zeros"], L["scales"], self.w_bits, self.group)
        assert np.array_equal(self.qw, self.o_qw) and np.array_equal(self.qz, self.o_qz)
        assert np.array_equal(self.sc.view(np.uint16), self.o_sc.view(np.uint16))
        self.A = self.B = self.As = self.Bs = None
        if self.r > 0 and self.ab_bits == 16:
            self.A, self.B = e.pack_factor_f16(L["A"]), e.pack_factor_f16(L["B"])
            assert np.array_equal(self.A.view(np.uint16), self.o_A.view(np.uint16))
            assert np.array_equal(self.B.view(np.uint16), self.o_B.view(np.uint16))
        elif self.r > 0:
            pack = e.pack_factor_q3 if self.ab_bits == 3 else e.pack_factor_q4
            self.A, self.As = pack(L["ca"], L["sa"])
            self.B, self.Bs = pack(L["cb"], L["sb"])
            assert np.array_equal(self.A, self.o_A) and np.array_equal(self.B, self.o_B)
            assert np.array_equal(self.As.view(np.uint16), self.o_As.view(np.uint16))
            assert np.array_equal(self.Bs.view(np.uint16), self.o_Bs.view(np.uint16))

    def oracle_y(self, rows=None, r=None, x=None):
        from oracle import linear
        x = self.x if x is None else x
        x = x if rows is None else x[rows]
        r = self.r if r is None else r
        return linear.eora_linear_q(x, self.o_qw, self.o_sc, self.o_qz, self.o_A, self.o_B, self.o_As, self.o_Bs,
                                    x.shape[0], self.d_in, self.d_out, r, self.w_bits, self.group, self.ab_bits)


class SparseCase:
    def __init__(self, seed, d_in, d_out, M, r, packer=None):
        self.d_in, self.d_out, self.M, self.r = d_in, d_out, M, r
        W, A, B, x = synth.draw_layer(seed, d_in, d_out, M, r)
        vals, pos = synth.prune_24(W.astype(np.float16))
        self.logical = dict(vals=vals, pos=pos, A=A, B=B)
        self.x = x
        self.o_values, self.o_indices = layout.pack_sp24(vals, pos)
        self.o_A = self.o_B = None
        if r > 0:
            self.o_A, self.o_B = layout.pack_f16(A), layout.pack_f16(B)
        if packer is not None:
            self.pack_with(packer)

    def pack_with(self, e):
        L = self.logical
        self.values, self.indices = e.pack_sp24(L["vals"], L["pos"])
        assert np.array_equal(self.values.view(np.uint16), self.o_values.view(np.uint16))
        assert np.array_equal(self.indices, self.o_indices)
        self.A = self.B = None
        if self.r > 0:
            self.A, self.B = e.pack_factor_f16(L["A"]), e.pack_factor_f16(L["B"])

    def oracle_y(self, rows=None, x=None):
        from oracle import linear
        x = self.x if x is None else x
        x = x if rows is None else x[rows]
        return linear.eora_linear_sp24(x, self.o_values, self.o_indices, self.o_A, self.o_B,
                                       x.shape[0], self.d_in, self.d_out, self.r)


class SparseQCase:
    """2:4 pruned, then 4-bit quantised backbone (kept values as codes), fp16 factors."""

    def __init__(self, seed, d_in, d_out, M, r, group=128, packer=None):
        self.d_in, self.d_out, self.M, self.r, self.group = d_in, d_out, M, r, group
        W, A, B, x = synth.draw_layer(seed, d_in, d_out, M, r)
        vals, pos = synth.prune_24(W.astype(np.float16))
        codes, zeros, scales = synth.quantize_kept_rtn(vals, pos, group)
        self.logical = dict(codes=codes, pos=pos, zeros=zeros, scales=scales, A=A, B=B)
        self.x = x
        self.o_tiles, self.o_meta = layout.pack_sp24q4(codes, pos, zeros, scales, group)
        self.o_A = self.o_B = None
        if r > 0:
            self.o_A, self.o_B = layout.pack_f16(A), layout.pack_f16(B)
        if packer is not None:
            self.pack_with(packer)

    def pack_with(self, e):
        L = self.logical
        self.tiles, self.meta = e.pack_sp24q4(L["codes"], L["pos"], L["zeros"], L["scales"], self.group)
        assert np.array_equal(self.tiles, self.o_tiles) and np.array_equal(self.meta, self.o_meta)
        self.A = self.B = None
        if self.r > 0:
            self.A, self.B = e.pack_factor_f16(L["A"]), e.pack_factor_f16(L["B"])

    def oracle_y(self, rows=None):
        from oracle import linear
        x = self.x if rows is None else self.x[rows]
        return linear.eora_linear_sp24q4(x, self.o_tiles, self.o_meta, self.o_A, self.o_B,
                                         x.shape[0], self.d_in, self.d_out, self.r)
