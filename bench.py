#!/usr/bin/env python3
"""Benchmark of the EoRA compensated compressed linear layer on one MI355X.

A step is one pass over all seven linears of a LLaMA-3-8B-shaped decoder layer (q, k, v, o, gate,
up, down) at M = 1 with a 3-bit group-128 backbone and fp16 rank-128 EoRA factors: synthetic,
seeded inputs already resident in HBM.  Steps rotate over enough distinct copies of the weights
that neither L2 nor the 256 MB last-level cache can hold them.  The timed region is one HIP graph
holding exactly --steps steps, bracketed by events on the launch stream.

Prints ONE JSON line (see the keys at the end of main()).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0         # dense fp16

WORKLOADS = {
    # name: (shapes, w_bits, ab_bits, r, M, outlier_frac, config id for the seeds)
    "llama3-8b-layer-decode-w3g128-r128fp16-M1": dict(model="8b", w_bits=3, ab_bits=16, r=128, M=1, cfg=2),
    "llama3-8b-layer-decode-w4g128-r128fp16-M1": dict(model="8b", w_bits=4, ab_bits=16, r=128, M=1, cfg=1),
    "llama3-8b-layer-decode-w4g128-r128q4-M1": dict(model="8b", w_bits=4, ab_bits=4, r=128, M=1, cfg=3),
    "llama3-8b-layer-decode-w4g128-bare-M1": dict(model="8b", w_bits=4, ab_bits=16, r=0, M=1, cfg=3),
    "llama3-8b-layer-decode-w3g128-bare-M1": dict(model="8b", w_bits=3, ab_bits=16, r=0, M=1, cfg=2),
    "llama3-8b-layer-decode-w4g128-r128fp16-M16": dict(model="8b", w_bits=4, ab_bits=16, r=128, M=16, cfg=1),
    "llama3-8b-layer-decode-w4g128-r128q4-M8": dict(model="8b", w_bits=4, ab_bits=4, r=128, M=8, cfg=3),
    "llama3-8b-layer-decode-w4g128-bare-M8": dict(model="8b", w_bits=4, ab_bits=4, r=0, M=8, cfg=3),
    "llama3-8b-layer-prefill-w4g128-r256fp16-M2048": dict(model="8b", w_bits=4, ab_bits=16, r=256, M=2048, cfg=4, outlier=0.01),
    "llama3-8b-layer-prefill-w4g128-bare-M2048": dict(model="8b", w_bits=4, ab_bits=16, r=0, M=2048, cfg=4, outlier=0.01),
    "llama3-70b-layer-decode-sp24-r128fp16-M1": dict(model="70b", w_bits=0, ab_bits=16, r=128, M=1, cfg=5),
    "llama3-70b-layer-decode-sp24-bare-M1": dict(model="70b", w_bits=0, ab_bits=16, r=0, M=1, cfg=5),
    "llama3-70b-layer-decode-sp24-r128fp16-M64": dict(model="70b", w_bits=0, ab_bits=16, r=128, M=64, cfg=5),
    # 2:4 pruned, then the kept values quantised to 4 bits (the paper's combined compression)
    "llama3-70b-layer-decode-sp24q4-r128fp16-M1": dict(model="70b", w_bits=0, sq=True, ab_bits=16, r=128, M=1, cfg=5),
    "llama3-70b-layer-decode-sp24q4-bare-M1": dict(model="70b", w_bits=0, sq=True, ab_bits=16, r=0, M=1, cfg=5),
    "llama3-70b-layer-decode-sp24q4-r128fp16-M64": dict(model="70b", w_bits=0, sq=True, ab_bits=16, r=128, M=64, cfg=5),
}
# four rank-128 adapters over one backbone, chosen per request (token row); r is their ranks together
WORKLOADS["llama3-8b-layer-decode-w4g128-4xr128fp16-M64-multi"] = dict(model="8b", w_bits=4, ab_bits=16, r=512, M=64, cfg=1, multi=4)
WORKLOADS["llama3-8b-layer-decode-w4g128-4xr128fp16-M8-multi"] = dict(model="8b", w_bits=4, ab_bits=16, r=512, M=8, cfg=1, multi=4)
WORKLOADS["llama3-8b-layer-decode-w4g128-r512fp16-M64"] = dict(model="8b", w_bits=4, ab_bits=16, r=512, M=64, cfg=1)    # same bytes, one adapter
WORKLOADS["llama3-8b-layer-decode-w4g128-r128fp16-M64"] = dict(model="8b", w_bits=4, ab_bits=16, r=128, M=64, cfg=1)
# 3-bit factors (App. A.9)
WORKLOADS["llama3-8b-layer-decode-w4g128-r128q3-M1"] = dict(model="8b", w_bits=4, ab_bits=3, r=128, M=1, cfg=3)
# 2-bit backbone (App. A.14 evaluates 2-bit models), same layer
WORKLOADS["llama3-8b-layer-decode-w2g128-r128fp16-M1"] = dict(model="8b", w_bits=2, ab_bits=16, r=128, M=1, cfg=2)
WORKLOADS["llama3-8b-layer-decode-w2g128-bare-M1"] = dict(model="8b", w_bits=2, ab_bits=16, r=0, M=1, cfg=2)
WORKLOADS["llama3-8b-layer-decode-w2g128-r128fp16-M16"] = dict(model="8b", w_bits=2, ab_bits=16, r=128, M=16, cfg=2)
WORKLOADS["llama3-8b-layer-prefill-w2g128-r256fp16-M2048"] = dict(model="8b", w_bits=2, ab_bits=16, r=256, M=2048, cfg=4, outlier=0.01)
# the paper's speed table is on a 70B model: the quantised layer at those shapes (not a BASELINE config)
WORKLOADS["llama3-70b-layer-decode-w3g128-r128fp16-M1"] = dict(model="70b", w_bits=3, ab_bits=16, r=128, M=1, cfg=2)
WORKLOADS["llama3-70b-layer-decode-w3g128-bare-M1"] = dict(model="70b", w_bits=3, ab_bits=16, r=0, M=1, cfg=2)
# the same layers with the linears that read the same x sharing a launch (q/k/v and gate/up): four launches a step
for _n in ("llama3-8b-layer-decode-w3g128-r128fp16-M1", "llama3-8b-layer-decode-w3g128-bare-M1",
           "llama3-8b-layer-decode-w4g128-r128fp16-M1", "llama3-8b-layer-decode-w4g128-r128q4-M1",
           "llama3-8b-layer-decode-w4g128-bare-M1", "llama3-8b-layer-prefill-w4g128-r256fp16-M2048",
           "llama3-8b-layer-prefill-w4g128-bare-M2048", "llama3-70b-layer-decode-w3g128-r128fp16-M1",
           "llama3-70b-layer-decode-w3g128-bare-M1", "llama3-8b-layer-decode-w2g128-r128fp16-M1",
           "llama3-8b-layer-decode-w2g128-bare-M1", "llama3-8b-layer-prefill-w2g128-r256fp16-M2048",
           "llama3-8b-layer-decode-w4g128-r128q3-M1", "llama3-8b-layer-decode-w4g128-r128fp16-M16",
           "llama3-8b-layer-decode-w4g128-r128q4-M8", "llama3-8b-layer-decode-w4g128-bare-M8",
           "llama3-8b-layer-decode-w4g128-r128fp16-M64", "llama3-70b-layer-decode-sp24-r128fp16-M1",
           "llama3-70b-layer-decode-sp24-bare-M1", "llama3-70b-layer-decode-sp24-r128fp16-M64",
           "llama3-70b-layer-decode-sp24q4-r128fp16-M1", "llama3-70b-layer-decode-sp24q4-bare-M1",
           "llama3-70b-layer-decode-sp24q4-r128fp16-M64"):
    WORKLOADS[_n + "-grouped"] = dict(WORKLOADS[_n], grouped=True)
GROUPS = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))
for _r in (64, 256, 512):
    WORKLOADS["llama3-8b-layer-decode-w4g128-r%dq4-M1" % _r] = dict(model="8b", w_bits=4, ab_bits=4, r=_r, M=1, cfg=3)
DEFAULT = "llama3-8b-layer-decode-w3g128-r128fp16-M1-grouped"
# Algorithm 1 steps 1-6 (the factors themselves) for one 4096 x 4096 linear of the 8B model, W4 g128 backbone,
# 8192 calibration tokens; a different metric (seconds per linear), run by calibration_main()
CALIBRATION = {
    "llama3-8b-q-factors-w4g128-r128-n8192": dict(d_in=4096, d_out=4096, n_tokens=8192, r=128, w_bits=4, sample=1536),
    "llama3-8b-k-factors-w4g128-r128-n8192": dict(d_in=4096, d_out=1024, n_tokens=8192, r=128, w_bits=4, sample=1536),
    "llama3-8b-gate-factors-w4g128-r128-n8192": dict(d_in=4096, d_out=14336, n_tokens=8192, r=128, w_bits=4, sample=1536),
    "llama3-8b-down-factors-w4g128-r128-n16384": dict(d_in=14336, d_out=4096, n_tokens=16384, r=128, w_bits=4, sample=1536),
    "small-factors-w4g128-r64-n2048": dict(d_in=1024, d_out=1024, n_tokens=2048, r=64, w_bits=4, sample=1024),
}


def dev(a):
    """numpy array -> device tensor (uint32 words travel as int32)."""
    import numpy as np
    import torch
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def algorithmic_bytes(d_in, d_out, M, r, w_bits, ab_bits, group=128, sq=False):
    """Bytes the method must move for one linear: packed codes, scales, zero-points, factors,
    x read once and y written once (the M x r intermediate never makes a y-sized round trip)."""
    if w_bits == 0 and sq:                                   # 2:4 sparse, 4-bit kept values: 8 + 4 bits per four positions
        b = d_out * d_in * 0.375 + d_out * (d_in // 128) * 4        # tile words, one scale/zero word per (row, tile)
    elif w_bits == 0:                                        # 2:4 sparse fp16: two values + 4 index bits per four positions
        b = d_out * d_in * 1.125
    else:
        b = d_out * d_in * w_bits / 8 + d_out * (d_in // group) * 2.5
    if r:
        if ab_bits == 16:
            b += 2 * r * (d_in + d_out)
        elif ab_bits == 3:
            b += r * d_in * 3 / 8 + 2 * r * (d_in // 128) + d_out * r * 3 / 8 + 2 * d_out * (r // 128)
        else:
            KTb = min(128, r)
            b += r * d_in / 2 + 2 * r * (d_in // 128) + d_out * r / 2 + 2 * d_out * (r // KTb)
    return b + 2 * M * (d_in + d_out)


class Linear:
    """Device-resident copies of one linear's stored operands."""

    def __init__(self, name, d_in, d_out, spec, seed, ncopies):
        import numpy as np
        import torch
        import synth
        import paper_2410_21271_amd as eora
        self.name, self.d_in, self.d_out = name, d_in, d_out
        self.M, self.r, self.w_bits, self.ab_bits = spec["M"], spec["r"], spec["w_bits"], spec["ab_bits"]
        self.sq = bool(spec.get("sq", False))
        self.multi = int(spec.get("multi", 0))
        if self.multi:                                    # adapter of each request: none, or one of the adapters, seeded
            self.sel = np.random.default_rng(seed + 7).integers(-1, self.multi, self.M).astype(np.int32)
            self.sel_dev = torch.from_numpy(self.sel).cuda()
        W, A, B, x = synth.draw_layer(seed, d_in, d_out, self.M, self.r, spec.get("outlier", 0.0))
        if self.w_bits == 0 and self.sq:
            vals, pos = synth.prune_24(W.astype(np.float16))
            del W
            codes, zeros, scales = synth.quantize_kept_rtn(vals, pos, 128)
            self.logical = (codes, pos, (zeros, scales), A, B, x)
            tiles, meta = eora.pack_sp24q4(codes, pos, zeros, scales, 128)
            host = [tiles, meta, None, None, None, None, None]
        elif self.w_bits == 0:
            vals, pos = synth.prune_24(W.astype(np.float16))
            del W
            self.logical = (vals, pos, None, A, B, x)
            values, indices = eora.pack_sp24(vals, pos)
            host = [values, indices, None, None, None, None, None]
        else:
            codes, zeros, scales = synth.quantize_rtn(W, self.w_bits, 128)
            del W
            self.logical = (codes, zeros, scales, A, B, x)
            qw, qz, sc = eora.pack_q(codes, zeros, scales, self.w_bits, 128)
            host = [qw, sc, qz, None, None, None, None]
        if self.r and self.ab_bits == 16:
            host[3], host[4] = eora.pack_factor_f16(A), eora.pack_factor_f16(B)
        elif self.r and self.ab_bits == 3:
            ca, sa = synth.quantize_sym3(A)
            cb, sb = synth.quantize_sym3(B)
            host[3], host[5] = eora.pack_factor_q3(ca, sa)
            host[4], host[6] = eora.pack_factor_q3(cb, sb)
            self.logical = (codes, zeros, scales, (ca, sa), (cb, sb), x)
        elif self.r:
            ca, sa = synth.quantize_sym4(A, 128)
            cb, sb = synth.quantize_sym4(B, min(128, self.r))
            host[3], host[5] = eora.pack_factor_q4(ca, sa)
            host[4], host[6] = eora.pack_factor_q4(cb, sb)
            self.logical = (codes, zeros, scales, (ca, sa), (cb, sb), x)
        first = [dev(h) for h in host]
        self.copies = [first] + [[None if t is None else t.clone() for t in first] for _ in range(ncopies - 1)]
        self.x = dev(x)
        self.y = torch.zeros((self.M, d_out), dtype=torch.float16, device="cuda")
        self.ws = eora.new_workspace(self.M, d_in, d_out, self.r)
        self.bytes = algorithmic_bytes(d_in, d_out, self.M, self.r, self.w_bits, self.ab_bits, sq=self.sq)
        self.flops = 2.0 * self.M * d_in * d_out + 2.0 * self.M * self.r * (d_in + d_out)

    def run(self, copy):
        import paper_2410_21271_amd as eora
        qw, sc, qz, A, B, As, Bs = self.copies[copy % len(self.copies)]
        if self.sq:
            eora.linear_sp24q4(self.x, qw, sc, A, B, self.y, self.M, self.d_in, self.d_out, self.r, self.ws)
            return
        if self.w_bits == 0:
            eora.linear_sp24(self.x, qw, sc, A, B, self.y, self.M, self.d_in, self.d_out, self.r, self.ws)
            return
        if self.multi:
            eora.linear_q_multi(self.x, qw, sc, qz, A, B, As, Bs, self.sel_dev, self.y, self.M, self.d_in, self.d_out,
                                self.r // self.multi, self.multi, self.w_bits, 128, self.ab_bits, self.ws)
            return
        eora.linear_q(self.x, qw, sc, qz, A, B, As, Bs, self.y, self.M, self.d_in, self.d_out, self.r,
                      self.w_bits, 128, self.ab_bits, self.ws)


class Group:
    """Linears that read the same x, served by one eora_linear_q_group call (x is the first member's)."""

    def __init__(self, members):
        import paper_2410_21271_amd as eora
        self.members = members
        self.name = "+".join(L.name for L in members)
        self.d_in = members[0].d_in
        m0 = members[0]
        for L in members[1:]:                             # everyone reads the first member's activations
            L.x = m0.x
            L.logical = L.logical[:5] + (m0.logical[5],)
        self.ws = eora.new_workspace(m0.M, m0.d_in, max(L.d_out for L in members), m0.r, n_members=len(members))
        # x is read once per launch, not once per member
        self.bytes = sum(L.bytes for L in members) - 2 * m0.M * m0.d_in * (len(members) - 1)
        self.flops = sum(L.flops for L in members)

    def run(self, copy):
        import paper_2410_21271_amd as eora
        m0 = self.members[0]
        if len(self.members) == 1:
            return m0.run(copy)
        if m0.w_bits == 0:                                # 2:4 members: (values, indices) or (qtiles, qmeta)
            mem = []
            for L in self.members:
                c = L.copies[copy % len(L.copies)]
                mem.append((None, None, c[0], c[1], c[3], c[4], L.y, L.d_out) if L.sq else (c[0], c[1], None, None, c[3], c[4], L.y, L.d_out))
            eora.linear_sp24_group(m0.x, mem, m0.M, m0.d_in, m0.r, self.ws)
            return
        mem = [tuple(L.copies[copy % len(L.copies)]) + (L.y, L.d_out) for L in self.members]
        eora.linear_q_group(m0.x, mem, m0.M, m0.d_in, m0.r, m0.w_bits, 128, m0.ab_bits, self.ws)


BATCHES = 11


def timed_graph(fn, count, batches=BATCHES):
    """Capture `count` calls fn(i) into one HIP graph, replay it once untimed and then `batches` times, each
    replay between two events on the launch stream; returns (median, min, max) milliseconds per call."""
    import torch
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(count):
            fn(i)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(batches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) / count)
    times.sort()
    return times[len(times) // 2], times[0], times[-1]


def parity_sample(linears, nblocks=6):
    """Every linear of the step against the oracle on sampled 16-row blocks (first, last, seeded ones), all token
    rows: the stored bytes of the sample are packed by the oracle's own packer from the logical arrays."""
    import numpy as np
    from oracle import layout, linear
    worst = 0.0
    for L in linears:
        nb = L.d_out // 16
        rng = np.random.default_rng(L.d_out + L.d_in)
        blocks = sorted({0, nb - 1, *rng.integers(0, nb, nblocks).tolist()})
        rows = np.concatenate([np.arange(16 * b, 16 * b + 16) for b in blocks])
        codes, zeros, scales, A, B, x = L.logical
        got = L.y.cpu().numpy()[:, rows]
        n = len(rows)
        if L.w_bits == 0:
            Ap, Bp = (layout.pack_f16(A), layout.pack_f16(B[rows])) if L.r else (None, None)
            if L.sq:
                tiles, meta = layout.pack_sp24q4(codes[rows], zeros[rows], scales[0][rows], scales[1][rows], 128)
                ref = linear.eora_linear_sp24q4(x, tiles, meta, Ap, Bp, L.M, L.d_in, n, L.r)
            else:
                values, indices = layout.pack_sp24(codes[rows], zeros[rows])
                ref = linear.eora_linear_sp24(x, values, indices, Ap, Bp, L.M, L.d_in, n, L.r)
        else:
            qw = {4: layout.pack_q4, 3: layout.pack_q3, 2: layout.pack_q2}[L.w_bits](codes[rows])
            qz, sc = layout.pack_zeros(zeros[rows]), layout.pack_scales(scales[rows])
            Ap = Bp = As = Bs = None
            if L.r and L.ab_bits == 16:
                Ap, Bp = layout.pack_f16(A), layout.pack_f16(B[rows])
            elif L.r and L.ab_bits == 3:
                Ap, As = layout.pack_q3(A[0]), layout.pack_scales(A[1])
                Bp, Bs = layout.pack_q3(B[0][rows]), layout.pack_scales(B[1][rows])
            elif L.r:
                Ap, As = layout.pack_q4(A[0], 128), layout.pack_scales(A[1])
                Bp, Bs = layout.pack_q4(B[0][rows], min(128, L.r)), layout.pack_scales(B[1][rows])
            if L.multi:
                ref = linear.eora_linear_q_multi(x, qw, sc, qz, Ap, Bp, As, Bs, L.sel, L.M, L.d_in, n, L.r // L.multi, L.multi,
                                                 L.w_bits, 128, L.ab_bits)
            else:
                ref = linear.eora_linear_q(x, qw, sc, qz, Ap, Bp, As, Bs, L.M, L.d_in, n, L.r, L.w_bits, 128, L.ab_bits)
        worst = max(worst, linear.y_error(got, ref))
    return worst


def clocks():
    """Clocks and power cap as rocm-smi reports them after the timed runs (best effort; None if unavailable)."""
    import subprocess
    try:
        p = subprocess.run(["rocm-smi", "--showclocks", "--showmaxpower", "--json"], capture_output=True, text=True, timeout=20)
        card = next(iter(json.loads(p.stdout).values()))
        keep = {}
        for k, v in card.items():
            kl = k.lower()
            if "sclk" in kl or "mclk" in kl or "fclk" in kl or "power" in kl:
                keep[k] = v
        return keep or None
    except Exception:
        return None


def device_context(nbytes):
    """Measured in this run, same protocol as the layer (graphs of 200 launches, median of BATCHES replays): the
    launch floor (an empty kernel) and the rate of a kernel that only reads nbytes (rotating over > 1 GB)."""
    import torch
    import paper_2410_21271_amd as eora
    sink = torch.zeros(256, dtype=torch.uint8, device="cuda")
    floor_us = 1e3 * timed_graph(lambda i: eora.debug_probe(0, None, 0, sink), 200)[0]
    nbytes = max(32768, int(nbytes) // 32768 * 32768)
    ncop = max(2, int(1.1e9 // nbytes) + 1)
    buf = torch.ones(ncop * nbytes, dtype=torch.uint8, device="cuda")
    us = 1e3 * timed_graph(lambda i: eora.debug_probe(1, buf[(i % ncop) * nbytes:], nbytes, sink), 200)[0]
    return round(floor_us, 3), round(nbytes / us / 1e3, 1), nbytes


def cpu_baseline(linears, names):
    """The float64 oracle as it stands, timed on the host cores on a bounded sample."""
    import numpy as np
    from oracle import layout, linear
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    total_t, total_b, worst = 0.0, 0.0, 0.0
    for L in linears:
        if L.name not in names:
            continue
        codes, zeros, scales, A, B, x = L.logical
        if L.w_bits == 0 and L.sq:
            tiles, meta = layout.pack_sp24q4(codes, zeros, scales[0], scales[1], 128)
            Ap, Bp = (layout.pack_f16(A), layout.pack_f16(B)) if L.r else (None, None)
            t0 = time.perf_counter()
            y = linear.eora_linear_sp24q4(x, tiles, meta, Ap, Bp, L.M, L.d_in, L.d_out, L.r)
            total_t += time.perf_counter() - t0
            total_b += L.bytes
            worst = max(worst, linear.y_error(L.y.cpu().numpy(), y))
            continue
        if L.w_bits == 0:
            values, indices = layout.pack_sp24(codes, zeros)
            Ap, Bp = (layout.pack_f16(A), layout.pack_f16(B)) if L.r else (None, None)
            t0 = time.perf_counter()
            y = linear.eora_linear_sp24(x, values, indices, Ap, Bp, L.M, L.d_in, L.d_out, L.r)
            total_t += time.perf_counter() - t0
            total_b += L.bytes
            worst = max(worst, linear.y_error(L.y.cpu().numpy(), y))
            continue
        qw = {4: layout.pack_q4, 3: layout.pack_q3, 2: layout.pack_q2}[L.w_bits](codes)
        qz, sc = layout.pack_zeros(zeros), layout.pack_scales(scales)
        Ap = Bp = As = Bs = None
        if L.r and L.ab_bits == 16:
            Ap, Bp = layout.pack_f16(A), layout.pack_f16(B)
        elif L.r and L.ab_bits == 3:
            Ap, As = layout.pack_q3(A[0]), layout.pack_scales(A[1])
            Bp, Bs = layout.pack_q3(B[0]), layout.pack_scales(B[1])
        elif L.r:
            Ap, As = layout.pack_q4(A[0], 128), layout.pack_scales(A[1])
            Bp, Bs = layout.pack_q4(B[0], min(128, L.r)), layout.pack_scales(B[1])
        t0 = time.perf_counter()
        if L.multi:
            y = linear.eora_linear_q_multi(x, qw, sc, qz, Ap, Bp, As, Bs, L.sel, L.M, L.d_in, L.d_out, L.r // L.multi, L.multi,
                                           L.w_bits, 128, L.ab_bits)
        else:
            y = linear.eora_linear_q(x, qw, sc, qz, Ap, Bp, As, Bs, L.M, L.d_in, L.d_out, L.r, L.w_bits, 128, L.ab_bits)
        total_t += time.perf_counter() - t0
        total_b += L.bytes
        worst = max(worst, linear.y_error(L.y.cpu().numpy(), y))
    return dict(value=total_b / total_t / 1e9, unit="GB/s", cores=int(threads), kind="oracle",
                sample="one pass of the numpy float64 oracle over the %s linears of the same layer "
                       "(%.1f s)" % ("/".join(names), total_t)), worst


def calibration_inputs(eora, synth, np, torch, seed, d_in, d_out, n_tokens, w_bits):
    """W (fp32), its compressed version from the library's own dequantisation, and X-tilde, all on the device."""
    W, _, _, _ = synth.draw_layer(seed, d_in, d_out, 1, 0)
    codes, zeros, scales = synth.quantize_rtn(W, w_bits, 128)
    qw, qz, sc = eora.pack_q(codes, zeros, scales, w_bits, 128)
    W_hat = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    eora.dequant_q(dev(qw), dev(sc), dev(qz), W_hat, d_in, d_out, w_bits, 128)
    Xt = synth.draw_calibration(seed + 1, d_in, n_tokens)
    return torch.from_numpy(W).cuda(), W_hat, torch.from_numpy(Xt).cuda()


def calibration_main(args):
    """One step = Algorithm 1 steps 1-6 for one linear (eora_factors).  The call synchronises, so steps are
    timed with the host clock between device synchronisations; the dominant kernel (a Jacobi round of the SVD of
    step 5, or of the eigendecomposition when the Gram matrix needs it) is timed by the library with events on the
    launch stream."""
    import numpy as np
    import torch
    import synth
    import paper_2410_21271_amd as eora
    spec = CALIBRATION[args.workload]
    d_in, d_out, n, r = spec["d_in"], spec["d_out"], spec["n_tokens"], spec["r"]
    steps, warmup = min(args.steps, 3), min(args.warmup, 1)

    def run(W, W_hat, Xt, d_in, d_out, n, r):
        B = torch.zeros((d_out, r), dtype=torch.float64, device="cuda")
        A = torch.zeros((r, d_in), dtype=torch.float64, device="cuda")
        ws = torch.empty(eora.factors_workspace_bytes(d_in, d_out, r), dtype=torch.uint8, device="cuda")
        st = eora.factors(W, W_hat, Xt, B, A, None, n, d_in, d_out, r, 1e-12, ws, stats=True)
        return B, A, st

    W, W_hat, Xt = calibration_inputs(eora, synth, np, torch, 4242, d_in, d_out, n, spec["w_bits"])
    for _ in range(warmup):
        run(W, W_hat, Xt, d_in, d_out, n, r)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        _, _, st = run(W, W_hat, Xt, d_in, d_out, n, r)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    # Dominant kernel: the Jacobi rounds of the SVD of step 5 (and of the eigendecomposition, when the Gram matrix
    # took that route: its rounds then dominate).  Algorithmic bytes of a round: every row of the rotated matrix
    # read once (the dot products / the Gram blocks); a workgroup that rotates its rows (2 of them, or 16 in a block
    # round, which reads them a second time for the MFMA product) also writes them, and with an eigenvector matrix
    # reads and writes as many rows of it.
    def jacobi_round(prefix, m, L, with_v):
        rows = st[prefix + "_rows"]
        rounds = st[prefix + "_sweeps"] * ((m - 1) if rows == 2 else (m // 8 - 1))
        per_rotation = 8.0 * rows * ((1 if rows == 2 else 2) * L + (2 * L if with_v else 0))
        return rows, rounds, rounds * 8.0 * m * L + st[prefix + "_rotations"] * per_rotation, st[prefix + "_ms"]
    if st["eig_rows"] > 0:
        what = "eigendecomposition"
        rows, rounds, bytes_total, ms = jacobi_round("eig", d_in, d_in, True)
        m_rows, length = d_in, d_in
    else:
        what = "SVD of step 5"
        m_rows, length = min(d_out, d_in), int(st["eig_rotations"])      # (Cholesky route: that counter holds the rotated rows' length)
        rows, rounds, bytes_total, ms = jacobi_round("svd", m_rows, length, False)
    us_round = 1e3 * ms / rounds
    kernel = "Jacobi round of the %s (%d rows of length %d per workgroup)" % (what, rows, length)
    traffic = None                                    # HBM bytes per round from the committed counter runs, if they are of this kernel
    tpath = os.path.join(ROOT, "profiles", "factors_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            rec = json.load(f).get(args.workload)
        if isinstance(rec, dict) and rec.get("kernel") == kernel:
            traffic = rec.get("bytes")
    roofline = dict(bound="hbm", achieved=round(bytes_total / rounds / us_round / 1e3, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(bytes_total / rounds / us_round / 1e3 / HBM_PEAK_GBS, 4), traffic=traffic, kernel=kernel,
                    bytes_per_launch=int(bytes_total / rounds), us_per_launch=round(us_round, 3), launches=rounds)
    out = dict(metric="seconds for Algorithm 1 steps 1-6 of one %d x %d linear (rank %d, %d calibration tokens)" % (d_out, d_in, r, n),
               value=round(sec, 4), unit="s", n_gpus=1, steps=steps, warmup=warmup, ms_per_step=round(1e3 * sec, 3),
               higher_is_better=False, scaling="weak", vs_baseline=None, dtype="f64", data="synthetic",
               config=dict(workload=args.workload, gram_route="cholesky" if st["eig_rows"] == 0 else "eigendecomposition",
                           eig_sweeps=st["eig_sweeps"], eig_seconds=round(st["eig_ms"] / 1e3, 4),
                           svd_sweeps=st["svd_sweeps"], svd_seconds=round(st["svd_ms"] / 1e3, 4)),
               roofline=roofline)
    if not args.no_cpu_baseline:
        from oracle import calibrate
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
        sd = spec["sample"]                                   # the oracle on a smaller linear of the same recipe
        so = min(sd, d_out)
        Ws, Whs, Xs = calibration_inputs(eora, synth, np, torch, 4343, sd, so, 2 * sd, spec["w_bits"])
        Bg, Ag, _ = run(Ws, Whs, Xs, sd, so, 2 * sd, min(r, so))
        t0 = time.perf_counter()
        Bo, Ao = calibrate.eora_factors(Ws.cpu().numpy(), Whs.cpu().numpy(), Xs.cpu().numpy(), min(r, so))
        cpu_s = time.perf_counter() - t0
        Po = Bo @ Ao
        out["config"]["max_err_vs_oracle"] = float("%.3g" % (np.abs((Bg @ Ag).cpu().numpy() - Po).max() / np.abs(Po).max()))
        scale = (d_in / sd) ** 3 * (0.5 + 0.5 * d_out / d_in) / (0.5 + 0.5 * so / sd)
        out["cpu_baseline"] = dict(value=round(cpu_s * scale, 2), unit="s", cores=int(threads), kind="oracle",
                                   sample="numpy float64 oracle on a %d x %d linear with %d tokens took %.2f s; scaled by the "
                                          "cubic cost of the eigendecomposition and SVD to the full shape" % (so, sd, 2 * sd, cpu_s))
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT, choices=sorted(WORKLOADS) + sorted(CALIBRATION))
    ap.add_argument("--copies", type=int, default=0, help="distinct weight copies (0 = enough for 1.2 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--linears", default="", help="comma-separated subset of the layer's linears (q,k,v,o,gate,up,down) to run")
    ap.add_argument("--profile-only", action="store_true",
                    help="run --warmup + --steps steps eagerly (no graphs, no baselines) and exit: the program a "
                         "rocprofv3 counter run profiles")
    ap.add_argument("--spin-limit", type=int, default=None,
                    help="diagnosis: eora_debug_set_spin_limit before the runs (negative: every wait for t counts as "
                         "expired, so the low-rank term is skipped and results are NOT the layer's)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run plain device-to-device copies of 256 MiB (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the layer; --gpus %d is not supported "
              "(no collective or sharding code exists here)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    if args.copy_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel(), "copy_probe_bytes_written": src.numel(), "copies": 10}))
        return
    if args.spin_limit is not None:
        import paper_2410_21271_amd as eora
        eora.debug_set_spin_limit(args.spin_limit)
    if args.workload in CALIBRATION:
        return calibration_main(args)
    spec = WORKLOADS[args.workload]
    shapes = synth.LLAMA3_8B if spec["model"] == "8b" else synth.LLAMA3_70B
    layer_bytes = sum(algorithmic_bytes(di, do, spec["M"], spec["r"], spec["w_bits"], spec["ab_bits"], sq=bool(spec.get("sq")))
                      for _, di, do in shapes)
    # enough copies that the whole layer rotates over 1.2 GB and, up to 8 GB in all, even its smallest launch
    # over more than twice the 256 MB last-level cache
    smallest = min(algorithmic_bytes(di, do, spec["M"], spec["r"], spec["w_bits"], spec["ab_bits"], sq=bool(spec.get("sq")))
                   for n_, di, do in shapes if n_ in ("o", "down"))
    ncopies = args.copies or max(2, int(1.2e9 / layer_bytes) + 1, min(int(600e6 / smallest) + 1, int(8e9 / layer_bytes)))
    if spec["M"] > 16:
        args.steps = min(args.steps, 50)
    only = [n for n in args.linears.split(",") if n]
    if only:
        ncopies = 2 if args.profile_only else ncopies
    linears = [Linear(n, di, do, spec, synth.seed_for(spec["cfg"], i), ncopies) for i, (n, di, do) in enumerate(shapes)
               if not only or n in only]

    launches = linears
    if spec.get("grouped"):
        launches = [Group([L for L in linears if L.name in g]) for g in GROUPS if any(L.name in g for L in linears)]
        layer_bytes = sum(G.bytes for G in launches)
    elif only:
        layer_bytes = sum(L.bytes for L in linears)

    def step(i):
        for L in launches:
            L.run(i)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.profile_only:
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        print(json.dumps(dict(profile_only=True, workload=args.workload, linears=[L.name for L in linears],
                              steps=args.steps, warmup=args.warmup, launches_per_step=len(launches))))
        return
    ms_per_step, ms_min, ms_max = timed_graph(step, args.steps)

    # each linear on its own (graph of back-to-back launches over the rotating copies)
    per_linear = {}
    for L in launches:
        us = 1e3 * timed_graph(L.run, 200 if spec["M"] <= 16 else 40)[0]
        per_linear[L.name] = dict(us=round(us, 3), GBps=round(L.bytes / us / 1e3, 1),
                                  frac_hbm=round(L.bytes / us / 1e3 / HBM_PEAK_GBS, 4),
                                  TFLOPs=round(L.flops / us / 1e6, 1),
                                  # alone, a launch rotates over its own copies only: below the 256 MB last-level
                                  # cache (twice, to be safe) its figure may be cache-assisted; the layer's is not
                                  rotation_MB=round(ncopies * L.bytes / 1e6, 1), cache_assisted=bool(ncopies * L.bytes < 512e6))
    # Dominant kernel: launches are grouped by the kernel instantiation that serves them, as the library reports it
    # (eora_debug_last_launch without the run-time arguments); the instantiation whose launches move the most
    # algorithmic bytes per step is reported.  Its average launch moves the average algorithmic bytes of its
    # launches; its average duration is the mean of their event-timed back-to-back launches (which includes the
    # gap between launches).
    import re
    import paper_2410_21271_amd as eora
    for L in launches:
        L.run(0)
        torch.cuda.synchronize()
        L.kernel = re.sub(r" (n|wgs|q|ksplit|c2)=-?\d+", "", eora.debug_last_launch())
        per_linear[L.name]["kernel"] = L.kernel
    groups = {}
    for L in launches:
        groups.setdefault(L.kernel, []).append(L)
    dom = max(groups.values(), key=lambda g: (sum(L.bytes for L in g), sum(per_linear[L.name]["us"] for L in g)))
    dom_bytes = sum(L.bytes for L in dom) / len(dom)
    dom_us = sum(per_linear[L.name]["us"] for L in dom) / len(dom)
    # HBM bytes per launch of that kernel from the committed rocprofv3 counter runs of this workload (not collected
    # in this run: counters and timing need runs of their own); null when no such run is recorded for this kernel
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "decode_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            rec = json.load(f).get(args.workload)
        if isinstance(rec, dict) and rec.get("kernel") == dom[0].kernel:
            traffic, traffic_source = rec.get("bytes"), "profiles/decode_traffic.json"
    prefill = spec["M"] >= 128
    if prefill:
        # dominant kernel: the GEMM kernel; a launch contracts one linear (or one group of them)
        dom_flops = sum(L.flops for L in dom) / len(dom)
        roofline = dict(bound="mfma", achieved=round(dom_flops / dom_us / 1e6, 1), peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=round(dom_flops / dom_us / 1e6 / MFMA_PEAK_TFLOPS, 4), traffic=None,
                        kernel="%s (%s)" % (dom[0].kernel, ",".join(L.name for L in dom)),
                        flops_per_launch=int(dom_flops), us_per_launch=round(dom_us, 3))
    else:
        roofline = dict(bound="hbm", achieved=round(dom_bytes / dom_us / 1e3, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(dom_bytes / dom_us / 1e3 / HBM_PEAK_GBS, 4), traffic=traffic,
                        kernel="%s (%s)" % (dom[0].kernel, ",".join(L.name for L in dom)),
                        bytes_per_launch=int(dom_bytes), us_per_launch=round(dom_us, 3), traffic_source=traffic_source)
    floor_us, ceiling, probe_bytes = device_context(dom_bytes)
    roofline.update(launch_floor_us=floor_us, stream_ceiling_GBps=ceiling, stream_probe_bytes=probe_bytes)
    layer_flops = sum(L.flops for L in linears)
    if prefill:
        out = dict(metric="prefill TFLOP/s over one 8B decoder layer's linears (M=%d)" % spec["M"],
                   value=round(layer_flops / ms_per_step / 1e9, 1), unit="TFLOP/s")
    else:
        out = dict(metric="decode HBM GB/s over one %s decoder layer's linears (M=%d)" % (spec["model"].upper(), spec["M"]),
                   value=round(layer_bytes / ms_per_step / 1e6, 1), unit="GB/s")
    out.update(n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(ms_per_step, 6), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16", data="synthetic",
               config=dict(workload=args.workload, layer_bytes=int(layer_bytes), layer_flops=int(layer_flops), weight_copies=ncopies,
                           launches_per_step=len(launches), batches=BATCHES,
                           layer_us=round(1e3 * ms_per_step, 3), layer_us_min=round(1e3 * ms_min, 3), layer_us_max=round(1e3 * ms_max, 3), frac_hbm_peak=round(layer_bytes / ms_per_step / 1e6 / HBM_PEAK_GBS, 4),
                           per_linear=per_linear),
               roofline=roofline)
    out["config"]["clocks"] = clocks()
    if not args.no_cpu_baseline:
        # the 8B layer in full (about 10 s of CPU work for the default workload); of the 70B layer the two narrow linears
        base, worst = cpu_baseline(linears, ("q", "k", "v", "o", "gate", "up", "down") if spec["model"] == "8b" else ("k", "v"))
        out["cpu_baseline"] = base
        # every linear of the step on sampled row blocks, and the linears the baseline ran in full
        out["config"]["max_err_vs_oracle"] = float("%.3g" % max(worst, parity_sample(linears)))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
