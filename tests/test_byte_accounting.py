"""The stored size of the EoRA factors in this project's layouts against the model-size
deltas the paper prints for LLaMA3-8B (32 decoder layers, 7 linears each)."""
import os

import numpy as np

import synth
from oracle import layout
from tests.golden_io import GOLDEN


def _factor_bytes(r, bits):
    total = 0
    for _, d_in, d_out in synth.LLAMA3_8B:
        if bits == 16:
            total += 2 * r * (d_in + d_out)
        elif bits == 3:                                              # 3.0 bits per element, one fp16 scale per group of 128
            total += r * d_in * 3 // 8 + 2 * r * (d_in // 128)
            total += d_out * r * 3 // 8 + 2 * d_out * (r // 128)
        else:
            KTb = min(128, r)
            total += r * d_in // 2 + 2 * r * (d_in // 128)          # A codes + scales
            total += d_out * r // 2 + 2 * d_out * (r // KTb)        # B codes + scales
    return 32 * total


def test_factor_bytes_match_paper_size_deltas():
    rows = {}
    with open(os.path.join(GOLDEN, "model_size.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].split()
            if line:
                rows[(line[0], int(line[1]), int(line[2]))] = float(line[3])
    for (bb, r, bits), size in rows.items():
        if r == 0:
            continue
        delta = size - rows[(bb, 0, 0)]
        ours = _factor_bytes(r, bits) / 2 ** 30       # the table's unit fits GiB: rank 512 fp16 is 2.50 exactly
        if bits == 3:
            # the paper does not give its 3-bit storage; its deltas (0.11-0.12 at rank 128, 0.52-0.55 at rank 512)
            # come to about 3.5 bits per element, this project's tiles hold 3.0 bits plus one fp16 scale per 128
            assert abs(ours - delta) <= 0.015 + 0.12 * delta and ours <= delta + 0.015, (bb, r, bits, ours, delta)
            continue
        assert abs(ours - delta) <= 0.03 + 0.03 * delta, (bb, r, bits, ours, delta)


def test_packed_arrays_have_no_padding():
    # the packers produce exactly the byte counts the accounting above assumes
    r, d_in, d_out = 64, 256, 32
    A = np.zeros((r, d_in), np.float16)
    assert layout.pack_f16(A).nbytes == 2 * r * d_in
    assert layout.pack_q4(np.zeros((r, d_in), np.uint8), 128).nbytes == r * d_in // 2
    assert layout.pack_q4(np.zeros((d_out, r), np.uint8), 64).nbytes == d_out * r // 2
    assert layout.pack_q3(np.zeros((d_out, d_in), np.uint8)).nbytes == d_out * d_in * 3 // 8
    assert layout.pack_zeros(np.zeros((d_out, 8), np.uint8)).nbytes == d_out * 8 // 2
    v, i = layout.pack_sp24(np.zeros((d_out, d_in // 2), np.float16), np.tile(np.array([0, 1], np.uint8), (d_out, d_in // 4)))
    assert v.nbytes + i.nbytes == d_out * d_in * 9 // 8
    pos = np.tile(np.array([0, 1], np.uint8), (d_out, d_in // 4))
    t, m = layout.pack_sp24q4(np.zeros((d_out, d_in // 2), np.uint8), pos, np.zeros((d_out, 2), np.uint8),
                              np.ones((d_out, 2), np.float16), 128)
    assert t.nbytes == d_out * d_in * 3 // 8 and m.nbytes == d_out * (d_in // 128) * 4      # 0.375 + 0.031 B per dense weight
