"""Sanity of the seeded input generators (no layer arithmetic lives there)."""
import numpy as np

import synth


def test_quantizer_ranges_and_error_bound():
    W, _, _, _ = synth.draw_layer(1, 256, 32, 1, 0)
    for bits in (3, 4):
        q, z, s = synth.quantize_rtn(W, bits, 128)
        assert q.dtype == np.uint8 and q.max() <= (1 << bits) - 1
        assert z.max() <= (1 << bits) - 1 and s.dtype == np.float16 and np.all(s > 0)
        deq = np.repeat(s.astype(np.float64), 128, 1) * (q.astype(np.float64) - np.repeat(z.astype(np.float64), 128, 1))
        assert np.max(np.abs(deq - W)) <= 1.01 * np.max(s.astype(np.float64))   # within about one step (zero-point rounding adds to the half step)
        assert q.min() == 0 and q.max() == (1 << bits) - 1


def test_prune_24_structure():
    W = np.random.default_rng(0).standard_normal((16, 128)).astype(np.float16)
    vals, pos = synth.prune_24(W)
    assert vals.shape == (16, 64) and pos.max() <= 3
    assert np.all(pos[:, 0::2] < pos[:, 1::2])
    g = np.abs(W.astype(np.float32)).reshape(16, 32, 4)
    kept = np.sort(np.abs(vals.astype(np.float32)).reshape(16, 32, 2), axis=2)
    assert np.array_equal(kept, np.sort(g, axis=2)[:, :, 2:])
    tie = np.array([[1, 1, 1, 1] * 32], np.float16).repeat(16, 0)
    _, p = synth.prune_24(tie)
    assert np.all(p[:, 0::2] == 0) and np.all(p[:, 1::2] == 1)


def test_draws_are_seeded_and_shaped():
    a = synth.draw_layer(synth.seed_for(1), 256, 32, 4, 32)
    b = synth.draw_layer(synth.seed_for(1), 256, 32, 4, 32)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    W, A, B, x = a
    assert W.shape == (32, 256) and A.shape == (32, 256) and B.shape == (32, 32) and x.shape == (4, 256)
    assert A.dtype == np.float16 and x.dtype == np.float16
    _, _, _, xo = synth.draw_layer(3, 4096, 16, 8, 0, outlier_frac=0.01)
    big = np.sum(np.abs(xo.astype(np.float32)).mean(axis=0) > 8)
    assert 30 <= big <= 41                     # 41 channels scaled by 20
    assert synth.LLAMA3_8B[4] == ("gate", 4096, 14336) and synth.LLAMA3_70B[6] == ("down", 28672, 8192)
