"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

Nothing here performs the layer's arithmetic or knows a byte layout: the
functions only draw random matrices and turn them into the LOGICAL stored form
(integer codes, zero-points, fp16 scales, kept values and positions).  They stand
in for the paper's LLaMA checkpoints compressed with GPTQ / SparseGPT and for its
calibration and evaluation data (Sec. 4.1), none of which are available offline:
shapes are those of LLaMA-3-8B / 70B linear layers, weights are Gaussian with
standard deviation 0.02, EoRA factors Gaussian with standard deviation 0.01,
activations standard normal (optionally with 1 % of the input channels scaled by
20, the activation-outlier channels that motivate activation-aware methods).
"""
import numpy as np

# (name, d_in, d_out) of one decoder layer's linears
LLAMA3_8B = [("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
             ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096)]
LLAMA3_70B = [("q", 8192, 8192), ("k", 8192, 1024), ("v", 8192, 1024), ("o", 8192, 8192),
              ("gate", 8192, 28672), ("up", 8192, 28672), ("down", 28672, 8192)]

BASE_SEED = 2410_21271_00


def seed_for(config, linear_index=0):
    return BASE_SEED + 100 * config + linear_index


def quantize_rtn(W, bits, group):
    """Round-to-nearest min/max asymmetric quantiser per (row, group of `group`
    input columns).  Returns codes u8 (rows x K), zeros u8 and scales fp16
    (rows x K/group).  The range always contains 0; the fp16-rounded scale is
    the one used to form the codes."""
    W = np.asarray(W, dtype=np.float32)
    rows, K = W.shape
    qmax = (1 << bits) - 1
    Wg = W.reshape(rows, K // group, group)
    lo = np.minimum(Wg.min(axis=2), 0.0)
    hi = np.maximum(Wg.max(axis=2), 0.0)
    s32 = (hi - lo) / qmax
    s32 = np.where(s32 == 0, 1.0, s32)
    s16 = s32.astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(np.float32)
    z = np.clip(np.rint(-lo / s), 0, qmax)
    q = np.clip(np.rint(Wg / s[:, :, None]) + z[:, :, None], 0, qmax)
    return q.reshape(rows, K).astype(np.uint8), z.astype(np.uint8), s16


def quantize_sym4(Mat, KT):
    """Symmetric 4-bit quantiser for an EoRA factor: implicit zero-point 8, one
    fp16 scale per (row, group of KT columns).  Returns codes u8 in 1..15 and scales fp16."""
    Mat = np.asarray(Mat, dtype=np.float32)
    rows, K = Mat.shape
    Mg = Mat.reshape(rows, K // KT, KT)
    amax = np.abs(Mg).max(axis=2)
    s16 = (amax / 7.0).astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(np.float32)
    q = np.clip(np.rint(Mg / s[:, :, None]) + 8, 1, 15)
    return q.reshape(rows, K).astype(np.uint8), s16


def prune_24(W16):
    """Magnitude 2:4 pruning: in every four consecutive input columns keep the two
    of largest magnitude (ties keep the lower column).  Returns kept values fp16
    (rows x K/2) and their positions u8 in 0..3, ascending within each pair."""
    W16 = np.asarray(W16, dtype=np.float16)
    rows, K = W16.shape
    w4 = W16.reshape(rows, K // 4, 4)
    g = np.abs(w4)
    # rank of each element inside its group = number of elements that beat it (larger magnitude, or
    # equal magnitude and lower column); the two of rank 0 and 1 are kept.  Same result as a stable
    # descending sort, without sorting.
    rank = np.zeros(g.shape, dtype=np.int8)
    for i in range(4):
        for jdx in range(4):
            if i != jdx:
                beats = (g[:, :, jdx] > g[:, :, i]) if jdx > i else (g[:, :, jdx] >= g[:, :, i])
                rank[:, :, i] += beats
    keepmask = rank < 2                                    # exactly two per group
    pos = np.nonzero(keepmask.reshape(-1, 4))[1].reshape(rows, K // 2).astype(np.uint8)   # ascending within a group
    vals = w4[keepmask].reshape(rows, K // 2)
    return vals, pos


def quantize_sym3(Mat, KT=128):
    """Symmetric 3-bit quantiser for an EoRA factor: implicit zero-point 4, one fp16 scale per
    (row, group of KT columns).  Returns codes u8 in 1..7 and scales fp16."""
    Mat = np.asarray(Mat, dtype=np.float32)
    rows, K = Mat.shape
    Mg = Mat.reshape(rows, K // KT, KT)
    amax = np.abs(Mg).max(axis=2)
    s16 = (amax / 3.0).astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(np.float32)
    q = np.clip(np.rint(Mg / s[:, :, None]) + 4, 1, 7)
    return q.reshape(rows, K).astype(np.uint8), s16


def quantize_kept_rtn(vals, pos, group, bits=4):
    """Round-to-nearest min/max asymmetric quantiser of the KEPT values of a 2:4-pruned matrix, per
    (row, group of `group` dense columns); the group of a kept value is that of its dense column.
    Returns codes u8 (rows x K/2), zeros u8 and scales fp16 (rows x K/group).  The range always
    contains 0; the fp16-rounded scale is the one used to form the codes."""
    vals = np.asarray(vals, dtype=np.float32)
    rows, half = vals.shape
    K = 2 * half
    kept_per_group = group // 2                      # every four dense columns keep two
    qmax = (1 << bits) - 1
    Vg = vals.reshape(rows, K // group, kept_per_group)
    lo = np.minimum(Vg.min(axis=2), 0.0)
    hi = np.maximum(Vg.max(axis=2), 0.0)
    s32 = (hi - lo) / qmax
    s32 = np.where(s32 == 0, 1.0, s32)
    s16 = s32.astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(np.float32)
    z = np.clip(np.rint(-lo / s), 0, qmax)
    q = np.clip(np.rint(Vg / s[:, :, None]) + z[:, :, None], 0, qmax)
    return q.reshape(rows, half).astype(np.uint8), z.astype(np.uint8), s16


def draw_layer(seed, d_in, d_out, M, r, outlier_frac=0.0, outlier_scale=20.0):
    """Draw (W fp32, A fp16, B fp16, x fp16) in that order from PCG64(seed)."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(0.02)
    if r > 0:
        A = (rng.standard_normal((r, d_in), dtype=np.float32) * np.float32(0.01)).astype(np.float16)
        B = (rng.standard_normal((d_out, r), dtype=np.float32) * np.float32(0.01)).astype(np.float16)
    else:
        A = np.zeros((0, d_in), np.float16)
        B = np.zeros((d_out, 0), np.float16)
    x = rng.standard_normal((M, d_in), dtype=np.float32)
    if outlier_frac > 0:
        n_out = max(1, int(round(outlier_frac * d_in)))
        ch = rng.choice(d_in, size=n_out, replace=False)
        x[:, ch] *= np.float32(outlier_scale)
    return W, A, B, x.astype(np.float16)


def draw_calibration(seed, d_in, n_tokens, outlier_frac=0.01, outlier_scale=20.0):
    """Calibration activations X-tilde (d_in x n_tokens fp32, one column per token) from PCG64(seed):
    N(0,1) with per-channel energies spread over e^-1 .. e^1 and a fraction of outlier channels, the
    shape activation statistics of LLM layers have (stand-in for the paper's calibration sets, Sec. 4.1)."""
    rng = np.random.default_rng(seed)
    Xt = rng.standard_normal((d_in, n_tokens), dtype=np.float32)
    scale = np.exp(rng.uniform(-1.0, 1.0, d_in)).astype(np.float32)
    if outlier_frac > 0:
        n_out = max(1, int(round(outlier_frac * d_in)))
        ch = rng.choice(d_in, size=n_out, replace=False)
        scale[ch] *= np.float32(outlier_scale)
    return Xt * scale[:, None]
