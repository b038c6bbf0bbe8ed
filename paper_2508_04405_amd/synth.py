"""Seeded synthetic inputs shaped like the paper's linear-layer workloads.

This module holds no arithmetic of the method: it only draws real-valued
weights and activations.  Both the GPU path and the CPU checker start from
these same arrays.

Weights are i.i.d. N(0, sigma) in fp32, drawn per block of rows so that any
row range of a large matrix can be regenerated without building all of it.
Activations are fp16 N(0, 1) with a seeded subset of the K channels multiplied
by a constant for every token: the channel-persistent outliers the paper shows
for LLaMA activations (Section 3.2, Challenge 1 and its figure).
"""
import numpy as np

ROW_BLOCK = 256

# (K, N) of the linear layers the paper benchmarks at kernel level, by model
# (Section 5.2, "Kernel Performance"): fused QKV, attention output, fused
# gate+up, down projection.
LLAMA2_7B = {"qkv": (4096, 12288), "o": (4096, 4096), "gate_up": (4096, 22016),
             "down": (11008, 4096)}
LLAMA2_70B = {"qkv": (8192, 10240), "o": (8192, 8192), "gate_up": (8192, 57344),
              "down": (28672, 8192)}
LLAMA2_13B = {"q": (5120, 5120), "k": (5120, 5120), "v": (5120, 5120), "o": (5120, 5120),
              "gate": (5120, 13824), "up": (5120, 13824), "down": (13824, 5120)}


def weight_rows(N, K, sigma, seed, row0, row1):
    """Rows [row0, row1) of the seeded fp32 weight matrix W[N, K]."""
    assert 0 <= row0 <= row1 <= N
    out = np.empty((row1 - row0, K), dtype=np.float32)
    b0, b1 = row0 // ROW_BLOCK, (row1 + ROW_BLOCK - 1) // ROW_BLOCK
    for b in range(b0, b1):
        lo, hi = b * ROW_BLOCK, min((b + 1) * ROW_BLOCK, N)
        rng = np.random.default_rng([seed, b])
        blk = rng.standard_normal((hi - lo, K), dtype=np.float32) * np.float32(sigma)
        s, e = max(lo, row0), min(hi, row1)
        out[s - row0:e - row0] = blk[s - lo:e - lo]
    return out


def weights(N, K, sigma, seed):
    """The whole seeded fp32 weight matrix W[N, K] (K contiguous)."""
    return weight_rows(N, K, sigma, seed, 0, N)


def weight_rows_at(N, K, sigma, seed, rows):
    """The listed rows of W[N, K], regenerated block by block."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((rows.size, K), dtype=np.float32)
    blocks = {}
    for i, r in enumerate(rows):
        b = int(r) // ROW_BLOCK
        if b not in blocks:
            blocks = {b: weight_rows(N, K, sigma, seed, b * ROW_BLOCK, min((b + 1) * ROW_BLOCK, N))}
        out[i] = blocks[b][int(r) - b * ROW_BLOCK]
    return out


def activations(M, K, seed, outlier_frac=0.01, outlier_scale=20.0):
    """fp16 X[M, K]: N(0, 1) with a seeded set of outlier channels scaled up."""
    rng = np.random.default_rng([seed, 7])
    x = rng.standard_normal((M, K), dtype=np.float32)
    n_out = int(round(outlier_frac * K))
    if n_out > 0:
        ch = np.random.default_rng([seed, 11]).choice(K, size=n_out, replace=False)
        x[:, ch] *= np.float32(outlier_scale)
    return x.astype(np.float16)


def norm_gain(K, seed):
    """fp16 gamma[K] of an RMS-norm layer: 1 + 0.1 N(0, 1), a few channels amplified the way
    trained norms amplify outlier channels."""
    rng = np.random.default_rng([seed, 13])
    g = 1.0 + 0.1 * rng.standard_normal(K, dtype=np.float32)
    ch = rng.choice(K, size=max(1, K // 256), replace=False)
    g[ch] *= np.float32(4.0)
    return g.astype(np.float16)


def gate_up(M, F, seed):
    """fp16 [M, 2F]: the output of a fused gate|up projection, N(0, 1.5) with sparse large
    entries (the massive activations ahead of a down projection)."""
    rng = np.random.default_rng([seed, 17])
    gu = np.float32(1.5) * rng.standard_normal((M, 2 * F), dtype=np.float32)
    hits = rng.random((M, 2 * F), dtype=np.float32) < np.float32(5e-4)
    gu[hits] *= np.float32(12.0)
    return gu.astype(np.float16)
