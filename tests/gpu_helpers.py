"""Helpers shared by the GPU parity tests: device transfer, fp16 comparison to the bar
(one ulp; group mode plus the fp32 summation bound), GPU-side quantize + pack of seeded
weights, stratified sampling of the outputs of full-size cases."""
import numpy as np
import torch

import paper_2508_04405_amd as fq
from paper_2508_04405_amd import synth

DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def ordered(h):
    """Map fp16 bit patterns to integers that order like the values."""
    b = h.view(np.uint16).astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7fff), b)


def assert_y_close(got, want, slack=None):
    """Within 1 fp16 ulp.  `slack` (absolute, per element) widens it where the
    kernel sums fp32 group terms in its own order."""
    got = np.asarray(got)
    want = np.asarray(want)
    d = np.abs(ordered(got) - ordered(want))
    bad = d > 1
    if slack is not None:
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        ulp = np.abs(want.astype(np.float64)) * 2.0**-10 + 2.0**-24
        bad &= err > ulp + slack
        # The bound is a worst case; with rounding errors of random sign the fp32 sum of G
        # terms is off by about sqrt(G) 2^-25 of a typical term, which crosses a second
        # fp16 boundary only where the terms cancel almost completely.  So at most one
        # output in a thousand (two, for small cases) may lie beyond one ulp at all.
        beyond = int((d > 1).sum())
        say(f"    group mode: {d.size} outputs, beyond 1 ulp: {beyond}, worst distance {int(d.max())} ulp")
        assert beyond <= max(2, d.size // 1000), (beyond, d.size)
    assert not bad.any(), (int(bad.sum()), got[bad][:5], want[bad][:5])
    rel = np.abs(got.astype(np.float64) - want.astype(np.float64))
    big = np.abs(want.astype(np.float64)) > 2.0**-14
    if slack is None:
        assert np.all(rel[big] <= 1e-3 * np.abs(want.astype(np.float64))[big])


def prepare(w, group=0):
    """fp32 weights -> GPU quantize + pack; returns (packed, wq, sw) on device."""
    wq, sw = fq.quant_w6(to_dev(w), group)
    return fq.pack_w6(wq, sw, group), wq, sw


def group_slack(ref):
    # fp32 sum of G terms in any order: at most G * 2^-23 * sum |term|, times sx
    terms = np.abs(ref["acc_g"].astype(np.float64) * ref["sw"].astype(np.float64)[None, :, :])
    G = terms.shape[2]
    return ref["sx"].astype(np.float64)[:, None] * terms.sum(2) * G * 2.0**-23


def build_packed(N, K, sigma, seed, group=0):
    """Quantize + pack W[N,K] on the GPU in row blocks (bounds host memory)."""
    wq = torch.empty((N, K), dtype=torch.int8, device=DEV)
    sw = torch.empty((N,) if group == 0 else (N, K // 128), dtype=torch.float16, device=DEV)
    step = 4096
    for r0 in range(0, N, step):
        r1 = min(N, r0 + step)
        q, s = fq.quant_w6(to_dev(synth.weight_rows(N, K, sigma, seed, r0, r1)), group)
        wq[r0:r1] = q
        sw[r0:r1] = s
    packed = fq.pack_w6(wq, sw, group)
    del wq
    return packed


def stratified(total, block, rng, extra=()):
    """One seeded index in every `block`-wide slice of range(total), plus `extra`."""
    starts = np.arange(0, total, block)
    picks = starts + rng.integers(0, block, starts.size)
    return np.unique(np.concatenate([np.minimum(picks, total - 1), np.asarray(extra, dtype=np.int64)]))


def sampled_columns(N, K, sigma, seed):
    """The output columns a full-size case checks, and their weight rows: one column in
    every 32-column block (every weight tile, hence every workgroup tile and every slot of
    the kernels' tile orders, is hit), plus the edges of the first two blocks and the last."""
    cols = stratified(N, 32, np.random.default_rng(seed + 1), [0, 31, 32, N - 1])
    return cols, synth.weight_rows_at(N, K, sigma, seed, cols)


