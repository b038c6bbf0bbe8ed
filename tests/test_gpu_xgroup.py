"""GPU parity of the scheme with group-128 scales on BOTH operands (Section 4.1.1, Eq. 7)
against the CPU oracle: codes and scales bit-exact, outputs within one fp16 ulp plus the
bound of an fp32 sum of K/128 terms taken in the kernel's own order."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_04405_amd as fq
from paper_2508_04405_amd import dev, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def ordered(h):
    b = h.view(np.uint16).astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7fff), b)


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("M,K", [(1, 128), (37, 1152), (130, 8192), (3, 65536)])
def test_quant_act_g128_bit_exact(M, K, bits):
    say(f"quant_act_g128 M={M} K={K} bits={bits}")
    qmax = 31 if bits == 6 else 127
    x = synth.activations(M, K, seed=50 + K, outlier_frac=0.02).astype(np.float32)
    x[0, :128] = 0.0                                     # an all-zero group
    if K >= 256:
        ks = np.arange(128) % (2 * qmax) - qmax
        x[0, 128:256] = (ks + 0.5) * 0.5                 # every quotient a tie
        x[0, 128] = qmax * 0.5
    if M > 1:
        x[1, :128] = 0.0
        x[1, 5] = 6e-8                                   # fp16 subnormal input
    x16 = x.astype(np.float16)
    xq, sxg = fq.quant_act_g128(to_dev(x16), bits)
    rq, rs = oracle.quantize(x16.astype(np.float32), bits, 128)      # rs is [M, K/128]
    assert np.array_equal(sxg.cpu().numpy().view(np.uint16)[:, :M], rs.view(np.uint16).T)
    assert np.array_equal(xq.cpu().numpy(), rq)


def summation_slack(acc_g, sxg, sw):
    """Eq. 7 summed in fp32 in the kernel's own order.  Every rounding is at most 2^-24 of
    a partial sum, itself at most T = sum_g |sx_g sw_g acc_g|.  The kernels make: one
    rounding per term (its product, or the fused multiply-add that adds it), one more per
    term where both scales multiply it separately, at most G - 1 further additions when
    the wavefronts' and K splits' partial sums are combined (an empty partial adds
    exactly), and one for the token scale applied at the end: fewer than
    (2 G + 4) 2^-24 T = (G + 2) 2^-23 T in all, which is the slack returned."""
    terms = np.abs(acc_g.astype(np.float64) * sw.astype(np.float64)[None, :, :] *
                   sxg.astype(np.float64)[:, None, :])
    return terms.sum(2) * (terms.shape[2] + 2) * 2.0**-23


def reference(x16, w, bits):
    wq, sw = oracle.quantize(w, 6, 128)
    xq, sxg = oracle.quantize(x16.astype(np.float32), bits, 128)
    acc_g = oracle.matmul(xq, wq, 128)                               # [M, N, G]
    y = oracle.dequant_xgroup(acc_g, sxg, sw)
    return xq, sxg, y, summation_slack(acc_g, sxg, sw)


def assert_close(got, want, slack, what=""):
    """Within one fp16 ulp, or within one ulp plus the fp32 summation bound `slack`.  The
    bound is a worst case: with rounding errors of random sign the fp32 sum is off by about
    sqrt(G) 2^-25 of a typical term, which moves a result past a second fp16 boundary only
    where the terms cancel almost completely.  So besides the bound itself, at most one
    output in a thousand (two outputs, for small cases) may need it, and the worst distance
    is printed."""
    d = np.abs(ordered(got) - ordered(want))
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    ulp = np.abs(want.astype(np.float64)) * 2.0**-10 + 2.0**-24
    bad = (d > 1) & (err > ulp + slack)
    beyond = int((d > 1).sum())
    print(f"    {what} outputs {d.size}, beyond 1 ulp: {beyond}, worst distance {int(d.max())} ulp", flush=True)
    assert not bad.any(), (int(bad.sum()), got[bad][:5], want[bad][:5])
    assert beyond <= max(2, d.size // 1000), (beyond, d.size)


CASES = [(1, 256, 128), (4, 1280, 160), (8, 4096, 64), (32, 1024, 320), (33, 640, 96),
         (64, 2048, 128), (100, 1024, 64), (200, 512, 128), (129, 128, 32), (300, 1408, 288)]


@pytest.mark.parametrize("kernel", ["auto", "stream", "tiled"])
@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("M,K,N", CASES)
def test_linear_g128(M, K, N, bits, kernel):
    say(f"linear_g128 M={M} K={K} N={N} A{bits} {kernel}")
    dev.set_dispatch({"auto": 0, "stream": 1, "tiled": 2}[kernel], 0, 0, 0)
    try:
        run_linear_g128(M, K, N, bits)
        torch.cuda.synchronize()
    finally:
        dev.set_dispatch(0, 0, 0, 0)


def run_linear_g128(M, K, N, bits):
    w = synth.weights(N, K, 0.02, seed=200 + N)
    x = synth.activations(M, K, seed=300 + M, outlier_frac=0.02)
    rq, rsg, ry, slack = reference(x, w, bits)
    packed = fq.pack_w6(*fq.quant_w6(to_dev(w), 128), 128)
    xq, sxg = fq.quant_act_g128(to_dev(x), bits)
    assert np.array_equal(xq.cpu().numpy(), rq)
    assert np.array_equal(sxg.cpu().numpy().view(np.uint16)[:, :M], rsg.view(np.uint16).T)
    y = dev.linear_g128(packed, N, K, xq, sxg)
    assert_close(y.cpu().numpy(), ry, slack, "group scales:")
    # scales that are constant along K must reproduce the per-token entry point: both
    # against the oracle on those flat scales, with the summation bound of THOSE terms
    sx = sxg[0, :M].contiguous()
    flat = sxg[0][None, :].expand(K // 128, sxg.shape[1]).contiguous()
    y_tok = dev.gemv_w6a8(packed, N, K, 128, xq=xq, sx=sx)
    y_grp = dev.linear_g128(packed, N, K, xq, flat)
    wq_ref, sw_ref = oracle.quantize(w, 6, 128)
    acc_g = oracle.matmul(rq, wq_ref, 128)
    sx_flat = np.repeat(rsg[:, :1], K // 128, 1)
    ref_flat = oracle.dequant_xgroup(acc_g, sx_flat, sw_ref)
    slack_flat = summation_slack(acc_g, sx_flat, sw_ref)
    assert_close(y_grp.cpu().numpy(), ref_flat, slack_flat, "flat scales, group entry:")
    assert_close(y_tok.cpu().numpy(), ref_flat, slack_flat, "flat scales, token entry:")


@pytest.mark.parametrize("split,waves", [(2, 4), (3, 8), (5, 16)])
def test_linear_g128_k_splits(split, waves):
    say(f"linear_g128 split={split} waves={waves}")
    M, K, N = 9, 2560, 96
    w = synth.weights(N, K, 0.02, seed=7)
    x = synth.activations(M, K, seed=8, outlier_frac=0.02)
    _, _, ry, slack = reference(x, w, 8)
    packed = fq.pack_w6(*fq.quant_w6(to_dev(w), 128), 128)
    xq, sxg = fq.quant_act_g128(to_dev(x), 8)
    dev.set_dispatch(1, split, waves, 0)
    try:
        y = dev.linear_g128(packed, N, K, xq, sxg,
                            workspace=fq.make_workspace(M, N, K, DEV, extra=split * M * N * 4))
        torch.cuda.synchronize()
    finally:
        dev.set_dispatch(0, 0, 0, 0)
    assert_close(y.cpu().numpy(), ry, slack)


@pytest.mark.parametrize("split", [2, 3])
@pytest.mark.parametrize("M", [70, 260])
def test_linear_g128_tiled_k_splits(split, M):
    say(f"linear_g128 tiled split={split} M={M}")
    K, N = 2560, 160
    w = synth.weights(N, K, 0.02, seed=9)
    x = synth.activations(M, K, seed=10, outlier_frac=0.02)
    _, _, ry, slack = reference(x, w, 6)
    packed = fq.pack_w6(*fq.quant_w6(to_dev(w), 128), 128)
    xq, sxg = fq.quant_act_g128(to_dev(x), 6)
    dev.set_dispatch(2, split, 0, 0)
    try:
        y = dev.linear_g128(packed, N, K, xq, sxg,
                            workspace=fq.make_workspace(M, N, K, DEV, extra=split * M * N * 4))
        torch.cuda.synchronize()
    finally:
        dev.set_dispatch(0, 0, 0, 0)
    assert_close(y.cpu().numpy(), ry, slack)


def test_linear_g128_prefill_shape_sampled():
    """LLaMA-2-13B gate+up projection (5120 -> 13824), prefill M = 2048 (tiled kernel)."""
    say("linear_g128 13B 5120x13824 M=2048")
    M, K, N = 2048, 5120, 13824
    rows = np.unique(np.concatenate([[0, M - 1], np.random.default_rng(6).integers(0, M, 24)]))
    cols = np.unique(np.concatenate([[0, 31, 32, N - 1],
                                     np.random.default_rng(7).integers(0, N, 100)]))
    x = synth.activations(M, K, seed=24, outlier_frac=0.01)
    packed = fq.pack_w6(*fq.quant_w6(to_dev(synth.weights(N, K, 0.02, seed=23)), 128), 128)
    w_cols = synth.weight_rows_at(N, K, 0.02, 23, cols)
    _, _, ry, slack = reference(x[rows], w_cols, 8)
    xq, sxg = fq.quant_act_g128(to_dev(x), 8)
    y = fq.linear_g128(packed, N, K, xq, sxg).cpu().numpy()[np.ix_(rows, cols)]
    assert_close(y, ry, slack)


def test_linear_g128_decode_shape_sampled():
    """LLaMA-2-13B attention projection (5120 x 5120), batched decode M = 32."""
    say("linear_g128 13B 5120x5120 M=32")
    M, K, N = 32, 5120, 5120
    w = synth.weights(N, K, 0.02, seed=21)
    x = synth.activations(M, K, seed=22, outlier_frac=0.01, outlier_scale=50.0)
    cols = np.unique(np.concatenate([[0, 31, 32, N - 1],
                                     np.random.default_rng(5).integers(0, N, 150)]))
    _, _, ry, slack = reference(x, w[cols], 6)
    packed = fq.pack_w6(*fq.quant_w6(to_dev(w), 128), 128)
    xq, sxg = fq.quant_act_g128(to_dev(x), 6)
    y = fq.linear_g128(packed, N, K, xq, sxg).cpu().numpy()[:, cols]
    assert_close(y, ry, slack)
