"""GPU parity of the fused activation producers (Section 4.1.3) against the CPU
oracle.  The producer's fp16 output h is computed in fp32 on the GPU and in fp64
by the oracle, so it may differ by one fp16 ulp where the exact value lies next
to a rounding boundary; the codes and scales must then be, bit for bit, what the
oracle's quantizer gives for the GPU's own h."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_04405_amd as fq
from paper_2508_04405_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def ordered(h):
    """Map fp16 bit patterns to integers that order like the values."""
    b = h.view(np.uint16).astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7fff), b)


def check_h(h_gpu, h_ref):
    d = np.abs(ordered(h_gpu) - ordered(h_ref))
    assert d.max() <= 1, (int((d > 1).sum()), h_gpu[d > 1][:5], h_ref[d > 1][:5])
    # fp32 error is ~2^-21 relative against a half-ulp of 2^-11: boundary cases are rare
    assert (d != 0).mean() < 1e-2, float((d != 0).mean())


def check_quant_of(h_gpu, xq, sx, bits):
    rq, rs = oracle.quantize(h_gpu.astype(np.float32), bits, 0)
    assert np.array_equal(sx.cpu().numpy().view(np.uint16), rs.view(np.uint16))
    assert np.array_equal(xq.cpu().numpy(), rq)


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("M,K", [(1, 128), (37, 1152), (5, 8192), (3, 11008), (3, 28672),
                                 (2, 40960)])
def test_rmsnorm_quant(M, K, bits):
    say(f"rmsnorm_quant M={M} K={K} bits={bits}")
    x = synth.activations(M, K, seed=31 + K, outlier_frac=0.01)
    if M > 1:
        x[1] = 0.0                              # zero token: h = 0, scale 1
    if M > 2:
        x[2] *= np.float16(1.0 / 256)           # small token
    gamma = synth.norm_gain(K, seed=5)
    eps = 1e-5
    xq, sx, h = fq.rmsnorm_quant(to_dev(x), to_dev(gamma), eps, bits, want_h=True)
    h_gpu = h.cpu().numpy()
    check_h(h_gpu, oracle.rmsnorm(x, gamma, eps))
    check_quant_of(h_gpu, xq, sx, bits)
    # without the fp16 copy, and against the stand-alone quantizer on h
    xq2, sx2 = fq.rmsnorm_quant(to_dev(x), to_dev(gamma), eps, bits)
    assert torch.equal(xq2, xq) and torch.equal(sx2.view(torch.int16), sx.view(torch.int16))
    xq3, sx3 = fq.quant_act(h, bits)
    assert torch.equal(xq3, xq) and torch.equal(sx3.view(torch.int16), sx.view(torch.int16))


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("M,F", [(1, 128), (37, 1152), (3, 11008), (3, 28672), (2, 40960)])
def test_swiglu_quant(M, F, bits):
    say(f"swiglu_quant M={M} F={F} bits={bits}")
    gu = synth.gate_up(M, F, seed=77 + F)
    # the gate's extremes: silu(-large) = -0, silu(large) = large, silu(0) = 0
    gu[0, :8] = [0.0, -0.0, 20.0, -20.0, 88.0, -88.0, 1000.0, -65504.0]
    gu[0, F:F + 8] = [3.0, 3.0, -2.0, -2.0, 0.5, 0.5, 1.0, 65504.0]
    if M > 1:
        gu[1] = 0.0                             # zero token
    xq, sx, h = fq.swiglu_quant(to_dev(gu), bits, want_h=True)
    h_gpu = h.cpu().numpy()
    assert np.isfinite(h_gpu.astype(np.float32)).all()
    check_h(h_gpu, oracle.swiglu(gu))
    check_quant_of(h_gpu, xq, sx, bits)
    xq2, sx2 = fq.swiglu_quant(to_dev(gu), bits)
    assert torch.equal(xq2, xq) and torch.equal(sx2.view(torch.int16), sx.view(torch.int16))


def test_producers_feed_the_linear():
    """norm -> quantized linear -> gated SiLU -> quantized linear, codes handed from
    kernel to kernel; every stage is compared with the oracle on the GPU's own inputs."""
    say("producer chain M=24 K=1024 F=1408")
    M, K, F = 24, 1024, 1408
    x = synth.activations(M, K, seed=3)
    gamma = synth.norm_gain(K, seed=4)
    w_gu = synth.weights(2 * F, K, 0.02, seed=5)
    w_dn = synth.weights(K, F, 0.02, seed=6)
    p_gu = fq.pack_w6(*fq.quant_w6(to_dev(w_gu), 0), 0)
    p_dn = fq.pack_w6(*fq.quant_w6(to_dev(w_dn), 0), 0)

    xq, sx, h = fq.rmsnorm_quant(to_dev(x), to_dev(gamma), 1e-5, 6, want_h=True)
    gu = fq.gemm_w6a6(p_gu, 2 * F, K, xq=xq, sx=sx)
    ref = oracle.linear(h.cpu().numpy(), w_gu, 6, 0)
    assert np.array_equal(ref["xq"], xq.cpu().numpy())
    d = np.abs(ordered(gu.cpu().numpy()) - ordered(ref["y"]))
    assert d.max() <= 1

    aq, sa, a = fq.swiglu_quant(gu, 8, want_h=True)
    check_h(a.cpu().numpy(), oracle.swiglu(gu.cpu().numpy()))
    y = fq.gemm_w6a8(p_dn, K, F, xq=aq, sx=sa)
    ref2 = oracle.linear(a.cpu().numpy(), w_dn, 8, 0)
    assert np.array_equal(ref2["xq"], aq.cpu().numpy())
    d = np.abs(ordered(y.cpu().numpy()) - ordered(ref2["y"]))
    assert d.max() <= 1
