"""GPU parity of the decoder-block runner (flexq_layer_linears: norm + quantize -> QKV,
quantize -> O, norm + quantize -> gate|up, SiLU * up + quantize -> down; Section 4.1.3)
with the paper's activation policy (Section 4.1.2: 8 bits on the down projection, 6
elsewhere), stage by stage against the CPU oracle on the GPU's own stage inputs.

For each stage: the fp16 values h the fused producer quantized (asked for through the
optional h_* outputs) are within one fp16 ulp of the oracle's producer applied to the stage's
input; the stage's output equals, to the one-ulp bar, the oracle's quantize -> integer product
-> dequantize applied to the GPU's own h, on one output column in every 32-column block.
The stages are chained as in a decoder block: the gate|up projection reads the runner's own
attention-output projection, the down projection reads its own gate|up output."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_04405_amd as fq
from paper_2508_04405_amd import synth
from gpu_helpers import DEV, assert_y_close, build_packed, group_slack, ordered, sampled_columns, say, to_dev

pytestmark = pytest.mark.gpu

MODELS = {
    # name: hidden, FFN width, fused QKV width, sigma, weight-scale group
    "7b": (4096, 11008, 12288, 0.02, 0),
    "70b": (8192, 28672, 10240, 0.015, 0),
    "13b_g128": (5120, 13824, 15360, 0.02, 128),
}


def check_h(h_gpu, h_ref):
    d = np.abs(ordered(h_gpu) - ordered(h_ref))
    assert d.max() <= 1, (int((d > 1).sum()), h_gpu[d > 1][:5], h_ref[d > 1][:5])
    assert (d != 0).mean() < 1e-2, float((d != 0).mean())


def check_stage(name, h_gpu, bits, y_gpu, cols, w_cols, group):
    """y_gpu[:, cols] against the oracle's linear layer applied to the GPU's own fp16 h."""
    ref = oracle.linear(h_gpu, w_cols, bits, group)
    got = y_gpu[:, to_dev(cols)].cpu().numpy()
    say(f"    {name}: {got.shape[0]} x {got.shape[1]} sampled outputs, A{bits}")
    assert_y_close(got.view(np.float16), ref["y"], slack=group_slack(ref) if group else None)


@pytest.mark.parametrize("model", ["7b", "70b", "13b_g128"])
def test_layer_runner_stage_by_stage(model):
    H, F, QKV, sigma, group = MODELS[model]
    # (17 to 32 tokens: the producers hand their codes over in tile order, packed at 6 bits)
    Ms = (1, 16, 24, 32, 1024) if group == 0 else (32, 300)
    seed = 7000 + H
    say(f"layer runner {model}: packing")
    shapes = {"qkv": (QKV, H), "o": (H, H), "gate_up": (2 * F, H), "down": (H, F)}
    packed, sample = {}, {}
    for i, (k, (N, K)) in enumerate(shapes.items()):
        packed[k] = build_packed(N, K, sigma, seed + i, group)
        sample[k] = sampled_columns(N, K, sigma, seed + i)
    g_attn, g_ffn = synth.norm_gain(H, seed=seed + 10), synth.norm_gain(H, seed=seed + 11)
    bits = (6, 6, 6, 8)                                  # the paper's policy
    layer = fq.Layer(H, F, QKV, group, packed["qkv"], packed["o"], packed["gate_up"], packed["down"],
                     to_dev(g_attn), to_dev(g_ffn), 1e-5, bits)
    for M in Ms:
        say(f"layer runner {model}: M={M}")
        x = synth.activations(M, H, seed=seed + 20 + M, outlier_frac=0.01)
        attn = synth.activations(M, H, seed=seed + 30 + M, outlier_frac=0.01)
        buf = {k: torch.empty((M, n), dtype=torch.float16, device=DEV)
               for k, n in (("qkv", QKV), ("o", H), ("gate_up", 2 * F), ("down", H), ("h_attn_norm", H),
                            ("h_ffn_norm", H), ("h_swiglu", F))}
        ws = layer.make_workspace(M)
        for rep in range(2):                             # the workspace is ready for the next call
            fq.layer_linears(layer, M, ws, x=to_dev(x), attn=to_dev(attn), x_ffn=buf["o"], **buf)
        torch.cuda.synchronize()
        assert int(ws[:16384].view(torch.int32).abs().sum().item()) == 0

        # stage 0: RMS norm + quantize -> QKV
        h0 = buf["h_attn_norm"].cpu().numpy()
        check_h(h0, oracle.rmsnorm(x, g_attn, 1e-5))
        check_stage("qkv", h0, bits[0], buf["qkv"], *sample["qkv"], group)
        # stage 1: quantize -> O (the producer is the identity: h is the attention output)
        check_stage("o", attn, bits[1], buf["o"], *sample["o"], group)
        # stage 2: RMS norm of the runner's own o + quantize -> gate|up
        o_gpu = buf["o"].cpu().numpy()
        h2 = buf["h_ffn_norm"].cpu().numpy()
        check_h(h2, oracle.rmsnorm(o_gpu, g_ffn, 1e-5))
        check_stage("gate_up", h2, bits[2], buf["gate_up"], *sample["gate_up"], group)
        # stage 3: SiLU(gate) * up of the runner's own gate|up + quantize (8 bits) -> down
        gu_gpu = buf["gate_up"].cpu().numpy()
        h3 = buf["h_swiglu"].cpu().numpy()
        check_h(h3, oracle.swiglu(gu_gpu))
        check_stage("down", h3, bits[3], buf["down"], *sample["down"], group)

        # the same stages in two calls around the caller's attention, without the optional
        # outputs: identical results
        again = {k: torch.empty_like(buf[k]) for k in ("qkv", "o", "gate_up", "down")}
        fq.layer_linears(layer, M, ws, 0, 0, x=to_dev(x), qkv=again["qkv"])
        fq.layer_linears(layer, M, ws, 1, 3, attn=to_dev(attn), o=again["o"], x_ffn=again["o"],
                         gate_up=again["gate_up"], down=again["down"])
        torch.cuda.synchronize()
        for k in again:
            assert torch.equal(again[k], buf[k]), k


def test_layer_runner_all_eight_bits_differs_and_matches():
    """A layer flagged for 8-bit activations on all seven linears (the outlier-heavy layers
    of the 13B configuration): same checks on the gate|up stage, and its codes differ from
    the 6-bit policy's."""
    H, F, QKV, sigma, group = 1024, 2816, 3072, 0.02, 128
    M, seed = 40, 7700
    shapes = {"qkv": (QKV, H), "o": (H, H), "gate_up": (2 * F, H), "down": (H, F)}
    packed = {k: build_packed(N, K, sigma, seed + i, group) for i, (k, (N, K)) in enumerate(shapes.items())}
    g = to_dev(synth.norm_gain(H, seed=seed + 10))
    x = synth.activations(M, H, seed=seed + 20, outlier_frac=0.01, outlier_scale=50.0)
    outs = {}
    for bits in ((6, 6, 6, 8), (8, 8, 8, 8)):
        layer = fq.Layer(H, F, QKV, group, packed["qkv"], packed["o"], packed["gate_up"], packed["down"],
                         g, g, 1e-5, bits)
        ws = layer.make_workspace(M)
        qkv = torch.empty((M, QKV), dtype=torch.float16, device=DEV)
        h = torch.empty((M, H), dtype=torch.float16, device=DEV)
        fq.layer_linears(layer, M, ws, 0, 0, x=to_dev(x), qkv=qkv, h_attn_norm=h)
        torch.cuda.synchronize()
        w = synth.weights(QKV, H, sigma, seed)
        ref = oracle.linear(h.cpu().numpy(), w, bits[0], group)
        assert_y_close(qkv.cpu().numpy().view(np.float16), ref["y"], slack=group_slack(ref))
        outs[bits[0]] = qkv.clone()
    assert not torch.equal(outs[6], outs[8])
