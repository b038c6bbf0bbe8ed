"""GPU parity of activations quantized into tile order (Section 4.3.1: the activations are
packed online as well; 6-bit activations travel at 0.75 byte per value) and of the
streaming kernel reading them (flexq_quant_act_tiles, flexq_untile_act, flexq_gemv_tiles,
and the calls that take fp16 activations and go that way by themselves).

The tile order is the library's own format, so it is checked through what it must
preserve: un-tiling gives back, bit for bit, the codes of the oracle's quantizer; the
6-bit tile of 32 tokens is byte for byte the weight packer's tile of the same codes; and
the linear layer on tiles equals the oracle's to the usual bar (int32 sums bit-exact,
fp16 outputs within one ulp)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_04405_amd as fq
from paper_2508_04405_amd import dev, synth
from gpu_helpers import DEV, assert_y_close, build_packed, group_slack, prepare, sampled_columns, say, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("M,K", [(1, 128), (5, 256), (17, 1024), (32, 8192), (33, 640), (70, 28672), (128, 4096)])
def test_quantize_into_tiles_round_trip(bits, M, K):
    say(f"activation tiles A{bits} M={M} K={K}")
    x = synth.activations(M, K, seed=900 + M, outlier_frac=0.02)
    ref_q, ref_s = oracle.quantize(x.astype(np.float32), bits)
    xt, sx = fq.quant_act_tiles(to_dev(x), bits)
    blocks = (M + 31) // 32
    assert xt.numel() == blocks * (K // 128) * (3072 if bits == 6 else 4096)
    if bits == 6:
        assert xt.numel() * 4 == blocks * 32 * K * 3          # exactly 6 bits a value
    assert np.array_equal(sx.cpu().numpy().view(np.uint16), ref_s.view(np.uint16))
    back = fq.untile_act(xt, M, K, bits).cpu().numpy()
    assert np.array_equal(back, ref_q)
    # the row-major quantizer gives the same codes and scales
    xq, sx2 = fq.quant_act(to_dev(x), bits)
    assert torch.equal(sx, sx2) and np.array_equal(xq.cpu().numpy(), back)


@pytest.mark.parametrize("M,K", [(32, 384), (64, 1024)])
def test_six_bit_tiles_are_the_weight_tile_format(M, K):
    """Whole blocks of 32 tokens: the packed activation tiles are the bytes the weight
    packer makes of the same codes (tokens in the place of output channels)."""
    x = synth.activations(M, K, seed=77, outlier_frac=0.05)
    xt, _ = fq.quant_act_tiles(to_dev(x), 6)
    xq, _ = fq.quant_act(to_dev(x), 6)
    as_weights = fq.pack_w6(xq, torch.ones((M,), dtype=torch.float16, device=DEV), 0)
    assert torch.equal(xt, as_weights[: M * K * 3 // 4])


def check_linear(y, acc, ref, group):
    if group == 0:
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), ref["acc"])
    assert_y_close(y.cpu().numpy().view(np.float16), ref["y"], slack=group_slack(ref) if group else None)


@pytest.mark.parametrize("group", [0, 128])
@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("M,K,N", [(1, 256, 64), (9, 1024, 96), (16, 8192, 256), (31, 640, 160), (32, 2048, 512)])
def test_linear_on_tiles(M, K, N, bits, group):
    say(f"linear on activation tiles M={M} K={K} N={N} A{bits} group={group}")
    w = synth.weights(N, K, 0.02, seed=300 + M)
    x = synth.activations(M, K, seed=400 + M, outlier_frac=0.02)
    ref = oracle.linear(x, w, bits, group)
    packed, _, _ = prepare(w, group)
    xt, sx = fq.quant_act_tiles(to_dev(x), bits)
    ws = fq.make_workspace(M, N, K)
    for _ in range(2):
        if group == 0:
            y, acc = fq.gemv_tiles(bits, packed, N, K, group, xt, sx, workspace=ws, want_acc=True)
        else:
            y, acc = fq.gemv_tiles(bits, packed, N, K, group, xt, sx, workspace=ws), None
        check_linear(y, acc, ref, group)
    assert int(ws[:16384].view(torch.int32).abs().sum().item()) == 0


@pytest.mark.parametrize("split,waves", [(1, 4), (2, 8), (3, 4), (5, 8)])
@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("group", [0, 128])
def test_fp16_calls_through_tiles_with_k_splits(split, waves, bits, group):
    """The calls that take fp16 activations, made to go through tile order (development
    library), with the streaming kernel's K splits and workgroup sizes forced."""
    M, K, N = 20, 1408, 192                       # 11 tiles along k: uneven splits
    say(f"fp16 -> tiles -> streaming kernel, split={split} waves={waves} A{bits} group={group}")
    w = synth.weights(N, K, 0.02, seed=17)
    x = synth.activations(M, K, seed=18, outlier_frac=0.02)
    ref = oracle.linear(x, w, bits, group)
    packed, _, _ = prepare(w, group)
    ws = fq.make_workspace(M, N, K, extra=split * M * N * 4)
    dev.set_dispatch(1, split, waves)
    dev.set_tiles(1)
    try:
        fn = dev.gemv_w6a6 if bits == 6 else dev.gemv_w6a8
        for _ in range(3):
            if group == 0:
                y, acc = fn(packed, N, K, 0, x_fp16=to_dev(x), workspace=ws, want_acc=True)
            else:
                y, acc = fn(packed, N, K, group, x_fp16=to_dev(x), workspace=ws), None
            assert dev.last_dispatch() == (1, 500 + split)
            check_linear(y, acc, ref, group)
        dev.set_tiles(2)
        y2 = fn(packed, N, K, group, x_fp16=to_dev(x), workspace=ws)
        assert dev.last_dispatch() == (1, split)
        if group == 0:
            assert torch.equal(y2, y)             # the same sums, the same epilogue arithmetic
        else:                                     # fp32 group sums of 16x and 4x operands: same value, own rounding
            assert_y_close(y2.cpu().numpy().view(np.float16), ref["y"], slack=group_slack(ref))
    finally:
        dev.set_dispatch(0, 0)
        dev.set_tiles(0)
    assert int(ws[:16384].view(torch.int32).abs().sum().item()) == 0


@pytest.mark.parametrize("layer,K,N,bits", [("qkv", 8192, 10240, 6), ("down", 28672, 8192, 8),
                                             ("gate_up", 8192, 57344, 6)])
@pytest.mark.parametrize("M", [24, 32])
def test_full_size_fp16_calls_choose_tiles(layer, K, N, bits, M):
    """LLaMA-2-70B layers at 24 and 32 tokens through the library's own dispatch, fp16 in:
    the activations go through tile order (their slice does not fit the LDS staging; on
    the 57344-wide gate+up, 6-bit activations only: packed tiles are what makes streaming
    faster than the tiled kernel there); one output column in every 32-column block
    against the oracle."""
    say(f"full size through tiles: {layer} M={M} A{bits}")
    seed = 5100 + K // 1000
    packed = build_packed(N, K, 0.015, seed)
    cols, w_cols = sampled_columns(N, K, 0.015, seed)
    x = synth.activations(M, K, seed=seed + M, outlier_frac=0.01)
    ref = oracle.linear(x, w_cols, bits)
    fn = dev.gemv_w6a6 if bits == 6 else dev.gemv_w6a8
    y, acc = fn(packed, N, K, 0, x_fp16=to_dev(x), want_acc=True)
    kernel, code = dev.last_dispatch()
    assert kernel == 1 and code >= 500, (kernel, code)
    assert np.array_equal(acc[:, to_dev(cols)].cpu().numpy().astype(np.int64), ref["acc"])
    assert_y_close(y[:, to_dev(cols)].cpu().numpy().view(np.float16), ref["y"])
    # and the product library's call gives the same bits
    y_prod = (fq.gemv_w6a6 if bits == 6 else fq.gemv_w6a8)(packed, N, K, 0, x_fp16=to_dev(x))
    assert torch.equal(y_prod, y)
