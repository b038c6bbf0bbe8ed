"""The entry point that allocates nothing (flexq_gemv_w6a8_noalloc: its workspace is a
fixed array inside the library's device image) against flexq_gemv_w6a8 on a caller's
workspace: same kernels, so the outputs must be identical, bit for bit, and the int32 sums
must equal the oracle's.  Two calls in a row, the second with a smaller input, so whatever
the first left in the shared array is there when the second runs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_04405_amd as fq
from paper_2508_04405_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def test_noalloc_matches_the_workspace_entry_point():
    # K splits (few row blocks) so that counters and partial sums in the array are in use;
    # the second case is smaller in every dimension and takes the fused quantize prologue
    cases = [(16, 2048, 512, False), (3, 1024, 256, True), (1, 8192, 8192, False)]
    for M, K, N, fp16_in in cases:
        print(f"noalloc: M={M} K={K} N={N} fp16_in={fp16_in}", flush=True)
        w = synth.weights(N, K, 0.02, seed=700 + M)
        x = synth.activations(M, K, seed=800 + M, outlier_frac=0.02)
        ref = oracle.linear(x, w, 8)
        packed = fq.pack_w6(*fq.quant_w6(to_dev(w)))
        if fp16_in:
            args = dict(x_fp16=to_dev(x))
        else:
            xq, sx = fq.quant_act(to_dev(x), 8)
            args = dict(xq=xq, sx=sx)
        y_ws, acc_ws = fq.gemv_w6a8(packed, N, K, 0, want_acc=True, **args)
        y = torch.empty((M, N), dtype=torch.float16, device=DEV)
        for rep in range(2):
            y.zero_()
            out, acc = fq.gemv_w6a8_noalloc(packed, N, K, 0, want_acc=True, out=y, **args)
            torch.cuda.synchronize()
            assert torch.equal(out, y_ws), (M, rep)
            assert torch.equal(acc, acc_ws), (M, rep)
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), ref["acc"])
        got = y.cpu().numpy().view(np.uint16).astype(np.int32)
        want = ref["y"].view(np.uint16).astype(np.int32)
        order = lambda b: np.where(b & 0x8000, -(b & 0x7fff), b)
        assert np.abs(order(got) - order(want)).max() <= 1


def test_noalloc_refuses_what_does_not_fit():
    M, K, N = 1024, 8192, 8192
    packed = torch.zeros(fq.packed_bytes(N, K, 0), dtype=torch.uint8, device=DEV)
    xq = torch.zeros((M, K), dtype=torch.int8, device=DEV)
    sx = torch.ones((M,), dtype=torch.float16, device=DEV)
    with pytest.raises(fq.FlexQError, match="workspace"):
        fq.gemv_w6a8_noalloc(packed, N, K, 0, xq=xq, sx=sx)
