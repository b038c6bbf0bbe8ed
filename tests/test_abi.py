"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before any GPU call."""
import ctypes
import os
import re

import pytest

import paper_2508_04405_amd as fq
from paper_2508_04405_amd import dev

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P16 = ctypes.c_void_p(0x1000)          # a non-null, 256-byte aligned fake pointer
ODD = ctypes.c_void_p(0x1008)          # 8-byte aligned only


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flexq_[a-z0-9_]+)\s*\(", text)))


def _exported(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], check=True, capture_output=True, text=True)
    return sorted(line.split()[-1] for line in out.stdout.splitlines() if " T " in line)


def test_every_declared_symbol_is_exported():
    lib = fq.load()
    names = _declared("flexq.h")
    assert {"flexq_pack_w6", "flexq_quant_act", "flexq_gemm_w6a6", "flexq_gemm_w6a8",
            "flexq_gemv_w6a8", "flexq_gemv_w6a8_noalloc"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    dlib = dev.load()
    for n in names + _declared("flexq_dev.h"):
        assert hasattr(dlib, n), n


def test_the_product_library_exports_the_header_and_nothing_else():
    """No tuning hook, probe or other development entry point in libflexq.so: its exported
    functions are exactly the ones include/flexq.h declares."""
    fq.load()
    from paper_2508_04405_amd import binding
    assert _exported(binding.LIB_PATH) == _declared("flexq.h")
    dev.load()
    assert _exported(dev.LIB_PATH) == sorted(set(_declared("flexq.h") + _declared("flexq_dev.h")))


def test_sizes():
    lib = fq.load()
    assert lib.flexq_layout_version() >= 1
    # exactly 0.75 bytes per weight, then the fp16 scales, rounded to 256
    assert lib.flexq_packed_bytes(128, 256, 0) == 128 * 256 * 6 // 8 + 256
    assert lib.flexq_packed_bytes(8192, 8192, 0) == 8192 * 8192 * 6 // 8 + 2 * 8192
    assert lib.flexq_packed_bytes(5120, 5120, 128) == 5120 * 5120 * 6 // 8 + 2 * 5120 * 40
    assert lib.flexq_packed_bytes(100, 256, 0) == 0
    assert lib.flexq_packed_bytes(128, 200, 0) == 0
    assert lib.flexq_packed_bytes(128, 256, 64) == 0
    assert lib.flexq_workspace_bytes(1, 8192, 8192) >= 16384 + 8192
    assert lib.flexq_workspace_bytes(0, 8192, 8192) == 0


def test_workspace_covers_the_partial_sums():
    """Host logic only: the workspace holds the counters, the quantized activations of the
    fused prologue, and the largest partial-sum area any kernel the dispatch may pick needs;
    for more than 128 tokens that includes 128 MiB for the tiles of a partial last round
    of 256, and nothing of the kind when the 256x256 tiles come in whole rounds."""
    lib = fq.load()
    fixed = lambda M, K: 16384 + -(-M * K // 256) * 256 + -(-M * 2 // 256) * 256
    cut = 2 * 256 * 256 * 256 * 4
    # 4096 x 8192 outputs = 512 tiles, 4096 x 57344 = 3584: whole rounds, nothing to cut,
    # and no K splits either
    assert lib.flexq_workspace_bytes(4096, 8192, 8192) == fixed(4096, 8192)
    assert lib.flexq_workspace_bytes(4096, 57344, 8192) == fixed(4096, 8192)
    # 4096 x 10240 = 640 tiles, 1024 x 8192 = 128: a partial round
    assert lib.flexq_workspace_bytes(4096, 10240, 8192) == fixed(4096, 8192) + cut
    assert lib.flexq_workspace_bytes(1024, 8192, 28672) == fixed(1024, 28672) + cut
    # a lone 256x256 tile of two 128-k stages can be cut in two at most: four slots
    assert lib.flexq_workspace_bytes(200, 256, 256) == fixed(200, 256) + 4 * 256 * 256 * 4
    # the answer depends on the shape alone (nothing a caller did before changes it)
    assert lib.flexq_workspace_bytes(1024, 8192, 28672) == dev.load().flexq_workspace_bytes(1024, 8192, 28672)
    # up to 128 tokens only the K splits of the streaming and 128x128 kernels count, and,
    # from 65 tokens, the pieces of 128x256 tiles cut along K (128 KiB each): 40 tiles in
    # four pieces on the 10240-wide layer, nothing of the kind on the 57344-wide one (224
    # tiles fill the chip uncut) or with rows too short to cut (16 stages)
    small = lib.flexq_workspace_bytes(128, 8192, 8192)
    assert fixed(128, 8192) < small < fixed(128, 8192) + 64 * 128 * 8192 * 4
    assert lib.flexq_workspace_bytes(128, 10240, 8192) == fixed(128, 8192) + 40 * 4 * 128 * 256 * 4
    assert lib.flexq_workspace_bytes(100, 57344, 8192) < fixed(100, 8192) + 16 * 128 * 256 * 4
    assert lib.flexq_workspace_bytes(128, 2048, 2048) < fixed(128, 2048) + 16 * 128 * 256 * 4
    # monotone enough for a caller that sizes one workspace for its largest batch
    assert lib.flexq_workspace_bytes(1, 8192, 8192) <= small


@pytest.mark.parametrize("fn", ["flexq_gemm_w6a6", "flexq_gemm_w6a8", "flexq_gemv_w6a6",
                                "flexq_gemv_w6a8"])
def test_linear_argument_errors(fn):
    lib = fq.load()
    f = getattr(lib, fn)
    big = 1 << 30
    ok = dict(packed=P16, group=0, xq=P16, sx=P16, x=None, M=4, N=128, K=256, y=P16, acc=None,
              ws=P16, wsb=big)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["packed"], a["group"], a["xq"], a["sx"], a["x"], a["M"], a["N"], a["K"], a["y"],
                 a["acc"], a["ws"], a["wsb"], None)

    assert call(packed=None) == -1
    assert call(y=None) == -1
    assert call(xq=None) == -1
    assert call(M=0) == -1
    assert call(group=64) == -1
    assert call(group=128, acc=P16) == -1
    assert call(N=100) == -2
    assert call(K=200) == -2
    assert call(K=65536 + 128) == -2
    assert call(packed=ODD) == -3
    assert call(y=ODD) == -3
    assert call(xq=ODD) == -3
    assert call(ws=None) == -5
    assert call(wsb=16) == -5
    assert call(ws=ODD) == -3


def test_other_entry_points_argument_errors():
    lib = fq.load()
    assert lib.flexq_quant_act(None, 1, 128, 8, P16, P16, None) == -1
    assert lib.flexq_quant_act(P16, 1, 128, 7, P16, P16, None) == -1
    assert lib.flexq_quant_act(P16, 1, 100, 8, P16, P16, None) == -2
    assert lib.flexq_quant_act(ODD, 1, 128, 8, P16, P16, None) == -3
    qg, lg = lib.flexq_quant_act_g128, lib.flexq_linear_g128
    assert qg(None, 1, 128, 8, P16, P16, 1, None) == -1
    assert qg(P16, 4, 128, 8, P16, P16, 3, None) == -1          # stride shorter than M
    assert qg(P16, 1, 128, 7, P16, P16, 1, None) == -1
    assert qg(P16, 1, 192, 8, P16, P16, 1, None) == -2
    assert qg(ODD, 1, 128, 8, P16, P16, 1, None) == -3
    big = 1 << 26
    assert lg(P16, P16, None, 4, 4, 128, 256, P16, P16, big, None) == -1
    assert lg(P16, None, P16, 4, 4, 128, 256, P16, P16, big, None) == -1
    assert lg(P16, P16, P16, 3, 4, 128, 256, P16, P16, big, None) == -1   # stride shorter than M
    assert lg(P16, P16, P16, 4, 4, 100, 256, P16, P16, big, None) == -2
    assert lg(P16, P16, P16, 4, 4, 128, 256, ODD, P16, big, None) == -3
    assert lg(P16, P16, P16, 4, 4, 128, 256, P16, None, big, None) == -5
    rn, sg = lib.flexq_rmsnorm_quant, lib.flexq_swiglu_quant
    rn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_int, ctypes.c_int,
                   ctypes.c_int] + [ctypes.c_void_p] * 4
    sg.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 3 + [ctypes.c_void_p] * 4
    assert rn(P16, None, 1e-5, 1, 128, 8, P16, P16, None, None) == -1
    assert rn(P16, P16, 0.0, 1, 128, 8, P16, P16, None, None) == -1
    assert rn(P16, P16, 1e-5, 1, 128, 5, P16, P16, None, None) == -1
    assert rn(P16, P16, 1e-5, 1, 192, 8, P16, P16, None, None) == -2
    assert rn(P16, P16, 1e-5, 1, 128, 8, P16, P16, ODD, None) == -3
    assert sg(None, 1, 128, 8, P16, P16, None, None) == -1
    assert sg(P16, 0, 128, 8, P16, P16, None, None) == -1
    assert sg(P16, 1, 65536 + 128, 8, P16, P16, None, None) == -2
    assert sg(ODD, 1, 128, 8, P16, P16, None, None) == -3
    assert lib.flexq_pack_w6(P16, P16, 96, 256, 0, None, None) == -1
    assert lib.flexq_pack_w6(P16, P16, 100, 256, 0, P16, None) == -2
    assert lib.flexq_pack_w6(P16, P16, 96, 256, 0, ODD, None) == -3
    assert lib.flexq_quant_w6(None, 96, 256, 0, P16, P16, None) == -1
    assert lib.flexq_quant_w6(P16, 96, 256, 32, P16, P16, None) == -1
    assert lib.flexq_unpack_w6(P16, 96, 300, 0, P16, P16, None) == -2
    assert lib.flexq_workspace_init(None, 1 << 20, None) == -1
    assert lib.flexq_workspace_init(P16, 16, None) == -5
    assert b"shape" in lib.flexq_status_string(-2)


def test_activation_tiles_sizes_and_argument_errors():
    """Activations in tile order: 3072 bytes (6-bit, packed) or 4096 bytes (8-bit) per tile of
    32 tokens x 128 k, whole token blocks; bad arguments are refused on the host."""
    lib = fq.load()
    size = lib.flexq_act_tiles_bytes
    assert size(6, 1, 128) == 3072 and size(8, 1, 128) == 4096
    assert size(6, 32, 8192) == 32 * 8192 * 6 // 8           # exactly 0.75 byte per value
    assert size(6, 33, 8192) == 2 * 32 * 8192 * 6 // 8
    assert size(8, 70, 28672) == 3 * 32 * 28672
    assert size(7, 1, 128) == 0 and size(6, 0, 128) == 0 and size(6, 1, 100) == 0 and size(6, 1, 65536 + 128) == 0
    # the prologue's area of the workspace holds one block of tiles for fewer than 32 tokens
    fixed = lambda M, K: 16384 + -(-max(M, 32) * K // 256) * 256 + 256
    assert lib.flexq_workspace_bytes(1, 57344, 8192) == fixed(1, 8192)        # 1792 row blocks: no K split
    assert lib.flexq_workspace_bytes(20, 57344, 8192) == fixed(20, 8192)
    qt, ut, gt = lib.flexq_quant_act_tiles, lib.flexq_untile_act, lib.flexq_gemv_tiles
    assert qt(None, 1, 128, 6, P16, P16, None) == -1
    assert qt(P16, 1, 128, 6, None, P16, None) == -1
    assert qt(P16, 0, 128, 6, P16, P16, None) == -1
    assert qt(P16, 1, 128, 7, P16, P16, None) == -1
    assert qt(P16, 1, 192, 6, P16, P16, None) == -2
    assert qt(P16, 1, 128, 6, ODD, P16, None) == -3
    assert ut(None, 1, 128, 6, P16, None) == -1
    assert ut(P16, 1, 128, 5, P16, None) == -1
    assert ut(P16, 1, 100, 6, P16, None) == -2
    assert ut(P16, 1, 128, 6, ODD, None) == -3
    big = 1 << 30
    ok = dict(bits=6, packed=P16, group=0, xt=P16, sx=P16, M=20, N=128, K=256, y=P16, acc=None, ws=P16, wsb=big)

    def call(**kw):
        a = dict(ok, **kw)
        return gt(a["bits"], a["packed"], a["group"], a["xt"], a["sx"], a["M"], a["N"], a["K"], a["y"], a["acc"],
                  a["ws"], a["wsb"], None)

    assert call(bits=4) == -1
    assert call(M=33) == -1                                  # one block of 32 tokens at most
    assert call(M=0) == -1
    assert call(xt=None) == -1
    assert call(sx=None) == -1
    assert call(group=128, acc=P16) == -1
    assert call(N=100) == -2
    assert call(xt=ODD) == -3
    assert call(ws=None) == -5
    assert call(wsb=1024) == -5
    # the development library refuses an unknown choice for the tile order
    t = dev.Tuning(tiles=3)
    got = ctypes.c_int(0)
    assert dev.load().flexq_dev_linear(ctypes.byref(t), 6, P16, 0, P16, P16, None, None, 0, 4, 128, 256, P16, None,
                                       P16, big, None, ctypes.byref(got)) == -1


def test_noalloc_entry_point_argument_errors():
    """The entry point without a workspace checks like flexq_gemv_w6a8, before it touches
    the GPU, and refuses shapes whose workspace would not fit its fixed array."""
    lib = fq.load()
    f = lib.flexq_gemv_w6a8_noalloc
    ok = dict(packed=P16, group=0, xq=P16, sx=P16, x=None, M=4, N=128, K=256, y=P16, acc=None)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["packed"], a["group"], a["xq"], a["sx"], a["x"], a["M"], a["N"], a["K"], a["y"],
                 a["acc"], None)

    assert call(packed=None) == -1
    assert call(y=None) == -1
    assert call(xq=None) == -1
    assert call(M=0) == -1
    assert call(group=64) == -1
    assert call(N=100) == -2
    assert call(K=200) == -2
    assert call(y=ODD) == -3
    limit = 16 << 20
    assert lib.flexq_workspace_bytes(64, 8192, 28672) <= limit      # every 70B layer at 64 tokens
    assert lib.flexq_workspace_bytes(64, 57344, 8192) <= limit
    assert lib.flexq_workspace_bytes(1024, 8192, 8192) > limit
    assert call(M=1024, N=8192, K=8192) == -5


def test_layer_runner_argument_errors():
    """flexq_layer_linears checks every requested stage's arguments on the host first."""
    from paper_2508_04405_amd.binding import _Layer, _LayerIO
    lib = fq.load()
    p = 0x1000

    def layer(**kw):
        a = dict(H=256, F=512, QKV=768, group=0, w_qkv=p, w_o=p, w_gate_up=p, w_down=p, gamma_attn=p,
                 gamma_ffn=p, eps=1e-5, bits_qkv=6, bits_o=6, bits_gate_up=6, bits_down=8)
        a.update(kw)
        return _Layer(**a)

    def io(**kw):
        a = dict(x=p, qkv=p, attn=p, o=p, x_ffn=p, gate_up=p, down=p)
        a.update(kw)
        return _LayerIO(**a)

    def call(L, M=4, buffers=None, first=0, last=3, ws=P16, wsb=1 << 30):
        return lib.flexq_layer_linears(ctypes.byref(L), M, ctypes.byref(buffers or io()), first, last, ws, wsb,
                                       None)

    need = lib.flexq_layer_workspace_bytes(ctypes.byref(layer()), 4)
    # the widest GEMM workspace, then the quantized input of a stage: codes [M, max(H, F)] (room
    # for one block of 32-token tiles when there are fewer tokens), scales [M]
    assert need == max(lib.flexq_workspace_bytes(4, n, k)
                       for n, k in ((768, 256), (256, 256), (1024, 256), (256, 512))) + 32 * 512 + 256
    assert lib.flexq_layer_workspace_bytes(ctypes.byref(layer()), 40) == max(
        lib.flexq_workspace_bytes(40, n, k) for n, k in ((768, 256), (256, 256), (1024, 256), (256, 512))) + 40 * 512 + 256
    assert lib.flexq_layer_workspace_bytes(ctypes.byref(layer(H=200)), 4) == 0
    assert call(layer(), M=0) == -1
    assert call(layer(), first=2, last=1) == -1
    assert call(layer(), last=4) == -1
    assert call(layer(bits_down=7)) == -1
    assert call(layer(group=64)) == -1
    assert call(layer(eps=0.0)) == -1
    assert call(layer(H=200)) == -2
    assert call(layer(w_down=None)) == -1
    assert call(layer(), buffers=io(attn=None)) == -1
    assert call(layer(), buffers=io(attn=None), first=0, last=0, wsb=16) == -5   # attn not needed for stage 0
    assert call(layer(), buffers=io(x=0x1008)) == -3
    assert call(layer(), buffers=io(h_swiglu=0x1008)) == -3
    assert call(layer(), ws=None) == -5
    assert call(layer(), wsb=need - 1) == -5
    assert call(layer(), ws=ODD) == -3


def test_dev_entry_points_argument_errors():
    d = dev.load()
    assert d.flexq_dev_probe_hbm_read(None, 4096, P16, None) == -1
    assert d.flexq_dev_probe_hbm_read(ODD, 4096, P16, None) == -3
    assert d.flexq_dev_probe_mfma_i8(P16, P16, 0, 1, P16, None) == -1
    mix = d.flexq_dev_probe_mfma_mix
    assert mix(None, P16, 3, 4, 100, 256, 8, P16, None) == -1
    assert mix(P16, P16, 3, 4, 101, 256, 8, P16, None) == -1       # an odd number of steps
    assert mix(P16, P16, 3, 4, 100, 256, 6, P16, None) == -1       # four or eight wavefronts
    assert mix(P16, P16, 5, 4, 100, 256, 8, P16, None) == -1       # a combination that is not built
    assert mix(ODD, P16, 3, 4, 100, 256, 8, P16, None) == -3
    big = 1 << 30

    def call(tuning, bits=8, **kw):
        a = dict(packed=P16, group=0, xq=P16, sx=P16, x=None, sxg=None, stride=0, M=4, N=128, K=256,
                 y=P16, acc=None, ws=P16, wsb=big)
        a.update(kw)
        t = dev.Tuning(**tuning) if tuning is not None else None
        return d.flexq_dev_linear(t, bits, a["packed"], a["group"], a["xq"], a["sx"], a["x"], a["sxg"],
                                  a["stride"], a["M"], a["N"], a["K"], a["y"], a["acc"], a["ws"],
                                  a["wsb"], None, None)

    zero = dict(kernel=0, split_k=0, waves=0, gemm_cfg=0, ablate=0, fuse=0)
    for bad in (dict(kernel=3), dict(waves=5), dict(split_k=65), dict(gemm_cfg=33), dict(ablate=5),
                dict(ablate=-1), dict(kernel=-1), dict(fuse=3), dict(tiles=3), dict(spin=-2),
                dict(spin=(1 << 20) + 1)):
        assert call(dict(zero, **bad)) == -1, bad
    assert call(zero, bits=7) == -1
    assert call(zero, y=None) == -1              # the same checks as the product call, host side
    assert call(None, N=100) == -2
    assert call(zero, ws=None) == -5
