"""ctypes binding of libflexq_dev.so (include/flexq_dev.h): the linear-layer call with
per-call kernel overrides, and the two ceiling probes.  Test and measurement
infrastructure; the product path is `binding`.

`set_dispatch` / `set_ablation` only record, in this module, the overrides that the
calls made through this module pass along with each call; the library itself keeps
no state.  `last_dispatch` is what the last call through this module reported.
"""
import ctypes
import os

import torch

from . import binding
from .binding import _check, _dev, _ptr, _stream, make_workspace

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflexq_dev.so")
_lib = None
_tuning = dict(kernel=0, split_k=0, waves=0, gemm_cfg=0, ablate=0, fuse=0, tiles=0, spin=0)
_last = 0


class Tuning(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("kernel", "split_k", "waves", "gemm_cfg", "ablate", "fuse", "tiles", "spin")]


def load():
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if _build.sources_newer_than(LIB_PATH):
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_size, vp = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
    lib.flexq_dev_linear.restype = c_int
    lib.flexq_dev_linear.argtypes = [ctypes.POINTER(Tuning), c_int, vp, c_int, vp, vp, vp, vp, c_int,
                                     c_int, c_int, c_int, vp, vp, vp, c_size, vp,
                                     ctypes.POINTER(c_int)]
    lib.flexq_dev_probe_hbm_read.restype = c_int
    lib.flexq_dev_probe_hbm_read.argtypes = [vp, c_size, vp, vp]
    lib.flexq_dev_probe_mfma_i8.restype = c_int
    lib.flexq_dev_probe_mfma_i8.argtypes = [vp, vp, c_int, c_int, vp, vp]
    lib.flexq_dev_probe_mfma_mix.restype = c_int
    lib.flexq_dev_probe_mfma_mix.argtypes = [vp, vp, c_int, c_int, c_int, c_int, c_int, vp, vp]
    _lib = lib
    return lib


def set_dispatch(which=0, split_k=0, waves=0, gemm_cfg=0):
    """Overrides for the following calls through this module (0 = the library's choice)."""
    _tuning.update(kernel=which, split_k=split_k, waves=waves, gemm_cfg=gemm_cfg)


def set_ablation(choice=0):
    _tuning.update(ablate=choice)


def set_fuse(choice=0):
    """1: quantize inside the streaming kernel whenever it can; 2: never; 0: the library's choice."""
    _tuning.update(fuse=choice)


def set_tiles(choice=0):
    """1: fp16 activations of up to 32 tokens always go through tile order; 2: never; 0: the
    library's choice."""
    _tuning.update(tiles=choice)


def set_spin(polls=0):
    """Evenly cut tiles (gemm_cfg 13): polls before a piece stops waiting for the others;
    -1: none (every piece gives up at once); 0: the library's choice."""
    _tuning.update(spin=polls)


def last_dispatch():
    """(kernel, splits) of the last call through this module: kernel 1 = streaming, else the
    tile configuration; for the forms that cut their last round the second number is the
    number of pieces."""
    return _last // 1000, _last % 1000


def _linear(act_bits, packed, N, K, group, xq, sx, x_fp16, sxg, workspace, want_acc, out):
    global _last
    lib = load()
    _dev(packed, torch.uint8)
    if x_fp16 is not None:
        _dev(x_fp16, torch.float16)
        M, dev = x_fp16.shape[0], x_fp16.device
    else:
        _dev(xq, torch.int8)
        M, dev = xq.shape[0], xq.device
    if workspace is None:
        workspace = make_workspace(M, N, K, dev)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    t = Tuning(**_tuning)
    got = ctypes.c_int(0)
    status = lib.flexq_dev_linear(ctypes.byref(t), act_bits, _ptr(packed), group, _ptr(xq), _ptr(sx),
                                  _ptr(x_fp16), _ptr(sxg), 0 if sxg is None else sxg.shape[1], M, N, K,
                                  _ptr(y), _ptr(acc), _ptr(workspace), workspace.numel(), _stream(),
                                  ctypes.byref(got))
    _last = got.value
    _check(status)
    return (y, acc) if want_acc else y


def gemm_w6a6(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, workspace=None,
              want_acc=False, out=None):
    return _linear(6, packed, N, K, group, xq, sx, x_fp16, None, workspace, want_acc, out)


def gemm_w6a8(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, workspace=None,
              want_acc=False, out=None):
    return _linear(8, packed, N, K, group, xq, sx, x_fp16, None, workspace, want_acc, out)


gemv_w6a6 = gemm_w6a6      # one dispatch behind both names, as in the product library
gemv_w6a8 = gemm_w6a8


def linear_g128(packed, N, K, xq, sxg, workspace=None, out=None):
    _dev(sxg, torch.float16)
    assert sxg.shape[0] == K // 128 and sxg.shape[1] >= xq.shape[0]
    return _linear(8, packed, N, K, 128, xq, None, None, sxg, workspace, False, out)


def probe_hbm_read(buf, sink):
    """Enqueue the read-only streaming kernel over `buf` (any dtype, contiguous)."""
    _check(load().flexq_dev_probe_hbm_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink),
                                           _stream()))


def probe_mfma_i8(a_operands, b_operands, iters, workgroups, sink):
    """Enqueue the MFMA-only kernel; operands are read from the first 16 KiB of each buffer."""
    assert a_operands.numel() * a_operands.element_size() >= 16384
    assert b_operands.numel() * b_operands.element_size() >= 16384
    _check(load().flexq_dev_probe_mfma_i8(_ptr(a_operands), _ptr(b_operands), iters, workgroups,
                                          _ptr(sink), _stream()))


def probe_mfma_mix(a_operands, b_operands, valu_per_mfma, lds_reads_per_8, iters, workgroups, waves, sink):
    """Enqueue the MFMA kernel with `valu_per_mfma` vector operations after every MFMA and
    `lds_reads_per_8` LDS reads per eight MFMAs; `waves` 4 or 8 per workgroup."""
    assert a_operands.numel() * a_operands.element_size() >= 16384
    assert b_operands.numel() * b_operands.element_size() >= 16384
    _check(load().flexq_dev_probe_mfma_mix(_ptr(a_operands), _ptr(b_operands), valu_per_mfma, lds_reads_per_8,
                                           iters, workgroups, waves, _ptr(sink), _stream()))
