"""ctypes binding of libflexq.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers and the current HIP stream through the C ABI declared in
include/flexq.h, and returns torch tensors.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflexq.so")
_lib = None


class FlexQError(RuntimeError):
    pass


class _Layer(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int), ("F", ctypes.c_int), ("QKV", ctypes.c_int), ("group", ctypes.c_int),
                ("w_qkv", ctypes.c_void_p), ("w_o", ctypes.c_void_p), ("w_gate_up", ctypes.c_void_p),
                ("w_down", ctypes.c_void_p), ("gamma_attn", ctypes.c_void_p), ("gamma_ffn", ctypes.c_void_p),
                ("eps", ctypes.c_float), ("bits_qkv", ctypes.c_int), ("bits_o", ctypes.c_int),
                ("bits_gate_up", ctypes.c_int), ("bits_down", ctypes.c_int)]


class _LayerIO(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("x", "qkv", "attn", "o", "x_ffn", "gate_up", "down",
                                               "h_attn_norm", "h_ffn_norm", "h_swiglu")]


def load():
    """Load libflexq.so, building it first if it is missing or older than its sources."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if _build.sources_newer_than(LIB_PATH):
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_size, vp = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
    lib.flexq_status_string.restype = ctypes.c_char_p
    lib.flexq_status_string.argtypes = [c_int]
    lib.flexq_layout_version.restype = c_int
    lib.flexq_layout_version.argtypes = []
    lib.flexq_packed_bytes.restype = c_size
    lib.flexq_packed_bytes.argtypes = [c_int, c_int, c_int]
    lib.flexq_quant_w6.restype = c_int
    lib.flexq_quant_w6.argtypes = [vp, c_int, c_int, c_int, vp, vp, vp]
    lib.flexq_pack_w6.restype = c_int
    lib.flexq_pack_w6.argtypes = [vp, vp, c_int, c_int, c_int, vp, vp]
    lib.flexq_unpack_w6.restype = c_int
    lib.flexq_unpack_w6.argtypes = [vp, c_int, c_int, c_int, vp, vp, vp]
    lib.flexq_quant_act.restype = c_int
    lib.flexq_quant_act.argtypes = [vp, c_int, c_int, c_int, vp, vp, vp]
    lib.flexq_act_tiles_bytes.restype = ctypes.c_size_t
    lib.flexq_act_tiles_bytes.argtypes = [c_int, c_int, c_int]
    lib.flexq_quant_act_tiles.restype = c_int
    lib.flexq_quant_act_tiles.argtypes = [vp, c_int, c_int, c_int, vp, vp, vp]
    lib.flexq_untile_act.restype = c_int
    lib.flexq_untile_act.argtypes = [vp, c_int, c_int, c_int, vp, vp]
    lib.flexq_gemv_tiles.restype = c_int
    lib.flexq_gemv_tiles.argtypes = [c_int, vp, c_int, vp, vp, c_int, c_int, c_int, vp, vp, vp, ctypes.c_size_t, vp]
    lib.flexq_quant_act_g128.restype = c_int
    lib.flexq_quant_act_g128.argtypes = [vp, c_int, c_int, c_int, vp, vp, c_int, vp]
    lib.flexq_linear_g128.restype = c_int
    lib.flexq_linear_g128.argtypes = [vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp, ctypes.c_size_t, vp]
    lib.flexq_rmsnorm_quant.restype = c_int
    lib.flexq_rmsnorm_quant.argtypes = [vp, vp, ctypes.c_float, c_int, c_int, c_int, vp, vp, vp, vp]
    lib.flexq_swiglu_quant.restype = c_int
    lib.flexq_swiglu_quant.argtypes = [vp, c_int, c_int, c_int, vp, vp, vp, vp]
    lib.flexq_workspace_bytes.restype = c_size
    lib.flexq_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.flexq_workspace_init.restype = c_int
    lib.flexq_workspace_init.argtypes = [vp, c_size, vp]
    for name in ("flexq_gemm_w6a6", "flexq_gemm_w6a8", "flexq_gemv_w6a6", "flexq_gemv_w6a8"):
        fn = getattr(lib, name)
        fn.restype = c_int
        fn.argtypes = [vp, c_int, vp, vp, vp, c_int, c_int, c_int, vp, vp, vp, c_size, vp]
    lib.flexq_layer_workspace_bytes.restype = c_size
    lib.flexq_layer_workspace_bytes.argtypes = [ctypes.POINTER(_Layer), c_int]
    lib.flexq_layer_linears.restype = c_int
    lib.flexq_layer_linears.argtypes = [ctypes.POINTER(_Layer), c_int, ctypes.POINTER(_LayerIO), c_int, c_int,
                                        vp, c_size, vp]
    lib.flexq_gemv_w6a8_noalloc.restype = c_int
    lib.flexq_gemv_w6a8_noalloc.argtypes = [vp, c_int, vp, vp, vp, c_int, c_int, c_int, vp, vp, vp]
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise FlexQError(f"flexq: {load().flexq_status_string(status).decode()} ({status})")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(t, dtype):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype)
    return t


def layout_version():
    return load().flexq_layout_version()


def packed_bytes(N, K, group=0):
    return load().flexq_packed_bytes(N, K, group)


def quant_w6(w, group=0):
    """fp32 W[N,K] -> (int8 codes [N,K], fp16 scales [N] or [N,K/128])."""
    lib = load()
    _dev(w, torch.float32)
    N, K = w.shape
    wq = torch.empty((N, K), dtype=torch.int8, device=w.device)
    sw = torch.empty((N,) if group == 0 else (N, K // 128), dtype=torch.float16, device=w.device)
    _check(lib.flexq_quant_w6(_ptr(w), N, K, group, _ptr(wq), _ptr(sw), _stream()))
    return wq, sw


def pack_w6(wq, sw, group=0):
    """int8 codes [N,K] + fp16 scales -> opaque packed buffer (uint8)."""
    lib = load()
    _dev(wq, torch.int8)
    _dev(sw, torch.float16)
    N, K = wq.shape
    nbytes = lib.flexq_packed_bytes(N, K, group)
    if nbytes == 0:
        _check(lib.flexq_pack_w6(_ptr(wq), _ptr(sw), N, K, group, _ptr(wq), _stream()))
    packed = torch.empty(nbytes, dtype=torch.uint8, device=wq.device)
    _check(lib.flexq_pack_w6(_ptr(wq), _ptr(sw), N, K, group, _ptr(packed), _stream()))
    return packed


def unpack_w6(packed, N, K, group=0):
    lib = load()
    _dev(packed, torch.uint8)
    wq = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    sw = torch.empty((N,) if group == 0 else (N, K // 128), dtype=torch.float16,
                     device=packed.device)
    _check(lib.flexq_unpack_w6(_ptr(packed), N, K, group, _ptr(wq), _ptr(sw), _stream()))
    return wq, sw


def quant_act(x, act_bits, out=None):
    """fp16 X[M,K] -> (int8 codes [M,K], fp16 scales [M]); `out` = (xq, sx) to reuse."""
    lib = load()
    _dev(x, torch.float16)
    M, K = x.shape
    if out is not None:
        xq, sx = _dev(out[0], torch.int8), _dev(out[1], torch.float16)
        assert xq.shape == (M, K) and sx.shape == (M,)
    else:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
        sx = torch.empty((M,), dtype=torch.float16, device=x.device)
    _check(lib.flexq_quant_act(_ptr(x), M, K, act_bits, _ptr(xq), _ptr(sx), _stream()))
    return xq, sx


def quant_act_tiles(x, act_bits, out=None):
    """fp16 X[M,K] -> (activations in tile order, uint8 [flexq_act_tiles_bytes], fp16 scales [M])."""
    lib = load()
    _dev(x, torch.float16)
    M, K = x.shape
    nbytes = lib.flexq_act_tiles_bytes(act_bits, M, K)
    if nbytes == 0:
        raise FlexQError("flexq: invalid shape for activation tiles")
    if out is not None:
        xt, sx = _dev(out[0], torch.uint8), _dev(out[1], torch.float16)
        assert xt.numel() >= nbytes and sx.shape == (M,)
    else:
        xt = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
        sx = torch.empty((M,), dtype=torch.float16, device=x.device)
    _check(lib.flexq_quant_act_tiles(_ptr(x), M, K, act_bits, _ptr(xt), _ptr(sx), _stream()))
    return xt, sx


def untile_act(xt, M, K, act_bits):
    """Activations in tile order -> int8 codes [M,K] row-major."""
    lib = load()
    _dev(xt, torch.uint8)
    xq = torch.empty((M, K), dtype=torch.int8, device=xt.device)
    _check(lib.flexq_untile_act(_ptr(xt), M, K, act_bits, _ptr(xq), _stream()))
    return xq


def gemv_tiles(act_bits, packed, N, K, group, xt, sx, workspace=None, want_acc=False, out=None):
    """The linear layer on activations in tile order (quant_act_tiles), M <= 32."""
    lib = load()
    _dev(packed, torch.uint8)
    _dev(xt, torch.uint8)
    _dev(sx, torch.float16)
    M, dev = sx.shape[0], sx.device
    if workspace is None:
        workspace = make_workspace(M, N, K, dev)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    _check(lib.flexq_gemv_tiles(act_bits, _ptr(packed), group, _ptr(xt), _ptr(sx), M, N, K, _ptr(y), _ptr(acc),
                                _ptr(workspace), workspace.numel(), _stream()))
    return (y, acc) if want_acc else y


def _producer_out(M, L, device, want_h, out):
    if out is not None:
        xq, sx = _dev(out[0], torch.int8), _dev(out[1], torch.float16)
        assert xq.shape == (M, L) and sx.shape == (M,)
    else:
        xq = torch.empty((M, L), dtype=torch.int8, device=device)
        sx = torch.empty((M,), dtype=torch.float16, device=device)
    h = torch.empty((M, L), dtype=torch.float16, device=device) if want_h else None
    return xq, sx, h


def rmsnorm_quant(x, gamma, eps, act_bits, want_h=False, out=None):
    """RMS norm of fp16 X[M,K] with fp16 gamma[K], quantized per token in the same
    kernel -> (xq, sx) or (xq, sx, h) with the fp16 normed values when want_h."""
    lib = load()
    _dev(x, torch.float16)
    _dev(gamma, torch.float16)
    M, K = x.shape
    assert gamma.shape == (K,)
    xq, sx, h = _producer_out(M, K, x.device, want_h, out)
    _check(lib.flexq_rmsnorm_quant(_ptr(x), _ptr(gamma), float(eps), M, K, act_bits, _ptr(xq),
                                   _ptr(sx), _ptr(h) if want_h else None, _stream()))
    return (xq, sx, h) if want_h else (xq, sx)


def swiglu_quant(gate_up, act_bits, want_h=False, out=None):
    """silu(gate) * up of fp16 [M, 2F] (gate columns first), quantized per token in the
    same kernel -> (xq, sx) or (xq, sx, h)."""
    lib = load()
    _dev(gate_up, torch.float16)
    M, F2 = gate_up.shape
    assert F2 % 2 == 0
    F = F2 // 2
    xq, sx, h = _producer_out(M, F, gate_up.device, want_h, out)
    _check(lib.flexq_swiglu_quant(_ptr(gate_up), M, F, act_bits, _ptr(xq), _ptr(sx),
                                  _ptr(h) if want_h else None, _stream()))
    return (xq, sx, h) if want_h else (xq, sx)


def quant_act_g128(x, act_bits):
    """fp16 X[M,K] -> (int8 codes [M,K], fp16 scales [K/128, stride >= M]) with one scale per
    token and group of 128 along K; the scales are group-major, rows padded to a multiple of 64."""
    lib = load()
    _dev(x, torch.float16)
    M, K = x.shape
    xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    stride = (M + 63) // 64 * 64         # even, as the tiled kernel wants; padding stays unwritten
    sxg = torch.zeros((K // 128, stride), dtype=torch.float16, device=x.device)
    _check(lib.flexq_quant_act_g128(_ptr(x), M, K, act_bits, _ptr(xq), _ptr(sxg), stride, _stream()))
    return xq, sxg


def linear_g128(packed, N, K, xq, sxg, workspace=None, out=None):
    """Y[M,N] for group-128 scales on both operands (packed made with group = 128)."""
    lib = load()
    _dev(packed, torch.uint8)
    _dev(xq, torch.int8)
    _dev(sxg, torch.float16)
    M = xq.shape[0]
    assert xq.shape == (M, K) and sxg.shape[0] == K // 128 and sxg.shape[1] >= M
    dev = xq.device
    if workspace is None:
        workspace = make_workspace(M, N, K, dev)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=dev)
    _check(lib.flexq_linear_g128(_ptr(packed), _ptr(xq), _ptr(sxg), sxg.shape[1], M, N, K, _ptr(y),
                                 _ptr(workspace), workspace.numel(), _stream()))
    return y


def workspace_bytes(M, N, K):
    return load().flexq_workspace_bytes(M, N, K)


def make_workspace(M, N, K, device="cuda", extra=0):
    """Allocate (with torch) and zero-initialise a workspace for (M,N,K)."""
    lib = load()
    nbytes = lib.flexq_workspace_bytes(M, N, K) + extra
    if nbytes == extra:
        raise FlexQError("flexq: invalid shape for workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    _check(lib.flexq_workspace_init(_ptr(ws), nbytes, _stream()))
    return ws


def _linear(name, packed, N, K, group, xq, sx, x_fp16, workspace, want_acc, out):
    lib = load()
    _dev(packed, torch.uint8)
    if x_fp16 is not None:
        _dev(x_fp16, torch.float16)
        M = x_fp16.shape[0]
        dev = x_fp16.device
    else:
        _dev(xq, torch.int8)
        _dev(sx, torch.float16)
        M = xq.shape[0]
        dev = xq.device
    if workspace is None:
        workspace = make_workspace(M, N, K, dev)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    _check(getattr(lib, name)(_ptr(packed), group, _ptr(xq), _ptr(sx), _ptr(x_fp16), M, N, K,
                              _ptr(y), _ptr(acc), _ptr(workspace), workspace.numel(), _stream()))
    return (y, acc) if want_acc else y


def gemm_w6a6(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, workspace=None,
              want_acc=False, out=None):
    return _linear("flexq_gemm_w6a6", packed, N, K, group, xq, sx, x_fp16, workspace, want_acc, out)


def gemm_w6a8(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, workspace=None,
              want_acc=False, out=None):
    return _linear("flexq_gemm_w6a8", packed, N, K, group, xq, sx, x_fp16, workspace, want_acc, out)


def gemv_w6a6(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, workspace=None,
              want_acc=False, out=None):
    return _linear("flexq_gemv_w6a6", packed, N, K, group, xq, sx, x_fp16, workspace, want_acc, out)


def gemv_w6a8(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, workspace=None,
              want_acc=False, out=None):
    return _linear("flexq_gemv_w6a8", packed, N, K, group, xq, sx, x_fp16, workspace, want_acc, out)


def gemv_w6a8_noalloc(packed, N, K, group=0, xq=None, sx=None, x_fp16=None, want_acc=False, out=None):
    """flexq_gemv_w6a8 on the library's own fixed scratch array: no workspace argument,
    nothing allocated by the call itself (the outputs here are made by torch unless given)."""
    lib = load()
    _dev(packed, torch.uint8)
    if x_fp16 is not None:
        _dev(x_fp16, torch.float16)
        M, dev = x_fp16.shape[0], x_fp16.device
    else:
        _dev(xq, torch.int8)
        _dev(sx, torch.float16)
        M, dev = xq.shape[0], xq.device
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    _check(lib.flexq_gemv_w6a8_noalloc(_ptr(packed), group, _ptr(xq), _ptr(sx), _ptr(x_fp16), M, N, K,
                                       _ptr(y), _ptr(acc), _stream()))
    return (y, acc) if want_acc else y


class Layer:
    """The packed weights, norm gains and activation widths of one decoder block's linear
    layers (a flexq_layer; keeps the tensors alive)."""

    def __init__(self, H, F, QKV, group, w_qkv, w_o, w_gate_up, w_down, gamma_attn, gamma_ffn,
                 eps=1e-5, bits=(6, 6, 6, 8)):
        for w in (w_qkv, w_o, w_gate_up, w_down):
            _dev(w, torch.uint8)
        for g in (gamma_attn, gamma_ffn):
            _dev(g, torch.float16)
            assert g.shape == (H,)
        self.tensors = (w_qkv, w_o, w_gate_up, w_down, gamma_attn, gamma_ffn)
        self.H, self.F, self.QKV, self.group = H, F, QKV, group
        self.c = _Layer(H, F, QKV, group, w_qkv.data_ptr(), w_o.data_ptr(), w_gate_up.data_ptr(),
                        w_down.data_ptr(), gamma_attn.data_ptr(), gamma_ffn.data_ptr(), float(eps), *bits)

    def workspace_bytes(self, M):
        return load().flexq_layer_workspace_bytes(ctypes.byref(self.c), M)

    def make_workspace(self, M, device="cuda"):
        nbytes = self.workspace_bytes(M)
        if nbytes == 0:
            raise FlexQError("flexq: invalid layer shape for workspace")
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _check(load().flexq_workspace_init(_ptr(ws), nbytes, _stream()))
        return ws


def layer_linears(layer, M, workspace, first_stage=0, last_stage=3, **buffers):
    """flexq_layer_linears: `buffers` are the fp16 tensors of flexq_layer_io by name (x, qkv, attn,
    o, x_ffn, gate_up, down, and the optional h_attn_norm, h_ffn_norm, h_swiglu); only those the
    requested stages touch are needed."""
    shapes = dict(x=layer.H, qkv=layer.QKV, attn=layer.H, o=layer.H, x_ffn=layer.H, gate_up=2 * layer.F,
                  down=layer.H, h_attn_norm=layer.H, h_ffn_norm=layer.H, h_swiglu=layer.F)
    io = _LayerIO()
    for name, t in buffers.items():
        _dev(t, torch.float16)
        assert t.shape == (M, shapes[name]), (name, tuple(t.shape))
        setattr(io, name, t.data_ptr())
    _check(load().flexq_layer_linears(ctypes.byref(layer.c), M, ctypes.byref(io), first_stage, last_stage,
                                      _ptr(workspace), workspace.numel(), _stream()))
