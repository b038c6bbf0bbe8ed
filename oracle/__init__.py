"""CPU oracle for the FlexQ W6A6 / W6A8 linear layer -- TEST INFRASTRUCTURE.

Thin ctypes access to ``flexq_oracle.c`` (plain C, fp64 / int64).  Only tests,
the smoke check and the benchmark's cpu_baseline leg import this package; the
GPU library never does.  Every function takes and returns numpy arrays; fp16
values travel as ``numpy.float16``.

Paper passages: Section 2.1 (symmetric quantization), Section 4.1.1 (groups of
128), Section 4.2 Eq. 3-5 (bit-plane product), Eq. 7 and Section 4.3.4 (fused
dequantization with fp16 scales).
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.flexq_oracle_f16_to_f64.restype = ctypes.c_double
        lib.flexq_oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
        lib.flexq_oracle_f64_to_f16.restype = ctypes.c_uint16
        lib.flexq_oracle_f64_to_f16.argtypes = [ctypes.c_double]
        lib.flexq_oracle_quantize.restype = None
        lib.flexq_oracle_quantize.argtypes = [vp, i64, i64, i64, ctypes.c_int, vp, vp]
        lib.flexq_oracle_matmul.restype = i64
        lib.flexq_oracle_matmul.argtypes = [vp, vp, i64, i64, i64, i64, vp]
        lib.flexq_oracle_bitplane_matmul.restype = None
        lib.flexq_oracle_bitplane_matmul.argtypes = [vp, vp, i64, i64, i64, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, vp]
        lib.flexq_oracle_dequant.restype = None
        lib.flexq_oracle_dequant.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        lib.flexq_oracle_dequant_xgroup.restype = None
        lib.flexq_oracle_dequant_xgroup.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        lib.flexq_oracle_pack6_dense.restype = None
        lib.flexq_oracle_pack6_dense.argtypes = [vp, i64, vp]
        lib.flexq_oracle_unpack6_dense.restype = None
        lib.flexq_oracle_unpack6_dense.argtypes = [vp, i64, vp]
        lib.flexq_oracle_rmsnorm.restype = None
        lib.flexq_oracle_rmsnorm.argtypes = [vp, vp, i64, i64, ctypes.c_double, vp]
        lib.flexq_oracle_swiglu.restype = None
        lib.flexq_oracle_swiglu.argtypes = [vp, i64, i64, vp]
        lib.flexq_oracle_num_threads.restype = ctypes.c_int
        lib.flexq_oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    return int(_load().flexq_oracle_num_threads())


def f64_to_f16(x):
    """Direct round-half-even conversion of fp64 values to fp16."""
    lib = _load()
    x = np.asarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = lib.flexq_oracle_f64_to_f16(float(flat_in[i]))
    return out.view(np.float16)


def f16_to_f64(h):
    lib = _load()
    h = np.asarray(h, dtype=np.float16)
    bits = h.view(np.uint16).reshape(-1)
    out = np.empty(bits.size, dtype=np.float64)
    for i in range(bits.size):
        out[i] = lib.flexq_oracle_f16_to_f64(int(bits[i]))
    return out.reshape(h.shape)


def quantize(v, bits, group=0):
    """Symmetric quantization of each row of ``v`` (fp32, or fp16 widened exactly).

    ``group`` = 0 gives one scale per row, otherwise one per ``group`` consecutive
    elements.  Returns (codes int8 [rows, L], scales float16 [rows] or
    [rows, L // group]).
    """
    lib = _load()
    v = np.ascontiguousarray(np.asarray(v), dtype=np.float32)
    assert v.ndim == 2 and bits in (6, 8)
    rows, L = v.shape
    G = L if group == 0 else group
    assert L % G == 0
    q = np.empty((rows, L), dtype=np.int8)
    s = np.empty((rows, L // G), dtype=np.uint16)
    lib.flexq_oracle_quantize(_p(v), rows, L, G, bits, _p(q), _p(s))
    s = s.view(np.float16)
    return q, (s.reshape(rows) if group == 0 else s)


def matmul(xq, wq, group=0):
    """Exact integer product xq [M,K] . wq[N,K]^T -> int64 [M,N] (group = 0) or
    per-group partial products [M,N,K//group].  Raises if a total leaves int32."""
    lib = _load()
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    G = K if group == 0 else group
    assert K % G == 0
    acc = np.empty((M, N, K // G), dtype=np.int64)
    bad = lib.flexq_oracle_matmul(_p(xq), _p(wq), M, N, K, G, _p(acc))
    if bad:
        raise OverflowError(f"{bad} accumulators do not fit int32")
    return acc.reshape(M, N) if group == 0 else acc


def bitplane_matmul(xq, wq, p, q, signed=True):
    """Eq. 4-5: sum over the p*q pairs of 1-bit planes, weighted by 2^(s+t)."""
    lib = _load()
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = xq.shape
    N, _ = wq.shape
    acc = np.empty((M, N), dtype=np.int64)
    lib.flexq_oracle_bitplane_matmul(_p(xq), _p(wq), M, N, K, p, q, int(bool(signed)), _p(acc))
    return acc


def dequant(acc, sx, sw):
    """fp16( sx[m] * sum_g sw[n,g] * acc[m,n,g] ) in fp64; acc [M,N] or [M,N,G]."""
    lib = _load()
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    if acc.ndim == 2:
        acc = acc[:, :, None]
    M, N, ng = acc.shape
    sx = np.ascontiguousarray(sx, dtype=np.float16).reshape(M)
    sw = np.ascontiguousarray(sw, dtype=np.float16).reshape(N, ng)
    y = np.empty((M, N), dtype=np.uint16)
    lib.flexq_oracle_dequant(_p(np.ascontiguousarray(acc)), M, N, ng, _p(sx), _p(sw), _p(y))
    return y.view(np.float16)


def dequant_xgroup(acc, sx, sw):
    """Eq. 7 with a scale per group on both operands: sx [M,G], sw [N,G]."""
    lib = _load()
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    M, N, ng = acc.shape
    sx = np.ascontiguousarray(sx, dtype=np.float16).reshape(M, ng)
    sw = np.ascontiguousarray(sw, dtype=np.float16).reshape(N, ng)
    y = np.empty((M, N), dtype=np.uint16)
    lib.flexq_oracle_dequant_xgroup(_p(acc), M, N, ng, _p(sx), _p(sw), _p(y))
    return y.view(np.float16)


def linear(x_fp16, w_fp32, act_bits, group=0):
    """The whole path on real-valued inputs: quantize weights (6 bits, per
    channel or per ``group``), quantize activations per token to ``act_bits``,
    integer product, dequantize.  Returns a dict of every intermediate."""
    wq, sw = quantize(w_fp32, 6, group)
    xq, sx = quantize(np.asarray(x_fp16, dtype=np.float16).astype(np.float32), act_bits, 0)
    acc = matmul(xq, wq, group)
    y = dequant(acc, sx, sw)
    total = acc if group == 0 else acc.sum(axis=2)
    return {"wq": wq, "sw": sw, "xq": xq, "sx": sx, "acc": total, "acc_g": acc, "y": y}


def rmsnorm(x_fp16, gamma_fp16, eps):
    """fp16( x / sqrt(mean(x^2) + eps) * gamma ) per row, evaluated in fp64."""
    lib = _load()
    x = np.ascontiguousarray(x_fp16, dtype=np.float16)
    g = np.ascontiguousarray(gamma_fp16, dtype=np.float16)
    M, K = x.shape
    assert g.shape == (K,)
    h = np.empty((M, K), dtype=np.uint16)
    lib.flexq_oracle_rmsnorm(_p(x), _p(g), M, K, float(eps), _p(h))
    return h.view(np.float16)


def swiglu(gate_up_fp16):
    """fp16( silu(gate) * up ) for the fused [M, 2F] gate|up layout, evaluated in fp64."""
    lib = _load()
    gu = np.ascontiguousarray(gate_up_fp16, dtype=np.float16)
    M, F2 = gu.shape
    assert F2 % 2 == 0
    h = np.empty((M, F2 // 2), dtype=np.uint16)
    lib.flexq_oracle_swiglu(_p(gu), M, F2 // 2, _p(h))
    return h.view(np.float16)


def pack6_dense(wq):
    lib = _load()
    wq = np.ascontiguousarray(wq, dtype=np.int8).reshape(-1)
    assert wq.size % 4 == 0
    out = np.empty(wq.size * 6 // 8, dtype=np.uint8)
    lib.flexq_oracle_pack6_dense(_p(wq), wq.size, _p(out))
    return out


def unpack6_dense(packed, count):
    lib = _load()
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.empty(count, dtype=np.int8)
    lib.flexq_oracle_unpack6_dense(_p(packed), count, _p(out))
    return out
