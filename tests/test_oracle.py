"""Pins for the CPU oracle (no GPU): each check compares it with something that
does not go through the oracle's own arithmetic -- numpy library routines,
exact rational arithmetic, brute force, the paper's worked example (Section
4.2, Eq. 3), closed forms and crafted ties."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2508_04405_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ fp16

def test_f16_to_f64_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ours = oracle.f16_to_f64(bits.view(np.float16))
    ref = bits.view(np.float16).astype(np.float64)
    both_nan = np.isnan(ours) & np.isnan(ref)
    assert np.all((ours == ref) | both_nan)
    assert np.all(np.signbit(ours) == np.signbit(ref))


def test_f64_to_f16_matches_numpy_direct_rounding():
    rng = np.random.default_rng(1)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.999, 65520.0, 1e6, -1e6, 2.0**-24,
            2.0**-25, 2.0**-25 * (1 + 1e-12), 2.0**-14, 2.0**-14 * (1 - 2.0**-11),
            2.0**-14 - 2.0**-25, 1.5 * 2.0**-24, 2.5 * 2.0**-24, 0.1, 1 / 3]
    # every tie between neighbouring normal fp16 values in a few binades
    for e in (-14, -3, 0, 5, 15):
        for m in (0, 1, 2, 511, 1022, 1023):
            lo = (1024 + m) * 2.0 ** (e - 10)
            vals += [lo + 2.0 ** (e - 11), lo + 2.0 ** (e - 11) * (1 + 1e-9),
                     lo + 2.0 ** (e - 11) * (1 - 1e-9)]
    vals = np.array(vals)
    rand = np.concatenate([
        rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 5, 4000),
        rng.uniform(-2.0**-13, 2.0**-13, 2000),            # subnormal region
        (rng.integers(0, 2**16, 2000) + 0.5) * 2.0**-20,   # many exact ties
    ])
    x = np.concatenate([vals, -vals, rand])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    ours = oracle.f64_to_f16(x).view(np.uint16)
    assert np.array_equal(ours, ref)


# ------------------------------------------------ bit planes (Eq. 3, 4, 5)

def _read_eq3():
    terms = {}
    with open(os.path.join(GOLDEN, "eq3_partial_products.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            terms[int(parts[0])] = [(int(t[0]), int(t[1])) for t in parts[1:]]
    return terms


def test_eq3_worked_example_every_a_b():
    terms = _read_eq3()
    # the paper's grouping covers each of the 2*4 bit pairs once, at power i+j
    pairs = [(i, j) for p in terms for (i, j) in terms[p]]
    assert sorted(pairs) == [(i, j) for i in range(2) for j in range(4)]
    for power, lst in terms.items():
        assert all(i + j == power for i, j in lst)
    for a in range(4):
        for b in range(16):
            printed = sum((1 << power) * sum(((a >> i) & 1) * ((b >> j) & 1) for i, j in lst)
                          for power, lst in terms.items())
            assert printed == a * b
            w = np.array([[a]], dtype=np.int8)
            x = np.array([[b]], dtype=np.int8)
            assert oracle.bitplane_matmul(x, w, p=2, q=4, signed=False)[0, 0] == a * b
            assert oracle.matmul(x, w)[0, 0] == a * b


@pytest.mark.parametrize("act_bits", [6, 8])
def test_bitplane_identity_signed_and_offset(act_bits):
    rng = np.random.default_rng(act_bits)
    M, N, K = 3, 5, 64
    wq = rng.integers(-32, 32, (N, K)).astype(np.int8)
    lo = -(1 << (act_bits - 1))
    xq = rng.integers(lo, -lo, (M, K)).astype(np.int8)
    wq[0, :4] = [-32, 31, -1, 0]
    xq[0, :4] = [lo, -lo - 1, -1, lo]
    direct = oracle.matmul(xq, wq)
    ref = xq.astype(np.int64) @ wq.astype(np.int64).T          # library routine
    assert np.array_equal(direct, ref)
    # signed planes: the top plane of each operand weighs -2^(bits-1)
    assert np.array_equal(oracle.bitplane_matmul(xq, wq, 6, act_bits, signed=True), ref)
    # unsigned planes on offset values u = v + 2^(bits-1), expanded back
    wu = (wq.astype(np.int16) + 32).astype(np.int8)
    xu_wide = xq.astype(np.int16) - lo
    xu = xu_wide.astype(np.uint8).view(np.int8)
    uu = oracle.bitplane_matmul(xu, wu, 6, act_bits, signed=False)
    # (wu - 32)(xu + lo) = wu*xu + lo*wu - 32*xu - 32*lo, summed over k
    back = (uu + lo * wu.astype(np.int64).sum(1)[None, :]
            - 32 * xu_wide.astype(np.int64).sum(1)[:, None] - 32 * lo * K)
    assert np.array_equal(back, ref)


def test_bitplane_drops_a_plane_if_width_too_small():
    # guards the test above: with p = 5 the signed expansion must NOT match
    wq = np.array([[-32, 31, 17, -5]], dtype=np.int8)
    xq = np.array([[3, -7, 11, 2]], dtype=np.int8)
    ref = xq.astype(np.int64) @ wq.astype(np.int64).T
    assert np.array_equal(oracle.bitplane_matmul(xq, wq, 6, 8, True), ref)
    assert not np.array_equal(oracle.bitplane_matmul(xq, wq, 5, 8, True), ref)


# --------------------------------------------------------- integer product

def test_matmul_brute_force_tiny():
    rng = np.random.default_rng(3)
    M, N, K = 2, 3, 8
    xq = rng.integers(-128, 128, (M, K)).astype(np.int8)
    wq = rng.integers(-32, 32, (N, K)).astype(np.int8)
    acc = oracle.matmul(xq, wq)
    for m in range(M):
        for n in range(N):
            s = 0
            for k in range(K):
                s += int(xq[m, k]) * int(wq[n, k])
            assert acc[m, n] == s


def test_matmul_vs_numpy_and_not_transposed():
    rng = np.random.default_rng(4)
    M, N, K = 7, 96, 384                     # M != N so a transposed result fails
    xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    wq = rng.integers(-32, 32, (N, K)).astype(np.int8)
    ref = xq.astype(np.int64) @ wq.astype(np.int64).T
    assert oracle.matmul(xq, wq).shape == (M, N)
    assert np.array_equal(oracle.matmul(xq, wq), ref)
    g = oracle.matmul(xq, wq, group=128)
    assert g.shape == (M, N, 3)
    for i in range(3):                       # K-concatenation: groups are K slices
        sl = slice(128 * i, 128 * (i + 1))
        assert np.array_equal(g[:, :, i], xq[:, sl].astype(np.int64) @ wq[:, sl].astype(np.int64).T)
    assert np.array_equal(g.sum(2), ref)


def test_matmul_closed_forms():
    K = 1024
    xq = np.full((2, K), 127, dtype=np.int8)
    wq = np.full((4, K), 31, dtype=np.int8)
    assert np.all(oracle.matmul(xq, wq) == 31 * 127 * K)
    wq[:] = -32
    xq[:] = -128
    assert np.all(oracle.matmul(xq, wq) == 32 * 128 * K)
    rng = np.random.default_rng(5)
    xq = rng.integers(-127, 128, (3, K)).astype(np.int8)
    wq = np.zeros((6, K), dtype=np.int8)
    cols = [0, 5, 100, 511, 1000, 1023]
    for n, k in enumerate(cols):
        wq[n, k] = 1                          # one-hot rows pick a column of X
    assert np.array_equal(oracle.matmul(xq, wq), xq[:, cols].astype(np.int64))
    wr = rng.integers(-32, 32, (6, K)).astype(np.int8)
    assert np.array_equal(oracle.matmul((-xq.astype(np.int16)).astype(np.int8), wr),
                          -oracle.matmul(xq, wr))


def test_matmul_reports_int32_overflow():
    K = 140000                               # 128 * 128 * K > 2^31
    xq = np.full((1, K), -128, dtype=np.int8)
    wq = np.full((1, K), -128, dtype=np.int8)
    with pytest.raises(OverflowError):
        oracle.matmul(xq, wq)


# ---------------------------------------------------------------- quantizer

def test_quantizer_ties_go_to_even():
    # scale = 15.5 / 31 = 0.5 exactly, so v / s = 2 v is exact
    v = np.array([[15.5, 1.25, 1.75, -1.25, -1.75, 0.25, 0.75, -0.25, 2.25, 0.0]], dtype=np.float32)
    q, s = oracle.quantize(v, 6)
    assert float(s[0]) == 0.5
    assert q[0].tolist() == [31, 2, 4, -2, -4, 0, 2, 0, 4, 0]
    v8 = np.array([[127.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5]], dtype=np.float32)
    q, s = oracle.quantize(v8, 8)
    assert float(s[0]) == 1.0
    assert q[0].tolist() == [127, 2, 4, -2, -4, 0, 2]


@pytest.mark.parametrize("bits", [6, 8])
def test_quantizer_grid_values_reproduce_and_idempotent(bits):
    qmax = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(bits)
    for s in (2.0**-7, 0.25, 8.0):
        k = rng.integers(-qmax, qmax + 1, (5, 256))
        k[:, 0] = qmax                        # pins absmax, hence the scale
        v = (k * s).astype(np.float32)
        q, sc = oracle.quantize(v, bits)
        assert np.all(sc.astype(np.float64) == s)
        assert np.array_equal(q, k)
        q2, sc2 = oracle.quantize((q.astype(np.float32) * np.float32(s)), bits)
        assert np.array_equal(q2, q) and np.array_equal(sc2, sc)


@pytest.mark.parametrize("bits,group", [(6, 0), (6, 128), (8, 0)])
def test_quantizer_invariants_random(bits, group):
    qmax = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(10 + bits + group)
    v = (rng.standard_normal((16, 512)) * 0.02).astype(np.float32)
    v[:, 5] *= 20
    q, s = oracle.quantize(v, bits, group)
    G = 512 if group == 0 else group
    s2 = s.reshape(16, 512 // G).astype(np.float64)
    vg = v.reshape(16, 512 // G, G).astype(np.float64)
    qg = q.reshape(16, 512 // G, G).astype(np.float64)
    amax = np.abs(vg).max(2)
    # scale is the fp16 nearest to absmax / qmax
    assert np.all(np.abs(s2 * qmax - amax) <= amax * 2.0**-11 * (1 + 1e-6))
    assert q.min() >= -qmax - 1 and q.max() <= qmax
    # reconstruction error at most half a step (plus fp32 division rounding)
    assert np.all(np.abs(vg - qg * s2[:, :, None]) <= 0.5 * s2[:, :, None] * (1 + 1e-5))
    # the largest element of each group lands on +-qmax
    idx = np.abs(vg).argmax(2)
    top = np.take_along_axis(qg, idx[:, :, None], 2)[:, :, 0]
    assert np.all(np.abs(top) == qmax)
    # a second implementation with numpy's own fp32 divide / rint / fp16 cast
    sref = (amax.astype(np.float32) / np.float32(qmax)).astype(np.float16)
    assert np.array_equal(sref, s.reshape(sref.shape))
    qref = np.clip(np.rint(vg.astype(np.float32) / sref.astype(np.float32)[:, :, None]),
                   -qmax - 1, qmax)
    assert np.array_equal(qref.reshape(16, 512), q.astype(np.float32))


def test_quantizer_zero_row_and_clamp():
    v = np.zeros((2, 128), dtype=np.float32)
    v[1, 3] = 1.0
    q, s = oracle.quantize(v, 6)
    assert float(s[0]) == 1.0 and np.all(q[0] == 0)
    # absmax / 31 = 1.4 * 2^-24 rounds DOWN to the fp16 subnormal 2^-24, so the
    # quotient 43.4 leaves the code range: +absmax clamps to 31, -absmax to -32
    a = np.float32(31 * 1.4 * 2.0**-24)
    v = np.array([[a, -a, a / 4, 0.0]], dtype=np.float32)
    q, s = oracle.quantize(v, 6)
    assert float(s[0]) == 2.0**-24
    assert q[0].tolist() == [31, -32, 11, 0]
    # absmax so small that the fp16 scale underflows to zero -> scale 1.0
    v = np.array([[1e-9, -1e-9]], dtype=np.float32)
    q, s = oracle.quantize(v, 8)
    assert float(s[0]) == 1.0 and np.all(q == 0)


# --------------------------------------------------------------- dequantize

def _nearest_fp16_check(exact, got_bits):
    """True iff fp16 `got_bits` is a nearest fp16 to the exact rational."""
    got = np.array([got_bits], dtype=np.uint16).view(np.float16)[0]
    if not np.isfinite(got):
        return abs(exact) >= Fraction(65520)
    g = Fraction(float(got))
    err = abs(g - exact)
    for nb in (np.nextafter(got, np.float16(np.inf)), np.nextafter(got, np.float16(-np.inf))):
        if np.isfinite(nb) and abs(Fraction(float(nb)) - exact) < err:
            return False
    return True


def test_dequant_per_channel_is_correctly_rounded():
    rng = np.random.default_rng(20)
    M, N = 6, 40
    acc = rng.integers(-2**30, 2**30, (M, N))
    acc[0, :4] = [0, 1, -1, 2**31 - 1]
    sx = (rng.uniform(0.001, 0.2, M)).astype(np.float16)
    sw = (rng.uniform(1e-4, 4e-3, N)).astype(np.float16)
    y = oracle.dequant(acc, sx, sw).view(np.uint16)
    for m in range(M):
        for n in range(N):
            exact = Fraction(int(acc[m, n])) * Fraction(float(sx[m])) * Fraction(float(sw[n]))
            assert _nearest_fp16_check(exact, y[m, n]), (m, n)
    # and against numpy: the fp64 product is exact here, its fp16 cast is one rounding
    with np.errstate(over="ignore"):
        ref = (acc.astype(np.float64) * sx.astype(np.float64)[:, None]
               * sw.astype(np.float64)[None, :]).astype(np.float16)
    assert np.array_equal(ref.view(np.uint16), y)


def test_dequant_power_of_two_scales_exact():
    acc = np.array([[3, -5, 1024, 2047, -2048, 0]], dtype=np.int64)
    sx = np.array([0.5], dtype=np.float16)
    sw = np.full(6, 2.0**-3, dtype=np.float16)
    y = oracle.dequant(acc, sx, sw).astype(np.float64)
    assert np.array_equal(y, acc.astype(np.float64) * 2.0**-4)


def test_dequant_group_mode_exact_rational():
    rng = np.random.default_rng(21)
    M, N, G = 3, 17, 5
    acc = rng.integers(-2**21, 2**21, (M, N, G))
    sx = rng.uniform(0.01, 0.1, M).astype(np.float16)
    sw = rng.uniform(1e-4, 4e-3, (N, G)).astype(np.float16)
    y = oracle.dequant(acc, sx, sw).view(np.uint16)
    y2 = oracle.dequant_xgroup(acc, np.repeat(sx[:, None], G, 1), sw).view(np.uint16)
    for m in range(M):
        for n in range(N):
            exact = Fraction(float(sx[m])) * sum(
                Fraction(float(sw[n, g])) * int(acc[m, n, g]) for g in range(G))
            assert _nearest_fp16_check(exact, y[m, n])
            assert _nearest_fp16_check(exact, y2[m, n])
    # one group with the whole sum == per-channel call
    assert np.array_equal(oracle.dequant(acc[:, :, :1], sx, sw[:, :1]),
                          oracle.dequant(acc[:, :, 0], sx, sw[:, 0]))


def test_dequant_xgroup_scales_belong_to_their_group():
    # acc only in group 1: the result must use sx[:,1] and sw[:,1]
    acc = np.zeros((1, 1, 3), dtype=np.int64)
    acc[0, 0, 1] = 8
    sx = np.array([[1.0, 0.5, 4.0]], dtype=np.float16)
    sw = np.array([[2.0, 0.25, 8.0]], dtype=np.float16)
    assert float(oracle.dequant_xgroup(acc, sx, sw)[0, 0]) == 1.0


# ------------------------------------------------------------------ 6 bits

def test_pack6_dense_round_trip_and_size():
    codes = np.arange(-32, 32, dtype=np.int8)
    w = np.concatenate([np.roll(codes, r) for r in range(64)])      # every code at every phase
    packed = oracle.pack6_dense(w)
    assert packed.size * 8 == w.size * 6
    assert np.array_equal(oracle.unpack6_dense(packed, w.size), w)
    # layout pin: four codes 1, 2, 3, -1 -> bits laid end to end, little endian
    four = oracle.pack6_dense(np.array([1, 2, 3, -1], dtype=np.int8))
    value = 1 | (2 << 6) | (3 << 12) | (63 << 18)
    assert four.tolist() == [value & 255, (value >> 8) & 255, value >> 16]


# ------------------------------------------------ activation producers

def test_rmsnorm_against_library_and_closed_forms():
    import torch
    rng = np.random.default_rng(40)
    M, K = 5, 384
    x = (rng.standard_normal((M, K)) * 3).astype(np.float16)
    g = rng.uniform(0.5, 1.5, K).astype(np.float16)
    eps = 1e-5
    h = oracle.rmsnorm(x, g, eps)
    # library routine, fp64, one rounding to fp16
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x.astype(np.float64)), (K,),
                                       torch.from_numpy(g.astype(np.float64)), eps).numpy()
    assert np.array_equal(h.view(np.uint16), ref.astype(np.float16).view(np.uint16))
    # all-ones row: every output is gamma / sqrt(1 + eps)
    ones = np.ones((1, K), dtype=np.float16)
    h1 = oracle.rmsnorm(ones, g, 0.25)
    assert np.array_equal(h1[0].view(np.uint16),
                          (g.astype(np.float64) / np.sqrt(1.25)).astype(np.float16).view(np.uint16))
    # eps = 0: scaling the input by a power of two changes nothing
    assert np.array_equal(oracle.rmsnorm(x, g, 0.0).view(np.uint16),
                          oracle.rmsnorm((x.astype(np.float32) * 4).astype(np.float16), g, 0.0).view(np.uint16))
    # gamma belongs to the column, not the row
    g2 = g.copy()
    g2[7] = 0
    assert np.all(oracle.rmsnorm(x, g2, eps)[:, 7] == 0)


def test_swiglu_against_library_and_identities():
    import torch
    rng = np.random.default_rng(41)
    M, F = 4, 320
    gu = (rng.standard_normal((M, 2 * F)) * 4).astype(np.float16)
    h = oracle.swiglu(gu)
    g64 = torch.from_numpy(gu[:, :F].astype(np.float64))
    u64 = torch.from_numpy(gu[:, F:].astype(np.float64))
    ref = (torch.nn.functional.silu(g64) * u64).numpy().astype(np.float16)
    assert np.array_equal(h.view(np.uint16), ref.view(np.uint16))
    # silu(g) - silu(-g) = g, so with up = 1 the two halves differ by exactly g (in fp64;
    # here checked on values where the fp16 roundings are exact: g = 0)
    z = np.zeros((1, 2 * F), dtype=np.float16)
    z[0, F:] = 3.0
    assert np.all(oracle.swiglu(z) == 0)
    big = np.zeros((1, 2 * F), dtype=np.float16)
    big[0, :F] = 30.0                       # silu(30) = 30 to fp16 precision
    big[0, F:] = 0.5
    assert np.all(oracle.swiglu(big) == 15.0)
    # gate and up are not interchangeable: silu(-30) ~ 0
    swapped = np.concatenate([big[:, F:], -big[:, :F]], axis=1)
    assert not np.array_equal(oracle.swiglu(swapped), oracle.swiglu(big))


# -------------------------------------------------------- end-to-end sanity

def test_linear_tracks_real_arithmetic_on_tiny_config():
    M, K, N = 4, 256, 128                     # the tiny configuration, seed 0
    w = synth.weights(N, K, 0.02, seed=0)
    x = synth.activations(M, K, seed=0, outlier_frac=0.02, outlier_scale=20.0)
    exact = x.astype(np.float64) @ w.astype(np.float64).T
    errs = {}
    for bits in (6, 8):
        r = oracle.linear(x, w, bits)
        y = r["y"].astype(np.float64)
        cos = (y * exact).sum() / np.sqrt((y * y).sum() * (exact * exact).sum())
        assert cos >= 0.99
        errs[bits] = np.abs(y - exact).mean()
        assert r["wq"].min() >= -32 and r["wq"].max() <= 31
        assert np.array_equal(r["acc"], r["xq"].astype(np.int64) @ r["wq"].astype(np.int64).T)
    assert errs[8] < errs[6]                  # outlier channels hurt A6 more than A8
    rg = oracle.linear(x, w, 8, group=128)
    assert rg["sw"].shape == (N, 2)
    yg = rg["y"].astype(np.float64)
    assert (yg * exact).sum() / np.sqrt((yg * yg).sum() * (exact * exact).sum()) >= 0.99


def test_synth_rows_regenerate_identically():
    w = synth.weights(600, 128, 0.015, seed=42)
    rows = [0, 255, 256, 599]
    assert np.array_equal(synth.weight_rows_at(600, 128, 0.015, 42, rows), w[rows])
    assert np.array_equal(synth.weight_rows(600, 128, 0.015, 42, 200, 300), w[200:300])
    x = synth.activations(8, 512, seed=3, outlier_frac=0.02)
    assert x.dtype == np.float16 and x.shape == (8, 512)
    big = np.abs(x.astype(np.float32)).mean(0)
    assert (big > 8).sum() == round(0.02 * 512)      # outliers persist across tokens
