"""Pins of the oracle's real-valued per-group path (Sec. 3.3.2 of the QQQ paper: FastINT4toFP16,
FusedDequantQuant as one fp16 FMA with 128 + 1024, low mantissa byte, XOR 0x80) against things
other than itself.  CPU only.

Pins: numpy's own float64 -> float16 conversion (library routine) for the rounding helper; exact
rational arithmetic with Python's round() (round half to even on Fractions) for the weight
conversion over every code and every finite fp16 scale in the no-overflow domain; a bit-level
walk through the paper's steps on exact rationals for a sample of out-of-domain scales; the
integer-scale oracle for integer scales (the two paths must agree where neither saturates); a
brute-force product for the GEMM.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import synth


def half_value(bits):
    """Exact rational value of a finite fp16 bit pattern (written from the IEEE 754 definition)."""
    sign = -1 if bits & 0x8000 else 1
    e, m = (bits >> 10) & 0x1F, bits & 0x3FF
    assert e != 31
    if e == 0:
        return sign * Fraction(m, 1 << 24)
    return sign * Fraction(1024 + m, 1024) * Fraction(2) ** (e - 15)


def round_to_half_bits(x):
    """Exact rational -> fp16 bits, round half to even, overflow to inf (independent of the C code:
    it searches the representable neighbours instead of scaling)."""
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    if a >= Fraction(65520):
        return sign | 0x7C00
    lo, hi = 0, 0x7BFF                      # magnitudes are ordered like their bit patterns
    while lo < hi:                          # largest pattern whose value <= a
        mid = (lo + hi + 1) // 2
        if half_value(mid) <= a:
            lo = mid
        else:
            hi = mid - 1
    below = half_value(lo)
    if below == a:
        return sign | lo
    above = half_value(lo + 1) if lo < 0x7BFF else Fraction(65536)
    if a - below < above - a or (a - below == above - a and lo % 2 == 0):
        return sign | lo
    return sign | (lo + 1)


def paper_steps(code, s_bits):
    """FastINT4toFP16 -> one FMA with 1152 -> low byte -> XOR 0x80, on exact rationals."""
    x = round_to_half_bits(Fraction(code) * half_value(s_bits) + 1152)
    b = (x & 0xFF) ^ 0x80
    return b - 256 if b >= 128 else b


def test_double_to_half_vs_numpy_conversion():
    g = synth.rng(11)
    x = np.concatenate([
        g.standard_normal(200000) * 300.0,
        g.standard_normal(50000) * 1e-6,
        g.uniform(-70000, 70000, 50000),
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, -65520.0, 1e9, 2.0 ** -24, 2.0 ** -25,
                  2.0 ** -25 * 1.0000001, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1152.5, 1153.5]),
    ])
    ref = x.astype(np.float16).view(np.uint16)
    got = np.array([orc.double_to_half(v) for v in x], dtype=np.uint16)
    assert np.array_equal(got, ref)
    # every fp16 value is a fixed point, every midpoint between neighbours goes to the even one
    bits = np.arange(0, 0x7C00, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    assert all(orc.double_to_half(v) == b for v, b in zip(vals[::7], bits[::7]))
    mid = (vals[:-1] + vals[1:]) / 2
    want = np.where(bits[:-1] % 2 == 0, bits[:-1], bits[1:])
    assert all(orc.double_to_half(v) == w for v, w in zip(mid[::5], want[::5]))


def test_rational_rounding_helper_agrees_with_numpy_on_a_sample():
    g = synth.rng(12)
    for v in np.concatenate([g.standard_normal(300) * 50, g.uniform(1100, 1300, 200)]):
        fr = Fraction(float(v))
        assert round_to_half_bits(fr) == int(np.float64(v).astype(np.float16).view(np.uint16))


def test_w8_f16scale_is_round_half_even_of_the_exact_product_in_domain():
    """Every code x every finite fp16 scale with |code*s| small enough that the rounded product
    fits int8: the result is the exact product rounded half to even (Sec. 3.3.2: the FMA's
    rounding in the [1024,2048) binade is a rounding to integer)."""
    checked = 0
    for s_bits in range(0, 0x10000):
        if (s_bits >> 10) & 0x1F == 31:
            continue
        s = half_value(s_bits)
        if abs(s) * 8 > 127:
            continue
        for code in range(-8, 8):
            want = round(Fraction(code) * s)          # Python: exact, ties to even
            assert -128 <= want <= 127
            assert orc.w8_f16scale_one(code, s_bits) == want, (code, hex(s_bits))
            checked += 1
    assert checked > 16 * 38000        # about 61 % of the finite fp16 patterns lie in the domain


def test_w8_f16scale_ties_and_unit_scales():
    half = int(np.float16(0.5).view(np.uint16))
    assert [orc.w8_f16scale_one(c, half) for c in range(-8, 8)] == \
        [-4, -4, -3, -2, -2, -2, -1, 0, 0, 0, 1, 2, 2, 2, 3, 4]      # x.5 goes to the even integer
    one = int(np.float16(1.0).view(np.uint16))
    assert [orc.w8_f16scale_one(c, one) for c in range(-8, 8)] == list(range(-8, 8))
    neg = int(np.float16(-2.0).view(np.uint16))
    assert [orc.w8_f16scale_one(c, neg) for c in range(-8, 8)] == [-2 * c for c in range(-8, 8)]


def test_w8_f16scale_follows_the_papers_steps_outside_the_domain_too():
    """No saturation: outside [-128,127] the byte extraction decides.  A walk through the paper's
    steps on exact rationals gives the same byte for a spread of large, tiny and negative scales."""
    g = synth.rng(13)
    sample = list(g.integers(0, 0x10000, 3000)) + [0x7BFF, 0xFBFF, 0x0001, 0x8001, 0x4C00, 0x5000,
                                                    0x5C00, 0x6400, 0xE400, 0x6800]
    for s_bits in sample:
        s_bits = int(s_bits)
        if (s_bits >> 10) & 0x1F == 31:
            continue
        for code in (-8, -7, -1, 0, 1, 5, 7):
            assert orc.w8_f16scale_one(code, s_bits) == paper_steps(code, s_bits), (code, hex(s_bits))


def test_integer_scales_reduce_to_the_integer_scale_oracle():
    """With integer scales up to 15 nothing saturates and both per-group oracles must agree."""
    N, K = 48, 512
    w = synth.random_w_nat(N, K, 21)
    s_int = synth.group_scales(K, N, 22, 1, 15)
    s_f16 = s_int.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.w8_pergroup_f16(w, s_f16, K), orc.w8_pergroup(w, s_int, K))


def test_gemm_pergroup_f16_vs_python_brute_force():
    M, N, K = 3, 16, 256
    g = synth.rng(31)
    a_q = synth.int8_activations(M, K, 32)
    s_a = synth.token_scales(M, 33)
    w = synth.random_w_nat(N, K, 34)
    s_g = g.uniform(0.05, 15.8, (K // 128, N)).astype(np.float16)
    s_w = synth.weight_scales_fp16(N, 35, 0.001, 0.005)
    acc, y32, y = orc.gemm_pergroup_f16(a_q, s_a, w, s_g.view(np.uint16), s_w.view(np.uint16))
    codes = np.zeros((N, K), np.int64)
    for n in range(N):
        for k in range(K):
            nib = (int(w[n, k // 8]) >> (4 * (k % 8))) & 0xF
            codes[n, k] = nib - 16 if nib >= 8 else nib
    for m in range(M):
        for n in range(N):
            tot = 0
            for k in range(K):
                w8 = round(Fraction(int(codes[n, k])) * Fraction(float(s_g[k // 128, n])))
                tot += int(a_q[m, k]) * w8
            assert acc[m, n] == tot
            ref = np.float32(float(tot) * float(s_a[m]) * float(np.float32(s_w[n])))
            assert y[m, n] == np.float16(ref).view(np.uint16)


def test_f16scale_shape_and_null_errors():
    w = synth.random_w_nat(16, 128, 1)
    with pytest.raises(AssertionError):
        orc.w8_pergroup_f16(w, np.zeros((2, 16), np.uint16), 128)


def test_sampled_evaluation_equals_the_full_product():
    M, N, K = 5, 48, 512
    a = synth.int8_activations(M, K, 1)
    sa = synth.token_scales(M, 2)
    w = synth.random_w_nat(N, K, 3)
    sg = synth.group_scales_f16(K, N, 4).view(np.uint16)
    sw = synth.weight_scales_fp16(N, 5, 0.001, 0.005).view(np.uint16)
    acc, _, y = orc.gemm_pergroup_f16(a, sa, w, sg, sw)
    im, jn = np.repeat(np.arange(M), N), np.tile(np.arange(N), M)
    a2, y2 = orc.gemm_samples_f16(a, sa, w, sg, sw, im, jn)
    assert np.array_equal(a2.reshape(M, N), acc) and np.array_equal(y2.reshape(M, N), y)
