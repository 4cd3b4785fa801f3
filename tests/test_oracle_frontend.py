"""Pins of the oracle's offline front-end (symmetric round-to-nearest int4 weights from fp16,
per-channel scale of Sec. 3.3.1 and the s_Wg / s_Wc / s*_Wg of Sec. 3.3.2, Fig. 5) against things
other than itself.  CPU only.

Pins: weights that lie exactly on a quantisation grid (codes and scales must come back exactly);
numpy's float16/float32 arithmetic for the scales; exact rational arithmetic (Fractions, Python's
round half to even) for every code of small matrices; the round-to-nearest error bound |w - code*s|
<= s/2; the s^2/12 noise law on uniform weights; the no-wrap property of the real-valued
conversion on the scales produced (checked through the already pinned code x scale conversion);
an end-to-end linear layer against float64.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import synth


def codes_of(w_nat, K):
    """int [N,K] codes from the natural nibble format (written out here, not the oracle's reader)."""
    w = np.asarray(w_nat, np.uint32)
    out = np.empty((w.shape[0], K), np.int64)
    for i in range(8):
        nib = ((w >> np.uint32(4 * i)) & np.uint32(0xF)).astype(np.int64)
        out[:, i::8] = np.where(nib >= 8, nib - 16, nib)
    return out


def f16(bits):
    return np.asarray(bits, np.uint16).view(np.float16).astype(np.float64)


def grid_weights(N, K, seed, scale_of_group):
    """codes in [-7,7] with a +-7 in every group of 128, times a power-of-two scale per (n, group)."""
    g = synth.rng(seed)
    codes = g.integers(-7, 8, size=(N, K))
    G = K // 128
    pos = g.integers(0, 128, size=(N, G))
    sign = g.choice([-7, 7], size=(N, G))
    for j in range(G):
        codes[np.arange(N), j * 128 + pos[:, j]] = sign[:, j]
    s = np.empty((N, G))
    for n in range(N):
        for j in range(G):
            s[n, j] = scale_of_group(n, j)
    w = codes * np.repeat(s, 128, axis=1)
    w16 = w.astype(np.float16)
    assert np.array_equal(w16.astype(np.float64), w)          # exactly representable
    return codes, s, w16


def test_perchannel_grid_weights_come_back_exactly():
    N, K = 24, 384
    codes, s, w16 = grid_weights(N, K, 1, lambda n, j: 2.0 ** -(4 + n % 5))
    w_nat, s_w = orc.quantize_w4_perchannel(w16.view(np.uint16))
    assert np.array_equal(f16(s_w), s[:, 0])                 # 7s/7 = s, a power of two
    assert np.array_equal(codes_of(w_nat, K), codes)
    assert np.array_equal(w_nat, synth.codes_to_w_nat(codes))  # nibble i of word j is W[n, 8j+i]


def test_pergroup_grid_weights_and_scales_in_closed_form():
    N, K = 20, 640                                           # G = 5 != N: a transposed scale table fails
    G = K // 128
    codes, s, w16 = grid_weights(N, K, 2, lambda n, j: 2.0 ** -(5 + (n + 2 * j) % 4))
    w_nat, s_wg, s_star, s_int, s_wc = orc.quantize_w4_pergroup(w16.view(np.uint16))
    assert np.array_equal(codes_of(w_nat, K), codes)
    assert np.array_equal(f16(s_wg), s.T)                    # [G, N]
    dmax = 7.0 * s.max(axis=1)                               # every group holds a +-7
    want_wc = (dmax.astype(np.float32) / np.float32(127)).astype(np.float16)
    assert np.array_equal(s_wc, want_wc.view(np.uint16))
    want_star = (s.T.astype(np.float32) / want_wc.astype(np.float32)[None, :]).astype(np.float16)
    assert np.array_equal(s_star, want_star.view(np.uint16))
    assert np.array_equal(s_int, np.clip(np.rint(want_star.astype(np.float64)), 1, 18).astype(np.int8))
    # the group with the channel's largest scale maps its +-7 to +-127
    top = f16(s_star).max(axis=0)
    assert np.all(np.rint(7 * top) == 127)


def exact_code(w_bits, s_bits):
    """clamp(round_half_even(fl32(w/s)), -7, 7) on exact rationals; fl32 = correctly rounded to 24 bits."""
    w = Fraction(float(np.uint16(w_bits).view(np.float16)))
    s = Fraction(float(np.uint16(s_bits).view(np.float16)))
    if s == 0:
        return 0
    q = w / s
    if q != 0:                                               # round the quotient to 24 significant bits
        a = abs(q)
        e = 0
        while a >= 2:
            a /= 2
            e += 1
        while a < 1:
            a *= 2
            e -= 1
        m = round(a * (1 << 23))                             # Python's round: half to even
        q = (1 if q > 0 else -1) * Fraction(m, 1 << 23) * Fraction(2) ** e
    return max(-7, min(7, round(q)))


def test_every_code_of_small_matrices_against_exact_rationals():
    w16 = synth.weights_fp16(6, 256, 3)
    w16[1, :] = 0                                            # an all-zero channel
    w16[2, 128:] = 0                                         # an all-zero group
    w16[3, :] = (w16[3, :].astype(np.float32) * 1e-4).astype(np.float16)   # subnormal scales
    bits = w16.view(np.uint16)
    w_nat, s_w = orc.quantize_w4_perchannel(bits)
    c = codes_of(w_nat, 256)
    for n in range(6):
        amax = Fraction(float(np.abs(w16[n].astype(np.float64)).max()))
        want_s = np.float16(np.float32(float(amax)) / np.float32(7))
        assert s_w[n] == want_s.view(np.uint16)
        for k in range(256):
            assert c[n, k] == exact_code(bits[n, k], s_w[n]), (n, k)
    w_nat, s_wg, s_star, s_int, s_wc = orc.quantize_w4_pergroup(bits)
    c = codes_of(w_nat, 256)
    for n in range(6):
        for k in range(256):
            assert c[n, k] == exact_code(bits[n, k], s_wg[k // 128, n]), (n, k)
    assert np.all(c[1] == 0) and s_w[1] == 0 and s_wc[1] == 0 and np.all(s_star[:, 1] == 0)
    assert np.all(c[2, 128:] == 0) and s_wg[1, 2] == 0 and s_star[1, 2] == 0 and s_int[1, 2] == 1


@pytest.mark.parametrize("variant", ["perchannel", "pergroup"])
def test_round_to_nearest_error_bound_and_full_range(variant):
    N, K = 64, 1024
    w16 = synth.weights_fp16(N, K, 4)
    w = w16.astype(np.float64)
    if variant == "perchannel":
        w_nat, s_w = orc.quantize_w4_perchannel(w16.view(np.uint16))
        s = np.repeat(f16(s_w)[:, None], K, axis=1)
    else:
        w_nat, s_wg, _, _, _ = orc.quantize_w4_pergroup(w16.view(np.uint16))
        s = np.repeat(f16(s_wg).T, 128, axis=1)
    c = codes_of(w_nat, K)
    assert c.min() >= -7 and c.max() <= 7
    # the scale is max|w|/7 up to one fp16 rounding, so no weight is clipped by more than that rounding
    assert np.all(np.abs(w - c * s) <= s * (0.5 + 7 * 2.0 ** -11) + 1e-12)
    blocks = np.abs(c).reshape(N, -1, K if variant == "perchannel" else 128).max(axis=2)
    assert np.all(blocks == 7)                               # the largest weight of a block maps to +-7
    # sign and order are kept
    assert np.all(np.sign(c) * np.sign(w) >= 0)


def test_uniform_weights_follow_the_step_squared_over_twelve_law():
    g = synth.rng(5)
    w16 = g.uniform(-1, 1, size=(32, 4096)).astype(np.float16)
    w_nat, s_w = orc.quantize_w4_perchannel(w16.view(np.uint16))
    s = f16(s_w)[:, None]
    err = w16.astype(np.float64) - codes_of(w_nat, 4096) * s
    ratio = (err ** 2).mean() / (s ** 2 / 12).mean()
    assert 0.97 < ratio < 1.03


def test_fused_scale_is_the_ratio_and_never_wraps():
    N, K = 48, 1024
    w16 = synth.weights_fp16(N, K, 6)
    w16[5] = (w16[5].astype(np.float32) * 2e-3).astype(np.float16)   # s_Wc subnormal in fp16: the cap may bind
    w16[6] = (w16[6].astype(np.float32) * 2e-4).astype(np.float16)
    w_nat, s_wg, s_star, s_int, s_wc = orc.quantize_w4_pergroup(w16.view(np.uint16))
    sg, st, wc = f16(s_wg), f16(s_star), f16(s_wc)
    normal = wc >= 2.0 ** -14
    rel = np.abs(st * wc[None, :] - sg) / np.maximum(sg, 1e-30)
    assert np.all(rel[:, normal] <= 2.0 ** -10)              # one fp16 rounding of the quotient
    assert st.max() <= 18.203125
    # dequantised weights w~ = code * s_Wg; s_Wc is their largest magnitude over 127
    c = codes_of(w_nat, K)
    wd = np.abs(c * np.repeat(sg.T, 128, axis=1)).max(axis=1)
    assert np.array_equal(s_wc, (wd.astype(np.float32) / np.float32(127)).astype(np.float16).view(np.uint16))
    # through the pinned code x scale conversion: the int8 weight is rne(code * s*), inside +-127
    w8 = orc.w8_pergroup_f16(w_nat, s_star, K).astype(np.int64)
    assert np.abs(w8).max() <= 127
    assert np.array_equal(w8, np.rint(c * np.repeat(st.T, 128, axis=1)).astype(np.int64))
    assert np.all(np.abs(w8[normal]).max(axis=1) >= 126)
    # int8 weight times s_Wc is the original weight up to the two roundings
    back = w8 * wc[:, None]
    bound = 0.5 * np.repeat(sg.T, 128, axis=1) * 1.01 + 0.5 * wc[:, None] * 1.01
    ok = np.abs(back - w16.astype(np.float64)) <= bound + 1e-12
    assert np.all(ok[normal])
    assert np.array_equal(s_int, np.clip(np.rint(st), 1, 18).astype(np.int8))


def test_linear_layer_from_fp16_weights_end_to_end():
    M, K, N = 8, 1024, 96
    w16 = synth.weights_fp16(N, K, 7)
    a16 = synth.activations_fp16(M, K, 8)
    ref = a16.astype(np.float64) @ w16.astype(np.float64).T
    a_q, s_a = orc.quant_act(a16.view(np.uint16))
    w_nat, s_w = orc.quantize_w4_perchannel(w16.view(np.uint16))
    _, _, y = orc.gemm_perchannel(a_q, s_a, w_nat, s_w)
    e_pc = np.linalg.norm(f16(y) - ref) / np.linalg.norm(ref)
    w_nat, _, s_star, s_int, s_wc = orc.quantize_w4_pergroup(w16.view(np.uint16))
    _, _, y = orc.gemm_pergroup_f16(a_q, s_a, w_nat, s_star, s_wc)
    e_pg = np.linalg.norm(f16(y) - ref) / np.linalg.norm(ref)
    _, _, y = orc.gemm_pergroup(a_q, s_a, w_nat, s_int, s_wc)
    e_int = np.linalg.norm(f16(y) - ref) / np.linalg.norm(ref)
    # prediction from the uniform-noise law: every weight carries independent noise of variance step^2/12
    a = a16.astype(np.float64)
    step_pc = np.repeat(f16(s_w)[:, None], K, axis=1)
    pred_pc = np.sqrt(((a ** 2) @ (step_pc ** 2 / 12).T).sum()) / np.linalg.norm(ref)
    step_pg = np.repeat(f16(orc.quantize_w4_pergroup(w16.view(np.uint16))[1]).T, 128, axis=1)
    pred_pg = np.sqrt(((a ** 2) @ (step_pg ** 2 / 12).T).sum()) / np.linalg.norm(ref)
    assert 0.8 * pred_pc < e_pc < 1.2 * pred_pc
    assert 0.8 * pred_pg < e_pg < 1.25 * pred_pg              # plus the int8 rounding of code * s*
    assert e_pg < e_pc                                        # finer scales, less noise
    assert e_pg <= e_int < 2.0 * e_pg + 0.1                   # the integer-rounded fused scale costs accuracy


def test_leading_dimension_and_shape_errors():
    w16 = synth.weights_fp16(4, 256, 9)
    wide = np.zeros((4, 320), np.float16)
    wide[:, :256] = w16
    wide[:, 256:] = 100.0                                    # must be ignored
    import ctypes
    L = orc.lib()
    w_nat = np.zeros((4, 32), np.uint32)
    s_w = np.zeros(4, np.uint16)
    rc = L.qqq_oracle_quantize_w4_perchannel(wide.view(np.uint16).ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                                             4, 256, 320, w_nat.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                                             s_w.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    assert rc == 0
    ref_nat, ref_s = orc.quantize_w4_perchannel(w16.view(np.uint16))
    assert np.array_equal(w_nat, ref_nat) and np.array_equal(s_w, ref_s)
    with pytest.raises(Exception):
        orc.quantize_w4_pergroup(synth.weights_fp16(4, 192, 9).view(np.uint16))   # K % 128 != 0
