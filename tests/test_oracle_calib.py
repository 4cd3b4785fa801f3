"""Pins of the calibration oracle (adaptive smoothing, Sec. 3.1 Eq. 1-2; Hessian-based compensation,
Sec. 3.2 Eq. 3-4) against what the mathematics fixes: closed forms, exact rationals on tiny layers,
special cases that reduce to the pinned front-end, an independent (Cholesky) formulation, invariants."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qqq_calib_oracle as cal
from oracle import qqq_oracle as orc
from paper_2406_09904_amd import synth


def f16bits(a):
    return np.ascontiguousarray(np.asarray(a, np.float16)).view(np.uint16)


def layer(M, K, N, seed, outliers=(), scale=30.0):
    g = synth.rng(seed)
    x = g.standard_normal((M, K)).astype(np.float32)
    for t in outliers:
        x[:, t] *= scale
    w = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    return f16bits(x), f16bits(w)


# ------------------------------------------------------------------ smoothing

def test_channel_absmax_and_grid():
    x, _ = layer(37, 24, 8, 1)
    ref = np.abs(x.view(np.float16).astype(np.float64)).max(axis=0)
    assert np.array_equal(cal.channel_absmax(x).astype(np.float64), ref)
    grid = cal.sigma_grid(cal.channel_absmax(x), 10)
    assert len(grid) == 10 and grid[-1] == np.float32(ref.max())
    assert np.allclose(np.diff(grid), ref.max() / 10, rtol=1e-6)


def test_no_channel_above_the_top_threshold_means_no_smoothing():
    x, w = layer(16, 32, 8, 2, outliers=(3,))
    am = cal.channel_absmax(x)
    s, sel = cal.smoothing_vector(am, am.max())          # strict ">": nothing selected
    assert not sel.any() and np.all(s == 1.0)
    xs, ws = cal.apply_smoothing(x, w, s)
    assert np.array_equal(xs, x) and np.array_equal(ws, w)
    # and the loss is then the plain quantisation error of the layer
    d = cal.quantised_product(x, w) - cal.reference_product(x, w)
    assert cal.smoothing_loss(x, w, s) == pytest.approx(float(np.sum(d * d)), rel=1e-12)


def test_selected_set_is_the_channels_above_the_threshold_and_they_land_on_it():
    x, w = layer(64, 48, 8, 3, outliers=(5, 17, 40))
    am = cal.channel_absmax(x)
    sigma = np.float32(np.sort(am)[-4] * 1.5)            # between the bulk and the three planted outliers
    s, sel = cal.smoothing_vector(am, sigma)
    assert sorted(np.nonzero(sel)[0].tolist()) == [5, 17, 40]
    assert np.all(s[~sel] == 1.0) and np.all(s[sel] > 1.0)
    xs, _ = cal.apply_smoothing(x, w, s)
    smoothed_max = np.abs(xs.view(np.float16).astype(np.float64)).max(axis=0)
    assert np.allclose(smoothed_max[sel], float(sigma), rtol=2e-3)          # scaled down to the threshold
    assert np.array_equal(smoothed_max[~sel], am[~sel].astype(np.float64))  # others untouched


def test_real_valued_product_is_unchanged_by_power_of_two_smoothing():
    x, w = layer(8, 16, 4, 4)
    s = np.array([1, 2, 4, 1, 8, 1, 1, 2, 1, 1, 16, 1, 1, 1, 4, 1], np.float32)
    xs, ws = cal.apply_smoothing(x, w, s)                 # exact in fp16: powers of two
    assert np.array_equal(cal.reference_product(xs, ws), cal.reference_product(x, w))


def test_loss_against_exact_rationals_on_a_tiny_layer():
    """Eq. 2 written out with Fractions: the oracle's quantisers give codes and scales, the rest is exact."""
    x, w = layer(2, 8, 2, 5, outliers=(1,))
    am = cal.channel_absmax(x)
    s, _ = cal.smoothing_vector(am, np.float32(am.max() / 4))
    xs, ws = cal.apply_smoothing(x, w, s)
    a_q, s_a = orc.quant_act(xs)
    w_nat, s_w = orc.quantize_w4_perchannel(ws)
    codes = orc.w8_perchannel(w_nat, 8)
    total = Fraction(0)
    X, W = x.view(np.float16), w.view(np.float16)
    for m in range(2):
        for n in range(2):
            acc = sum(int(a_q[m, k]) * int(codes[n, k]) for k in range(8))
            yq = Fraction(float(s_a[m])) * Fraction(float(orc.half_to_float(s_w)[n])) * acc
            yr = sum(Fraction(float(X[m, k])) * Fraction(float(W[n, k])) for k in range(8))
            total += (yq - yr) ** 2
    assert cal.smoothing_loss(x, w, s) == pytest.approx(float(total), rel=1e-12)


def test_grid_search_picks_a_threshold_below_the_outliers_and_lowers_the_loss():
    x, w = layer(96, 128, 32, 6, outliers=(7, 77), scale=60.0)
    res = cal.adaptive_smoothing(x, w, 16)
    assert res["losses"][-1] == pytest.approx(cal.smoothing_loss(x, w, np.ones(128, np.float32)), rel=1e-12)
    assert res["best"] < 15 and res["losses"][res["best"]] < 0.7 * res["losses"][-1]
    assert res["selected"][7] and res["selected"][77]
    assert res["best"] == int(np.argmin(res["losses"]))
    xs, ws = cal.apply_smoothing(x, w, res["s"])
    assert np.array_equal(xs, res["xs"]) and np.array_equal(ws, res["ws"])


# ------------------------------------------------------------------ Hessian-based compensation

def test_hessian_definition():
    x, _ = layer(20, 12, 4, 7)
    X = x.view(np.float16).astype(np.float64)
    H = cal.hessian(x)
    brute = np.array([[2.0 * sum(X[m, i] * X[m, j] for m in range(20)) for j in range(12)] for i in range(12)])
    assert np.allclose(H, brute, rtol=1e-13) and np.array_equal(H, H.T)


def test_two_channel_closed_form():
    """K = 2: after channel 0 is quantised, Eq. 4 moves channel 1 by (w0 - q0) * H01 / H11
    (H^-1_01 / H^-1_00 = -H01 / H11), exactly."""
    w = f16bits([[0.30, -0.11], [-0.07, 0.21], [0.05, 0.02]])
    H = np.array([[4.0, 1.5], [1.5, 3.0]])
    codes, s_bits, _ = cal.gptq_quantize(w, H, percdamp=0.0)
    W = w.view(np.float16).astype(np.float64)
    s = s_bits.view(np.float16).astype(np.float64)
    for n in range(3):
        q0 = float(cal.rtn_codes(W[n, 0], s[n]))
        assert codes[n, 0] == q0
        w1 = Fraction(float(W[n, 1])) + (Fraction(float(W[n, 0])) - Fraction(q0) * Fraction(float(s[n]))) * Fraction(3, 2) / 3
        assert codes[n, 1] == float(cal.rtn_codes(float(w1), s[n]))


def exact_inverse(Hf):
    """Inverse of a small matrix of Fractions by Gauss-Jordan elimination."""
    n = len(Hf)
    A = [list(r) + [Fraction(int(i == j)) for j in range(n)] for i, r in enumerate(Hf)]
    for c in range(n):
        p = next(r for r in range(c, n) if A[r][c] != 0)
        A[c], A[p] = A[p], A[c]
        A[c] = [v / A[c][c] for v in A[c]]
        for r in range(n):
            if r != c and A[r][c] != 0:
                A[r] = [a - A[r][c] * b for a, b in zip(A[r], A[c])]
    return [r[n:] for r in A]


def test_eq4_in_exact_rationals_on_tiny_layers():
    """Every step re-derived from the definition: H_F is the Hessian restricted to the channels not yet
    quantised, inverted exactly each time (no elimination formula), delta_F by Eq. 4."""
    g = synth.rng(8)
    for K, N in ((3, 2), (5, 3)):
        x = f16bits(g.standard_normal((3 * K, K)))
        w = f16bits(g.standard_normal((N, K)) * 0.1)
        H = cal.hessian(x)
        codes, s_bits, _ = cal.gptq_quantize(w, H, percdamp=0.0)
        Hf = [[Fraction(float(H[i, j])) for j in range(K)] for i in range(K)]
        s = s_bits.view(np.float16).astype(np.float64)
        for n in range(N):
            wr = [Fraction(float(v)) for v in w.view(np.float16)[n]]
            for i in range(K):
                F = list(range(i, K))
                inv = exact_inverse([[Hf[a][b] for b in F] for a in F])
                q = float(cal.rtn_codes(float(wr[i]), s[n]))
                assert codes[n, i] == q, (K, n, i)
                e = (wr[i] - Fraction(q) * Fraction(float(s[n]))) / inv[0][0]
                for pos, j in enumerate(F):
                    if j > i:
                        wr[j] -= e * inv[pos][0]


def test_diagonal_hessian_is_plain_round_to_nearest():
    _, w = layer(4, 64, 16, 9)
    H = np.diag(np.linspace(1.0, 5.0, 64))
    codes, s_bits, _ = cal.gptq_quantize(w, H, percdamp=0.0)
    w_nat, s_w = orc.quantize_w4_perchannel(w)
    assert np.array_equal(s_bits, s_w)
    assert np.array_equal(cal.codes_to_w_nat(codes), w_nat)
    assert np.array_equal(orc.w8_perchannel(cal.codes_to_w_nat(codes), 64), codes)


def test_cholesky_formulation_gives_the_same_codes():
    """Independent route: with U the upper Cholesky factor of H^-1, row i of U is
    (H_F^-1)[i, i:] / sqrt([H_F^-1]_ii), so the update is W[:, i:] -= ((w - q) / U_ii) U[i, i:]."""
    x, w = layer(200, 48, 12, 10, outliers=(3,), scale=8.0)
    H = cal.hessian(x)
    codes, s_bits, _ = cal.gptq_quantize(w, H, percdamp=0.01)
    Hd = H.copy()
    Hd[np.arange(48), np.arange(48)] += 0.01 * np.mean(np.diag(H))
    U = np.linalg.cholesky(np.linalg.inv(Hd)).T
    W = w.view(np.float16).astype(np.float64).copy()
    s = s_bits.view(np.float16).astype(np.float64)
    alt = np.zeros_like(codes)
    for i in range(48):
        q = cal.rtn_codes(W[:, i], s)
        alt[:, i] = q
        e = (W[:, i] - q * s) / U[i, i]
        W[:, i:] -= np.outer(e, U[i, i:])
    assert np.array_equal(alt, codes)


def test_dead_channel_and_damping():
    x, w = layer(50, 16, 4, 11)
    xv = x.view(np.float16).copy()
    xv[:, 5] = 0
    H = cal.hessian(xv.view(np.uint16))
    assert H[5, 5] == 0
    codes, _, _ = cal.gptq_quantize(w, H, percdamp=0.01)
    assert np.all(codes[:, 5] == 0)


def test_compensation_beats_round_to_nearest_in_the_hessian_norm():
    g = synth.rng(12)
    base = g.standard_normal((400, 8))
    x = f16bits(base @ g.standard_normal((8, 96)) + 0.3 * g.standard_normal((400, 96)))   # correlated channels
    w = f16bits(g.standard_normal((24, 96)) * 0.05)
    H = cal.hessian(x)
    codes, s_bits, wq = cal.gptq_quantize(w, H, percdamp=0.01)
    W = w.view(np.float16).astype(np.float64)
    s = s_bits.view(np.float16).astype(np.float64)
    rtn = cal.rtn_codes(W, s[:, None]) * s[:, None]
    assert np.abs(codes).max() <= 7
    assert cal.hessian_error(W, wq, H) < 0.6 * cal.hessian_error(W, rtn, H)
    # the layer output itself: || X (W - Wq)^T ||^2 is what the Hessian norm measures
    X = x.view(np.float16).astype(np.float64)
    assert cal.hessian_error(W, wq, H) == pytest.approx(float(np.sum((X @ (W - wq).T) ** 2)), rel=1e-9)


# ------------------------------------------------------------------ per-group compensation

def test_pergroup_with_a_diagonal_hessian_is_the_front_end():
    """Nothing moves, so codes, group scales and everything derived from them must be what the (C) front-end
    oracle gives for the same weights: pins the sweep's scale rule and the derived scales at once."""
    _, w = layer(4, 256, 24, 21)
    wv = w.view(np.float16).copy()
    wv[3, 128:] = 0                      # a group of zeros: scale 0, codes 0
    wv[5, :] = 0                         # a channel of zeros: s_Wc 0, fused scale 0, integer form 1
    w = wv.view(np.uint16)
    H = np.diag(np.linspace(1.0, 3.0, 256))
    codes, s_wg, _ = cal.gptq_quantize_pergroup(w, H, 128, percdamp=0.0)
    star, s_int, s_wc = cal.pergroup_scales_from_codes(codes, s_wg, 128)
    f_nat, f_wg, f_star, f_int, f_wc = orc.quantize_w4_pergroup(w, 128)
    assert np.array_equal(cal.codes_to_w_nat(codes), f_nat)
    assert np.array_equal(s_wg, f_wg) and np.array_equal(star, f_star)
    assert np.array_equal(s_int, f_int) and np.array_equal(s_wc, f_wc)


def test_pergroup_with_one_group_is_the_per_channel_sweep():
    x, w = layer(300, 128, 10, 22, outliers=(7,), scale=6.0)
    H = cal.hessian(x)
    c_pc, s_pc, wq_pc = cal.gptq_quantize(w, H, percdamp=0.01)
    c_pg, s_wg, wq_pg = cal.gptq_quantize_pergroup(w, H, 128, percdamp=0.01)
    assert np.array_equal(c_pc, c_pg) and np.array_equal(s_pc, s_wg[0]) and np.array_equal(wq_pc, wq_pg)


def test_pergroup_eq4_in_exact_rationals_on_a_tiny_layer():
    """Groups of two channels; H_F inverted exactly at every step; the group scale re-derived from the exactly
    compensated weights when the sweep enters the group."""
    g = synth.rng(23)
    K, N, group = 6, 3, 2
    x = f16bits(g.standard_normal((3 * K, K)))
    w = f16bits(g.standard_normal((N, K)) * 0.1)
    H = cal.hessian(x)
    codes, s_wg, _ = cal.gptq_quantize_pergroup(w, H, group, percdamp=0.0)
    Hf = [[Fraction(float(H[i, j])) for j in range(K)] for i in range(K)]
    for n in range(N):
        wr = [Fraction(float(v)) for v in w.view(np.float16)[n]]
        s = None
        for i in range(K):
            if i % group == 0:
                amax = max(abs(v) for v in wr[i:i + group])
                bits = (np.float32(float(amax)) / np.float32(7.0)).astype(np.float16).view(np.uint16)
                assert bits == s_wg[i // group, n], (n, i)
                s = float(bits.view(np.float16))
            F = list(range(i, K))
            inv = exact_inverse([[Hf[a][b] for b in F] for a in F])
            q = float(cal.rtn_codes(float(wr[i]), s))
            assert codes[n, i] == q, (n, i)
            e = (wr[i] - Fraction(q) * Fraction(s)) / inv[0][0]
            for pos, j in enumerate(F):
                if j > i:
                    wr[j] -= e * inv[pos][0]


def test_pergroup_compensation_beats_group_wise_round_to_nearest():
    g = synth.rng(24)
    base = g.standard_normal((600, 12))
    x = f16bits(base @ g.standard_normal((12, 256)) + 0.3 * g.standard_normal((600, 256)))
    w = f16bits(g.standard_normal((16, 256)) * 0.05)
    H = cal.hessian(x)
    codes, s_wg, wq = cal.gptq_quantize_pergroup(w, H, 128, percdamp=0.01)
    W = w.view(np.float16).astype(np.float64)
    f_nat, f_wg, _, _, _ = orc.quantize_w4_pergroup(w, 128)
    rtn = orc.w8_perchannel(f_nat, 256).astype(np.float64) * np.repeat(f_wg.view(np.float16).astype(np.float64).T, 128, axis=1)
    assert np.abs(codes).max() <= 7
    assert cal.hessian_error(W, wq, H) < 0.6 * cal.hessian_error(W, rtn, H)
