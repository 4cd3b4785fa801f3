"""CPU oracle for QQQ's offline stage on one layer: adaptive smoothing (Sec. 3.1, Eq. 1-2) and
Hessian-based quantisation compensation (Sec. 3.2, Eq. 3-4) of arXiv 2406.09904.

TEST INFRASTRUCTURE ONLY, like ``qqq_oracle``: plain numpy in float64, no blocking, no fusion,
each function a direct statement of what the paper's passage computes.  It never imports the HIP
package.  The quantisers Q(.) inside the loss of Eq. 2 are the oracle's own (``qqq_oracle``):
per-token int8 for activations (Sec. 4.1), symmetric per-channel int4 for weights (Sec. 3.3.1).

Readings taken where the paper is silent, ambiguous or at odds with itself:

* Eq. 1 prints ``max|X[:,t]| < sigma`` for the selected set while the sentence before it says that
  the channels whose outliers EXCEED the threshold are the ones smoothed.  The sentence (and the
  purpose: smooth only the channels with significant outliers) is taken: T = { t : max|X[:,t]| > sigma }.
* The paper does not say how the smoothing vector s of Eq. 2 is searched.  Reading (the way the
  outlier-suppression work it builds on does it): s is a function of the threshold,
  s_t = max|X[:,t]| / sigma for t in T (the channel is scaled down to the threshold) and 1 elsewhere,
  and the grid search over sigma in (0, max|X|] picks the sigma whose s minimises the loss of Eq. 2,
  evaluated over the whole product (channels outside T enter with s = 1).  Grid: sigma_g =
  max|X| * g / G for g = 1..G; g = G selects no channel, i.e. "no smoothing" is always a candidate.
  Ties go to the smallest g.
* Arithmetic of the smoothed tensors (they decide integer codes later, so it is pinned):
  s_t = fp32(max|X[:,t]|) / fp32(sigma) (one fp32 division), X' = fp16_rne(fp32(X) / s) and
  W' = fp16_rne(fp32(W) * s) (one fp32 operation each, then one rounding to fp16).
* Loss of Eq. 2: || s_a[m] s_w[n] acc[m,n] - (X W^T)[m,n] ||^2 summed over the layer output, with acc the
  exact integer product of the codes of X' and W', evaluated in float64.
* Sec. 3.2 gives Eq. 3 (which weight to quantise next) and Eq. 4 (how the remaining weights F move).
  Reading: the method it adopts processes the input channels in their natural order i = 0..K-1 for
  all output channels at once instead of the greedy choice of Eq. 3, so Eq. 3 fixes nothing here;
  Eq. 4 is applied literally with H_F^-1 the inverse Hessian of the channels not yet quantised,
  obtained from the previous one by eliminating channel i.  H = 2 X^T X over the calibration tokens,
  damped by `percdamp` times its mean diagonal; an input channel that never fires (H_ii = 0) gets
  H_ii = 1 and weight 0.  Q(.) is the per-channel quantiser of the front-end: scale
  fp16_rne(fp32(max_k |W[n,k]|) / 7) from the ORIGINAL weights, code = clamp(rne(fp32(w / s)), -7, 7)
  (w is a float64 running value here; its quotient by the stored scale is rounded to fp32 first, which
  makes the rule coincide with the front-end's on weights that were never moved).
* Per-group weights (Sec. 3.3.2 uses group 128 along the input channels; Sec. 3.2 does not say when a
  group's scale is fixed while Eq. 4 keeps moving the weights).  Reading: when the sweep reaches the
  first input channel of a group, the group's scale is taken from the weights as they stand then,
  compensated by everything quantised before: s_Wg[g,n] = fp16_rne(fp32(max_{k in g} |W[n,k]|) / 7); the
  channels of the group are quantised with it.  The per-channel scale s_Wc, the fused scale s*_Wg and
  its integer form then follow from the codes and s_Wg by the front-end's own rule.  With a diagonal
  Hessian nothing moves and all five outputs are the front-end's.

Pins (tests/test_oracle_calib.py): the K = 2 closed form and an exact-rational evaluation of Eq. 4
on tiny layers, diagonal Hessian = plain round-to-nearest, the Cholesky formulation as an
independent route, never worse than round-to-nearest in the Hessian norm on correlated inputs;
sigma = max|X| leaves the layer untouched, the smoothed real-valued product is unchanged, planted
outlier channels are the selected set and smoothing lowers the loss there, a brute-force loss on a
tiny layer in exact rationals.
"""
from __future__ import annotations

import numpy as np

from oracle import qqq_oracle as orc


def _f16(bits):
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16)


# ---------------------------------------------------------------- Sec. 3.1 adaptive smoothing

def channel_absmax(x_bits):
    """max over tokens of |X[m,t]| per input channel t, as float32 (exact: the values are fp16)."""
    return np.abs(_f16(x_bits).astype(np.float32)).max(axis=0)


def sigma_grid(absmax, grid_points):
    """Candidate thresholds of the grid search: sigma_g = max|X| * g / G, g = 1..G, as float32."""
    top = float(np.max(absmax))
    return np.array([np.float32(top * g / grid_points) for g in range(1, grid_points + 1)], np.float32)


def smoothing_vector(absmax, sigma):
    """Eq. 1 (as read above) and the smoothing vector it induces: s_t = max|X[:,t]| / sigma on the
    selected channels, 1 elsewhere.  float32, one fp32 division per selected channel."""
    absmax = np.asarray(absmax, np.float32)
    sigma = np.float32(sigma)
    s = np.ones_like(absmax)
    sel = absmax > sigma
    s[sel] = absmax[sel] / sigma
    return s, sel


def apply_smoothing(x_bits, w_bits, s):
    """X ./ s and W .* s (the operands of Q in Eq. 2) as fp16 bit patterns."""
    s = np.asarray(s, np.float32)
    xs = (_f16(x_bits).astype(np.float32) / s[None, :]).astype(np.float16)
    ws = (_f16(w_bits).astype(np.float32) * s[None, :]).astype(np.float16)
    return xs.view(np.uint16), ws.view(np.uint16)


def quantised_product(x_bits, w_bits):
    """Q(X) Q(W)^T of Eq. 2 for fp16 operands: per-token int8 codes and scale (Sec. 4.1), per-channel
    int4 codes and scale (Sec. 3.3.1), the exact integer product, dequantised in float64."""
    a_q, s_a = orc.quant_act(x_bits)
    w_nat, s_w = orc.quantize_w4_perchannel(w_bits)
    acc, _, _ = orc.gemm_perchannel(a_q, s_a, w_nat, s_w, want_y=False)
    return acc.astype(np.float64) * s_a.astype(np.float64)[:, None] * orc.half_to_float(s_w).astype(np.float64)[None, :]


def reference_product(x_bits, w_bits):
    return _f16(x_bits).astype(np.float64) @ _f16(w_bits).astype(np.float64).T


def smoothing_loss(x_bits, w_bits, s, y_ref=None):
    """Eq. 2 for one smoothing vector: || Q(X ./ s) Q(W .* s)^T - X W^T ||^2 (float64)."""
    xs, ws = apply_smoothing(x_bits, w_bits, s)
    if y_ref is None:
        y_ref = reference_product(x_bits, w_bits)
    d = quantised_product(xs, ws) - y_ref
    return float(np.sum(d * d))


def adaptive_smoothing(x_bits, w_bits, grid_points):
    """The grid search of Sec. 3.1.  Returns dict(absmax, sigmas, losses, best, sigma, s, selected,
    xs, ws) with xs/ws the smoothed layer for the winning threshold."""
    absmax = channel_absmax(x_bits)
    sigmas = sigma_grid(absmax, grid_points)
    y_ref = reference_product(x_bits, w_bits)
    losses = np.empty(grid_points, np.float64)
    for g, sigma in enumerate(sigmas):
        s, _ = smoothing_vector(absmax, sigma)
        losses[g] = smoothing_loss(x_bits, w_bits, s, y_ref)
    best = int(np.argmin(losses))                      # first minimum
    s, sel = smoothing_vector(absmax, sigmas[best])
    xs, ws = apply_smoothing(x_bits, w_bits, s)
    return {"absmax": absmax, "sigmas": sigmas, "losses": losses, "best": best, "sigma": sigmas[best],
            "s": s, "selected": sel, "xs": xs, "ws": ws}


# ---------------------------------------------------------------- Sec. 3.2 Hessian-based compensation

def hessian(x_bits):
    """H = 2 X^T X over the calibration tokens (float64)."""
    x = _f16(x_bits).astype(np.float64)
    return 2.0 * (x.T @ x)


def channel_scales(w_bits):
    """The front-end's per-channel scale: fp16_rne(fp32(max_k |W[n,k]|) / 7), as fp16 bits."""
    amax = np.abs(_f16(w_bits).astype(np.float32)).max(axis=1)
    return (amax / np.float32(7.0)).astype(np.float16).view(np.uint16)


def rtn_codes(w, s):
    """code = clamp(rne(fp32(w / s)), -7, 7): the quotient of the float64 running weight and the stored
    scale is rounded to fp32 before the integer rounding, as the front-end does for its fp16
    weights; a zero scale gives code 0."""
    w = np.asarray(w, np.float64)
    s = np.asarray(s, np.float64)
    safe = np.where(s == 0.0, 1.0, s)
    q = np.clip(np.rint((w / safe).astype(np.float32).astype(np.float64)), -7.0, 7.0)
    return np.where(s == 0.0, 0.0, q)


def gptq_quantize(w_bits, H, percdamp=0.01):
    """Eq. 4 applied channel by channel.  w_bits: fp16 bits [N,K]; H [K,K].  Returns (codes int8 [N,K],
    s_w fp16 bits [N], W_q float64 [N,K] = codes * scale)."""
    W = _f16(w_bits).astype(np.float64).copy()
    N, K = W.shape
    H = np.array(H, np.float64, copy=True)
    s_bits = channel_scales(w_bits)
    s = _f16(s_bits).astype(np.float64)
    dead = np.diag(H) == 0.0
    H[dead, dead] = 1.0
    W[:, dead] = 0.0
    H[np.arange(K), np.arange(K)] += percdamp * np.mean(np.diag(H))
    Hinv = np.linalg.inv(H)                              # H_F^-1 for F = all channels
    codes = np.zeros((N, K), np.int8)
    for i in range(K):
        w = W[:, i]
        q = rtn_codes(w, s)
        codes[:, i] = q.astype(np.int8)
        d = Hinv[i, i]
        err = (w - q * s) / d                            # (W_i - Q(W_i)) / [H_F^-1]_ii
        W[:, i + 1:] -= np.outer(err, Hinv[i, i + 1:])   # delta_F of Eq. 4 on the channels still in F
        # channel i leaves F: the inverse Hessian of the smaller set by eliminating row/column i
        Hinv[i + 1:, i + 1:] -= np.outer(Hinv[i + 1:, i], Hinv[i, i + 1:]) / d
    return codes, s_bits, codes.astype(np.float64) * s[:, None]


def group_scales_now(W_group):
    """fp16_rne(fp32(max_k |W[n,k]|) / 7) over one group of the running float64 weights, as fp16 bits [N]."""
    amax = np.abs(np.asarray(W_group, np.float64)).max(axis=1).astype(np.float32)
    return (amax / np.float32(7.0)).astype(np.float16).view(np.uint16)


def gptq_quantize_pergroup(w_bits, H, group=128, percdamp=0.01):
    """Eq. 4 channel by channel with per-group scales fixed when the sweep enters the group.
    Returns (codes int8 [N,K], s_Wg fp16 bits [K/group, N], W_q float64 [N,K])."""
    W = _f16(w_bits).astype(np.float64).copy()
    N, K = W.shape
    assert K % group == 0
    H = np.array(H, np.float64, copy=True)
    dead = np.diag(H) == 0.0
    H[dead, dead] = 1.0
    W[:, dead] = 0.0
    H[np.arange(K), np.arange(K)] += percdamp * np.mean(np.diag(H))
    Hinv = np.linalg.inv(H)
    codes = np.zeros((N, K), np.int8)
    s_wg = np.zeros((K // group, N), np.uint16)
    W_q = np.zeros((N, K), np.float64)
    s = None
    for i in range(K):
        if i % group == 0:
            s_wg[i // group] = group_scales_now(W[:, i:i + group])
            s = _f16(s_wg[i // group]).astype(np.float64)
        w = W[:, i]
        q = rtn_codes(w, s)
        codes[:, i] = q.astype(np.int8)
        W_q[:, i] = q * s
        d = Hinv[i, i]
        err = (w - q * s) / d
        W[:, i + 1:] -= np.outer(err, Hinv[i, i + 1:])
        Hinv[i + 1:, i + 1:] -= np.outer(Hinv[i + 1:, i], Hinv[i, i + 1:]) / d
    return codes, s_wg, W_q


def pergroup_scales_from_codes(codes, s_wg_bits, group=128):
    """The front-end's rule (Sec. 3.3.2, Fig. 5 offline) for what follows the codes and group scales:
    s_Wc[n] = fp16_rne(fp32(max_k |code * s_Wg|) / 127) with the product in fp32; s*_Wg = fp16_rne(fp32(s_Wg / s_Wc)),
    capped at 18.203125 (0 where s_Wc is 0); integer form clamp(rne(s*_Wg), 1, 18).
    Returns (s*_Wg fp16 bits [G,N], integer s* int8 [G,N], s_Wc fp16 bits [N])."""
    codes = np.asarray(codes)
    N, K = codes.shape
    G = K // group
    sg = _f16(s_wg_bits).astype(np.float32)                        # [G, N]
    per_weight = np.repeat(sg.T, group, axis=1)                    # [N, K]
    dmax = np.abs(codes.astype(np.float32) * per_weight).max(axis=1)
    s_wc_bits = (dmax / np.float32(127.0)).astype(np.float16).view(np.uint16)
    s_wc = _f16(s_wc_bits).astype(np.float32)
    safe = np.where(s_wc == 0.0, np.float32(1.0), s_wc)
    star = (sg / safe[None, :]).astype(np.float16)
    star = np.where(star.astype(np.float32) > np.float32(18.203125), np.float16(18.203125), star)
    star = np.where(s_wc[None, :] == 0.0, np.float16(0.0), star).astype(np.float16)
    s_int = np.clip(np.rint(star.astype(np.float64)), 1.0, 18.0).astype(np.int8)
    return star.view(np.uint16), s_int, s_wc_bits


def codes_to_w_nat(codes):
    """int8 codes [N,K] -> natural nibble words uint32 [N,K/8] (nibble i of word j = code of k = 8j+i)."""
    c = (np.asarray(codes, np.int64) & 0xF).astype(np.uint32)
    N, K = c.shape
    c = c.reshape(N, K // 8, 8)
    out = np.zeros((N, K // 8), np.uint32)
    for i in range(8):
        out |= c[:, :, i] << np.uint32(4 * i)
    return out


def hessian_error(W_ref, W_q, H):
    """tr((W - W_q) H (W - W_q)^T) / 2 = || X (W - W_q)^T ||^2, the layer-output error that Eq. 3-4 minimise."""
    d = np.asarray(W_ref, np.float64) - np.asarray(W_q, np.float64)
    return float(0.5 * np.sum((d @ H) * d))
