"""Pure-Python brute force of the path's definitions, for TINY shapes only.

Independent of ``oracle/qqq_oracle.c``: Python ints (unbounded), ``fractions.Fraction`` for
the exact quotient in the activation quantiser, explicit loops.  Used to pin the oracle.
Follows Sec. 4.1 (per-token symmetric quantisation), Sec. 3.3.1 (per-channel) and
Sec. 3.3.2 (per-group) of the QQQ paper.
"""
from fractions import Fraction

import numpy as np


def nibble_code(w_nat, n, k):
    word = int(w_nat[n][k // 8])
    nib = (word >> (4 * (k % 8))) & 0xF
    return nib - 16 if nib >= 8 else nib


def round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def to_f32_exact(fr: Fraction) -> Fraction:
    """Correctly rounded (nearest-even) binary32 value of a positive or negative rational,
    as an exact Fraction (normal range only, which is all these tests reach)."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = 0
    while a >= 2:
        a /= 2
        e += 1
    while a < 1:
        a *= 2
        e -= 1
    assert -126 <= e <= 127
    m = round_half_even(a * (1 << 23))  # 24-bit significand
    return sign * Fraction(m, 1 << 23) * (Fraction(2) ** e)


def quant_act(a_fp16):
    """a_fp16: numpy float16 [M,K] -> (list of lists of ints, list of exact Fractions s_a)."""
    M, K = a_fp16.shape
    q, s = [], []
    for m in range(M):
        row = [Fraction(float(a_fp16[m, k])) for k in range(K)]
        amax = max(abs(v) for v in row)
        if amax == 0:
            q.append([0] * K)
            s.append(Fraction(0))
            continue
        sa = to_f32_exact(amax / 127)
        out = []
        for v in row:
            t = to_f32_exact(v / sa)            # fp32 quotient, correctly rounded
            r = round_half_even(t)
            out.append(max(-127, min(127, r)))
        q.append(out)
        s.append(sa)
    return q, s


def w8(w_nat, N, K, s_g=None, group=128):
    out = []
    for n in range(N):
        row = []
        for k in range(K):
            c = nibble_code(w_nat, n, k)
            if s_g is not None:
                c = max(-128, min(127, c * int(s_g[k // group][n])))
            row.append(c)
        out.append(row)
    return out


def acc(a_q, w8_rows):
    M, N, K = len(a_q), len(w8_rows), len(w8_rows[0])
    return [[sum(int(a_q[m][k]) * int(w8_rows[n][k]) for k in range(K)) for n in range(N)]
            for m in range(M)]


def dequant_fp16_bits(acc_val: int, s_a: float, s_w_fp16) -> int:
    """numpy route: float64 product -> float32 -> float16 bits (library conversions)."""
    y = np.float64(acc_val) * np.float64(np.float32(s_a)) * np.float64(np.float16(s_w_fp16))
    return int(np.float32(y).astype(np.float16).view(np.uint16))
