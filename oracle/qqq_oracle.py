"""ctypes front end of the CPU oracle (``qqq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  It never imports the HIP package and the HIP package
never imports it.  Inputs and outputs are numpy arrays; all arithmetic happens in the C
file, which follows Sec. 3.3 / 3.3.1 / 3.3.2 / 4.1 of the QQQ paper (arXiv 2406.09904).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qqq_oracle.c")
# QQQ_ORACLE_SANITIZE=<directory>: a separate build under gcc's address and undefined-behaviour
# sanitizers, written to that directory (the process must then run with libasan preloaded;
# tests/test_sanitizers.py does that in a child process)
_SANITIZE = os.environ.get("QQQ_ORACLE_SANITIZE", "")
_LIB = os.path.join(_SANITIZE, "libqqq_oracle_san.so") if _SANITIZE else os.path.join(_HERE, "libqqq_oracle.so")
_lock = threading.Lock()
_lib = None

ORC_OK, ORC_NULL, ORC_SHAPE, ORC_OVERFLOW = 0, 1, 2, 5


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp); returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if _SANITIZE else ["-O2"]
        subprocess.check_call(
            ["gcc", *opt, "-fopenmp", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _p(arr, ctype):
    return None if arr is None else arr.ctypes.data_as(ctypes.POINTER(ctype))


def lib():
    global _lib
    with _lock:
        if _lib is None:
            L = ctypes.CDLL(build())
            i64 = ctypes.c_int64
            pu16 = ctypes.POINTER(ctypes.c_uint16)
            pu32 = ctypes.POINTER(ctypes.c_uint32)
            pi8 = ctypes.POINTER(ctypes.c_int8)
            pi32 = ctypes.POINTER(ctypes.c_int32)
            pi64 = ctypes.POINTER(ctypes.c_int64)
            pf32 = ctypes.POINTER(ctypes.c_float)
            L.qqq_oracle_half_to_float_array.argtypes = [pu16, i64, pf32]
            L.qqq_oracle_half_to_float_array.restype = None
            L.qqq_oracle_float_to_half_array.argtypes = [pf32, i64, pu16]
            L.qqq_oracle_float_to_half_array.restype = None
            L.qqq_oracle_quant_act.argtypes = [pu16, i64, i64, i64, pi8, pf32]
            L.qqq_oracle_w8_perchannel.argtypes = [pu32, i64, i64, pi8]
            L.qqq_oracle_w8_pergroup.argtypes = [pu32, pi8, i64, i64, i64, pi8]
            L.qqq_oracle_int8_gemm.argtypes = [pi8, pi8, i64, i64, i64, pi64]
            L.qqq_oracle_dequant.argtypes = [pi64, pf32, pu16, i64, i64, pf32, pu16]
            L.qqq_oracle_gemm_perchannel.argtypes = [pi8, pf32, pu32, pu16, i64, i64, i64,
                                                     pi32, pf32, pu16]
            L.qqq_oracle_gemm_pergroup.argtypes = [pi8, pf32, pu32, pi8, pu16, i64, i64, i64, i64,
                                                   pi32, pf32, pu16]
            L.qqq_oracle_gemm_samples.argtypes = [pi8, pf32, pu32, pi8, pu16, i64, i64, i64, i64,
                                                  pi64, pi64, i64, pi64, pu16]
            L.qqq_oracle_double_to_half.argtypes = [ctypes.c_double]
            L.qqq_oracle_double_to_half.restype = ctypes.c_uint16
            L.qqq_oracle_w8_f16scale_one.argtypes = [ctypes.c_int, ctypes.c_uint16]
            L.qqq_oracle_w8_f16scale_one.restype = ctypes.c_int8
            L.qqq_oracle_w8_pergroup_f16.argtypes = [pu32, pu16, i64, i64, i64, pi8]
            L.qqq_oracle_gemm_pergroup_f16.argtypes = [pi8, pf32, pu32, pu16, pu16, i64, i64, i64,
                                                       i64, pi32, pf32, pu16]
            L.qqq_oracle_quantize_w4_perchannel.argtypes = [pu16, i64, i64, i64, pu32, pu16]
            L.qqq_oracle_quantize_w4_pergroup.argtypes = [pu16, i64, i64, i64, i64, pu32, pu16, pu16,
                                                          pi8, pu16]
            L.qqq_oracle_gemm_samples_f16.argtypes = [pi8, pf32, pu32, pu16, pu16, i64, i64, i64, i64,
                                                      pi64, pi64, i64, pi64, pu16]
            _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle returned status %d" % code)
        self.code = code


def _check(rc):
    if rc != ORC_OK:
        raise OracleError(rc)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def half_to_float(bits):
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    lib().qqq_oracle_half_to_float_array(_p(bits, ctypes.c_uint16), bits.size, _p(out, ctypes.c_float))
    return out


def float_to_half(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().qqq_oracle_float_to_half_array(_p(x, ctypes.c_float), x.size, _p(out, ctypes.c_uint16))
    return out


def quant_act(a_fp16_bits):
    """a_fp16_bits: uint16 [M,K] (bit patterns of fp16) -> (a_q int8 [M,K], s_a float32 [M])."""
    a = _c(a_fp16_bits, np.uint16)
    M, K = a.shape
    a_q = np.empty((M, K), np.int8)
    s_a = np.empty((M,), np.float32)
    _check(lib().qqq_oracle_quant_act(_p(a, ctypes.c_uint16), M, K, K, _p(a_q, ctypes.c_int8),
                                      _p(s_a, ctypes.c_float)))
    return a_q, s_a


def w8_perchannel(w_nat, K):
    w = _c(w_nat, np.uint32)
    N = w.shape[0]
    out = np.empty((N, K), np.int8)
    _check(lib().qqq_oracle_w8_perchannel(_p(w, ctypes.c_uint32), N, K, _p(out, ctypes.c_int8)))
    return out


def w8_pergroup(w_nat, s_g, K, group=128):
    w = _c(w_nat, np.uint32)
    g = _c(s_g, np.int8)
    N = w.shape[0]
    out = np.empty((N, K), np.int8)
    _check(lib().qqq_oracle_w8_pergroup(_p(w, ctypes.c_uint32), _p(g, ctypes.c_int8), N, K, group,
                                        _p(out, ctypes.c_int8)))
    return out


def int8_gemm(a_q, w8):
    a = _c(a_q, np.int8)
    w = _c(w8, np.int8)
    M, K = a.shape
    N = w.shape[0]
    acc = np.empty((M, N), np.int64)
    _check(lib().qqq_oracle_int8_gemm(_p(a, ctypes.c_int8), _p(w, ctypes.c_int8), M, N, K,
                                      _p(acc, ctypes.c_int64)))
    return acc


def dequant(acc, s_a, s_w_fp16_bits):
    acc = _c(acc, np.int64)
    s_a = _c(s_a, np.float32)
    s_w = _c(s_w_fp16_bits, np.uint16)
    M, N = acc.shape
    y32 = np.empty((M, N), np.float32)
    y16 = np.empty((M, N), np.uint16)
    _check(lib().qqq_oracle_dequant(_p(acc, ctypes.c_int64), _p(s_a, ctypes.c_float),
                                    _p(s_w, ctypes.c_uint16), M, N, _p(y32, ctypes.c_float),
                                    _p(y16, ctypes.c_uint16)))
    return y32, y16


def gemm_perchannel(a_q, s_a, w_nat, s_w_fp16_bits, want_y=True):
    """-> (acc int32 [M,N], y32 float32 [M,N], y fp16 bits uint16 [M,N])."""
    a = _c(a_q, np.int8)
    s_a = _c(s_a, np.float32)
    w = _c(w_nat, np.uint32)
    s_w = _c(s_w_fp16_bits, np.uint16)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] * 8 == K and s_w.shape == (N,) and s_a.shape == (M,)
    acc = np.empty((M, N), np.int32)
    y32 = np.empty((M, N), np.float32) if want_y else None
    y16 = np.empty((M, N), np.uint16) if want_y else None
    _check(lib().qqq_oracle_gemm_perchannel(_p(a, ctypes.c_int8), _p(s_a, ctypes.c_float),
                                            _p(w, ctypes.c_uint32), _p(s_w, ctypes.c_uint16),
                                            M, N, K, _p(acc, ctypes.c_int32),
                                            _p(y32, ctypes.c_float), _p(y16, ctypes.c_uint16)))
    return acc, y32, y16


def gemm_pergroup(a_q, s_a, w_nat, s_g, s_w_fp16_bits, group=128, want_y=True):
    a = _c(a_q, np.int8)
    s_a = _c(s_a, np.float32)
    w = _c(w_nat, np.uint32)
    g = _c(s_g, np.int8)
    s_w = _c(s_w_fp16_bits, np.uint16)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] * 8 == K and s_w.shape == (N,) and s_a.shape == (M,)
    assert g.shape == (K // group, N)
    acc = np.empty((M, N), np.int32)
    y32 = np.empty((M, N), np.float32) if want_y else None
    y16 = np.empty((M, N), np.uint16) if want_y else None
    _check(lib().qqq_oracle_gemm_pergroup(_p(a, ctypes.c_int8), _p(s_a, ctypes.c_float),
                                          _p(w, ctypes.c_uint32), _p(g, ctypes.c_int8),
                                          _p(s_w, ctypes.c_uint16), group, M, N, K,
                                          _p(acc, ctypes.c_int32), _p(y32, ctypes.c_float),
                                          _p(y16, ctypes.c_uint16)))
    return acc, y32, y16


def double_to_half(x: float) -> int:
    """fp16 bit pattern of a double, round to nearest even (the oracle's own conversion)."""
    return int(lib().qqq_oracle_double_to_half(float(x)))


def w8_f16scale_one(code: int, s_bits: int) -> int:
    """One weight of the real-valued per-group path (Sec. 3.3.2): int8 from code and fp16 scale bits."""
    return int(lib().qqq_oracle_w8_f16scale_one(int(code), int(s_bits)))


def w8_pergroup_f16(w_nat, s_g_fp16_bits, K, group=128):
    w = _c(w_nat, np.uint32)
    g = _c(s_g_fp16_bits, np.uint16)
    N = w.shape[0]
    assert w.shape[1] * 8 == K and g.shape == (K // group, N)
    out = np.empty((N, K), np.int8)
    _check(lib().qqq_oracle_w8_pergroup_f16(_p(w, ctypes.c_uint32), _p(g, ctypes.c_uint16), N, K,
                                            group, _p(out, ctypes.c_int8)))
    return out


def gemm_pergroup_f16(a_q, s_a, w_nat, s_g_fp16_bits, s_w_fp16_bits, group=128, want_y=True):
    """Per-group GEMM with the paper's real-valued fp16 fused scale -> (acc, y32, y fp16 bits)."""
    a = _c(a_q, np.int8)
    s_a = _c(s_a, np.float32)
    w = _c(w_nat, np.uint32)
    g = _c(s_g_fp16_bits, np.uint16)
    s_w = _c(s_w_fp16_bits, np.uint16)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] * 8 == K and s_w.shape == (N,) and s_a.shape == (M,)
    assert g.shape == (K // group, N)
    acc = np.empty((M, N), np.int32)
    y32 = np.empty((M, N), np.float32) if want_y else None
    y16 = np.empty((M, N), np.uint16) if want_y else None
    _check(lib().qqq_oracle_gemm_pergroup_f16(_p(a, ctypes.c_int8), _p(s_a, ctypes.c_float),
                                              _p(w, ctypes.c_uint32), _p(g, ctypes.c_uint16),
                                              _p(s_w, ctypes.c_uint16), group, M, N, K,
                                              _p(acc, ctypes.c_int32), _p(y32, ctypes.c_float),
                                              _p(y16, ctypes.c_uint16)))
    return acc, y32, y16


def gemm_samples(a_q, s_a, w_nat, s_g, s_w_fp16_bits, idx_m, idx_n, group=128):
    """Selected outputs one by one; s_g=None selects per-channel. -> (acc int64 [S], y fp16 bits [S])."""
    a = _c(a_q, np.int8)
    s_a = _c(s_a, np.float32)
    w = _c(w_nat, np.uint32)
    g = None if s_g is None else _c(s_g, np.int8)
    s_w = _c(s_w_fp16_bits, np.uint16)
    im = _c(idx_m, np.int64)
    jn = _c(idx_n, np.int64)
    M, K = a.shape
    N = w.shape[0]
    acc = np.empty(im.shape, np.int64)
    y16 = np.empty(im.shape, np.uint16)
    _check(lib().qqq_oracle_gemm_samples(_p(a, ctypes.c_int8), _p(s_a, ctypes.c_float),
                                         _p(w, ctypes.c_uint32), _p(g, ctypes.c_int8),
                                         _p(s_w, ctypes.c_uint16), group, M, N, K,
                                         _p(im, ctypes.c_int64), _p(jn, ctypes.c_int64), im.size,
                                         _p(acc, ctypes.c_int64), _p(y16, ctypes.c_uint16)))
    return acc, y16


def gemm_samples_f16(a_q, s_a, w_nat, s_g_fp16_bits, s_w_fp16_bits, idx_m, idx_n, group=128):
    """Selected outputs of the real-valued per-group variant. -> (acc int64 [S], y fp16 bits [S])."""
    a = _c(a_q, np.int8)
    s_a = _c(s_a, np.float32)
    w = _c(w_nat, np.uint32)
    g = _c(s_g_fp16_bits, np.uint16)
    s_w = _c(s_w_fp16_bits, np.uint16)
    im = _c(idx_m, np.int64)
    jn = _c(idx_n, np.int64)
    M, K = a.shape
    N = w.shape[0]
    acc = np.empty(im.shape, np.int64)
    y16 = np.empty(im.shape, np.uint16)
    _check(lib().qqq_oracle_gemm_samples_f16(_p(a, ctypes.c_int8), _p(s_a, ctypes.c_float),
                                             _p(w, ctypes.c_uint32), _p(g, ctypes.c_uint16),
                                             _p(s_w, ctypes.c_uint16), group, M, N, K,
                                             _p(im, ctypes.c_int64), _p(jn, ctypes.c_int64), im.size,
                                             _p(acc, ctypes.c_int64), _p(y16, ctypes.c_uint16)))
    return acc, y16


def quantize_w4_perchannel(w_fp16_bits):
    """Offline front-end, per-channel (Sec. 3.3.1): fp16 bits [N,K] -> (w_nat [N,K/8], s_w fp16 bits [N])."""
    w = _c(w_fp16_bits, np.uint16)
    N, K = w.shape
    w_nat = np.zeros((N, K // 8), np.uint32)
    s_w = np.empty(N, np.uint16)
    _check(lib().qqq_oracle_quantize_w4_perchannel(_p(w, ctypes.c_uint16), N, K, K,
                                                   _p(w_nat, ctypes.c_uint32), _p(s_w, ctypes.c_uint16)))
    return w_nat, s_w


def quantize_w4_pergroup(w_fp16_bits, group=128):
    """Offline front-end, per-group (Sec. 3.3.2, Fig. 5): fp16 bits [N,K] ->
    (w_nat, s_Wg fp16 bits [G,N], s*_Wg fp16 bits [G,N], integer s* int8 [G,N], s_Wc fp16 bits [N])."""
    w = _c(w_fp16_bits, np.uint16)
    N, K = w.shape
    G = K // group
    w_nat = np.zeros((N, K // 8), np.uint32)
    s_wg = np.empty((G, N), np.uint16)
    s_star = np.empty((G, N), np.uint16)
    s_int = np.empty((G, N), np.int8)
    s_wc = np.empty(N, np.uint16)
    _check(lib().qqq_oracle_quantize_w4_pergroup(_p(w, ctypes.c_uint16), N, K, K, group,
                                                 _p(w_nat, ctypes.c_uint32), _p(s_wg, ctypes.c_uint16),
                                                 _p(s_star, ctypes.c_uint16), _p(s_int, ctypes.c_int8),
                                                 _p(s_wc, ctypes.c_uint16)))
    return w_nat, s_wg, s_star, s_int, s_wc
