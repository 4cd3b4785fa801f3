"""Thin ctypes binding over libqqq.so (the C ABI declared in include/qqq.h; tuning and
diagnostic controls in include/qqq_tuning.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch
supplies device memory and the stream.  There is no CPU fallback: if the library is missing or a
tensor is not on the GPU the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# QQQ_LIB_PATH: load another build of the same library (the host-sanitizer build of the CPU tests)
LIB_PATH = os.environ.get("QQQ_LIB_PATH") or os.path.join(_HERE, "libqqq.so")
GROUP = 128
SG_SYMMETRIC_CODES = 0x100   # QQQ_SG_SYMMETRIC_CODES of include/qqq.h, or-ed into sg_max

SYMBOLS = [
    "qqq_version", "qqq_last_error", "qqq_quant_act", "qqq_packed_w4_bytes", "qqq_pack_w4",
    "qqq_unpack_w4", "qqq_gemm_workspace_bytes", "qqq_gemm_w4a8_perchannel",
    "qqq_gemm_w4a8_pergroup", "qqq_gemm_w4a8_pergroup_f16scale", "qqq_linear_workspace_bytes", "qqq_linear_w4a8_perchannel",
    "qqq_linear_w4a8_pergroup", "qqq_set_fused_quant", "qqq_set_kernel_override",
    "qqq_set_group_mode_override", "qqq_set_skinny_tuning", "qqq_set_prefill_tuning",
    "qqq_quantize_w4_perchannel", "qqq_quantize_w4_pergroup", "qqq_set_prefill_ksplit",
    "qqq_gemm_workspace_zero_bytes", "qqq_linear_w4a8_perchannel_static", "qqq_last_route",
    "qqq_debug_count_sg_violations", "qqq_probe_stream_read", "qqq_probe_mfma_i8", "qqq_probe_prefill_loop",
    "qqq_smoothing_workspace_bytes", "qqq_adaptive_smoothing", "qqq_channel_absmax", "qqq_smooth_apply",
    "qqq_fp16_gemm_nt", "qqq_hessian", "qqq_gptq_workspace_bytes", "qqq_gptq_quantize_w4_perchannel",
    "qqq_gptq_quantize_w4_pergroup",
]

_lib = None


class QQQError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libqqq error %d: %s" % (code, msg))
        self.code = code


def lib():
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libqqq.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(or python paper_2406_09904_amd/build.py) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
        L.qqq_version.restype = ci
        L.qqq_last_error.restype = ctypes.c_char_p
        L.qqq_last_route.restype = ctypes.c_char_p
        L.qqq_debug_count_sg_violations.argtypes = [vp, i64, i64, ci, vp, vp]
        L.qqq_smoothing_workspace_bytes.argtypes = [i64, i64, i64]
        L.qqq_smoothing_workspace_bytes.restype = sz
        L.qqq_adaptive_smoothing.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.qqq_channel_absmax.argtypes = [vp, i64, i64, vp, vp]
        L.qqq_smooth_apply.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, vp]
        L.qqq_fp16_gemm_nt.argtypes = [vp, vp, i64, i64, i64, vp, vp]
        L.qqq_hessian.argtypes = [vp, i64, i64, vp, vp]
        L.qqq_gptq_workspace_bytes.argtypes = [i64, i64]
        L.qqq_gptq_workspace_bytes.restype = sz
        L.qqq_gptq_quantize_w4_perchannel.argtypes = [vp, vp, i64, i64, ctypes.c_double, vp, vp, vp, sz, vp]
        L.qqq_gptq_quantize_w4_pergroup.argtypes = [vp, vp, i64, i64, ci, ctypes.c_double, vp, vp, vp, vp, vp, vp, sz, vp]
        L.qqq_probe_stream_read.argtypes = [vp, sz, ci, vp, vp]
        L.qqq_probe_mfma_i8.argtypes = [vp, vp, ci, ci, vp, vp]
        L.qqq_probe_prefill_loop.argtypes = [vp, sz, ci, ci, ci, vp, vp]
        L.qqq_quant_act.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        L.qqq_packed_w4_bytes.argtypes = [i64, i64]
        L.qqq_packed_w4_bytes.restype = sz
        L.qqq_pack_w4.argtypes = [vp, i64, i64, vp, vp]
        L.qqq_unpack_w4.argtypes = [vp, i64, i64, vp, vp]
        L.qqq_gemm_workspace_bytes.argtypes = [i64, i64, i64]
        L.qqq_gemm_workspace_bytes.restype = sz
        L.qqq_gemm_workspace_zero_bytes.argtypes = [i64, i64, i64]
        L.qqq_gemm_workspace_zero_bytes.restype = sz
        L.qqq_gemm_w4a8_perchannel.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, sz, vp]
        L.qqq_gemm_w4a8_pergroup.argtypes = [vp, vp, vp, vp, vp, ci, ci, vp, vp, i64, i64, i64,
                                             vp, sz, vp]
        L.qqq_gemm_w4a8_pergroup_f16scale.argtypes = [vp, vp, vp, vp, vp, ci, vp, vp, i64, i64, i64,
                                                      vp, sz, vp]
        L.qqq_linear_workspace_bytes.argtypes = [i64, i64, i64]
        L.qqq_linear_workspace_bytes.restype = sz
        L.qqq_linear_w4a8_perchannel.argtypes = [vp, i64, vp, vp, vp, vp, i64, i64, i64, vp, sz, vp]
        L.qqq_linear_w4a8_pergroup.argtypes = [vp, i64, vp, vp, vp, ci, ci, vp, vp, i64, i64, i64,
                                               vp, sz, vp]
        L.qqq_linear_w4a8_perchannel_static.argtypes = [vp, i64, vp, vp, vp, vp, i64, i64, i64, vp]
        L.qqq_quantize_w4_perchannel.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        L.qqq_quantize_w4_pergroup.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp, vp, vp, vp]
        L.qqq_set_fused_quant.argtypes = [ci]
        L.qqq_set_kernel_override.argtypes = [ci]
        L.qqq_set_group_mode_override.argtypes = [ci]
        L.qqq_set_skinny_tuning.argtypes = [ci, ci, ci, ci]
        L.qqq_set_prefill_tuning.argtypes = [ci]
        L.qqq_set_prefill_ksplit.argtypes = [ci]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise QQQError(rc, lib().qqq_last_error().decode())


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libqqq takes device tensors only")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected %s, got %s" % (dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def qqq_quant_act(a_fp16: torch.Tensor, a_q: torch.Tensor = None, s_a: torch.Tensor = None):
    """a_fp16 [M,K] fp16 (row stride allowed) -> (a_q int8 [M,K], s_a fp32 [M])."""
    if a_fp16.dtype != torch.float16 or a_fp16.dim() != 2 or a_fp16.stride(1) != 1:
        raise ValueError("a_fp16 must be a 2-D fp16 tensor with unit inner stride")
    M, K = a_fp16.shape
    lda = a_fp16.stride(0) if M > 1 else max(K, a_fp16.stride(0))
    if a_q is None:
        a_q = torch.empty((M, K), dtype=torch.int8, device=a_fp16.device)
    if s_a is None:
        s_a = torch.empty((M,), dtype=torch.float32, device=a_fp16.device)
    if not a_fp16.is_cuda:
        raise ValueError("libqqq takes device tensors only")
    _check(lib().qqq_quant_act(ctypes.c_void_p(a_fp16.data_ptr()), M, K, lda,
                               _ptr(a_q, torch.int8), _ptr(s_a, torch.float32), _stream()))
    return a_q, s_a


def _weights_arg(w_fp16):
    if w_fp16.dtype != torch.float16 or w_fp16.dim() != 2 or w_fp16.stride(1) != 1 or not w_fp16.is_cuda:
        raise ValueError("w_fp16 must be a 2-D fp16 device tensor with unit inner stride")
    N, K = w_fp16.shape
    return N, K, (w_fp16.stride(0) if N > 1 else max(K, w_fp16.stride(0)))


def qqq_quantize_w4_perchannel(w_fp16: torch.Tensor, out=None):
    """fp16 weights [N,K] -> (w_nat int32 [N,K/8] natural nibble words, s_w fp16 [N]); out = a
    previous result to write into."""
    N, K, ldw = _weights_arg(w_fp16)
    if out is not None:
        w_nat, s_w = out
    else:
        w_nat = torch.empty((N, K // 8), dtype=torch.int32, device=w_fp16.device)
        s_w = torch.empty((N,), dtype=torch.float16, device=w_fp16.device)
    _check(lib().qqq_quantize_w4_perchannel(ctypes.c_void_p(w_fp16.data_ptr()), N, K, ldw,
                                            _ptr(w_nat, torch.int32), _ptr(s_w, torch.float16), _stream()))
    return w_nat, s_w


def qqq_quantize_w4_pergroup(w_fp16: torch.Tensor, group: int = 128, want_int: bool = True,
                             want_wg: bool = True, out=None):
    """fp16 weights [N,K] -> (w_nat, s_star fp16 [K/128,N], s_int int8 [K/128,N] or None, s_wc fp16 [N],
    s_wg fp16 [K/128,N] or None); out = a previous result to write into."""
    N, K, ldw = _weights_arg(w_fp16)
    dev = w_fp16.device
    G = K // group if group > 0 else 0
    if out is not None:
        w_nat, s_star, s_int, s_wc, s_wg = out
    else:
        w_nat = torch.empty((N, K // 8), dtype=torch.int32, device=dev)
        s_star = torch.empty((G, N), dtype=torch.float16, device=dev)
        s_int = torch.empty((G, N), dtype=torch.int8, device=dev) if want_int else None
        s_wg = torch.empty((G, N), dtype=torch.float16, device=dev) if want_wg else None
        s_wc = torch.empty((N,), dtype=torch.float16, device=dev)
    _check(lib().qqq_quantize_w4_pergroup(ctypes.c_void_p(w_fp16.data_ptr()), N, K, ldw, group,
                                          _ptr(w_nat, torch.int32), _ptr(s_star, torch.float16),
                                          _ptr(s_int, torch.int8), _ptr(s_wc, torch.float16),
                                          _ptr(s_wg, torch.float16), _stream()))
    return w_nat, s_star, s_int, s_wc, s_wg


def qqq_packed_w4_bytes(N: int, K: int) -> int:
    return int(lib().qqq_packed_w4_bytes(N, K))


def qqq_pack_w4(w_nat: torch.Tensor, K: int, out: torch.Tensor = None) -> torch.Tensor:
    """w_nat [N,K/8] int32 (bit pattern of the uint32 natural words) -> opaque packed uint8 [N*K/2]."""
    N = w_nat.shape[0]
    nbytes = qqq_packed_w4_bytes(N, K)
    if nbytes == 0 or w_nat.shape[1] * 8 != K:
        raise QQQError(2, "pack: unsupported N=%d K=%d" % (N, K))
    if out is None:
        out = torch.empty((nbytes,), dtype=torch.uint8, device=w_nat.device)
    _check(lib().qqq_pack_w4(_ptr(w_nat, torch.int32), N, K, _ptr(out, torch.uint8), _stream()))
    return out


def qqq_unpack_w4(w_packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K // 8), dtype=torch.int32, device=w_packed.device)
    _check(lib().qqq_unpack_w4(_ptr(w_packed, torch.uint8), N, K, _ptr(out, torch.int32), _stream()))
    return out


def qqq_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().qqq_gemm_workspace_bytes(M, N, K))


def split_k_part(workspace: torch.Tensor, M: int, N: int, K: int) -> torch.Tensor:
    """The part of a GEMM workspace that every call leaves zero (arrival counters and split-K partial
    sums of the decode kernel); what follows it is scratch of the prefill kernels with no invariant."""
    return workspace[:int(lib().qqq_gemm_workspace_zero_bytes(M, N, K))]


def new_workspace(M: int, N: int, K: int, device="cuda") -> torch.Tensor:
    """Zero-filled workspace (zeroed once here; every GEMM call leaves it zero)."""
    return torch.zeros((max(qqq_gemm_workspace_bytes(M, N, K), 16),), dtype=torch.uint8, device=device)


def qqq_gemm_w4a8_perchannel(a_q, s_a, w_packed, s_w, workspace, y=None, acc_out=None, N=None):
    M, K = a_q.shape
    N = s_w.shape[0] if N is None else N
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=a_q.device)
    _check(lib().qqq_gemm_w4a8_perchannel(
        _ptr(a_q, torch.int8), _ptr(s_a, torch.float32), _ptr(w_packed, torch.uint8),
        _ptr(s_w, torch.float16), _ptr(y, torch.float16), _ptr(acc_out, torch.int32), M, N, K,
        _ptr(workspace, torch.uint8), workspace.numel(), _stream()))
    return y


def qqq_gemm_w4a8_pergroup(a_q, s_a, w_packed, s_g, s_w, workspace, sg_max=0, y=None, acc_out=None,
                           group=GROUP):
    M, K = a_q.shape
    N = s_w.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=a_q.device)
    _check(lib().qqq_gemm_w4a8_pergroup(
        _ptr(a_q, torch.int8), _ptr(s_a, torch.float32), _ptr(w_packed, torch.uint8),
        _ptr(s_g, torch.int8), _ptr(s_w, torch.float16), group, sg_max, _ptr(y, torch.float16),
        _ptr(acc_out, torch.int32), M, N, K, _ptr(workspace, torch.uint8), workspace.numel(),
        _stream()))
    return y


def qqq_gemm_w4a8_pergroup_f16scale(a_q, s_a, w_packed, s_g_fp16, s_w, workspace, y=None,
                                    acc_out=None, group=GROUP):
    """Per-group GEMM with the real-valued fp16 fused scale s*_Wg [K/128, N] (no saturation)."""
    M, K = a_q.shape
    N = s_w.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=a_q.device)
    _check(lib().qqq_gemm_w4a8_pergroup_f16scale(
        _ptr(a_q, torch.int8), _ptr(s_a, torch.float32), _ptr(w_packed, torch.uint8),
        _ptr(s_g_fp16, torch.float16), _ptr(s_w, torch.float16), group, _ptr(y, torch.float16),
        _ptr(acc_out, torch.int32), M, N, K, _ptr(workspace, torch.uint8), workspace.numel(),
        _stream()))
    return y


def qqq_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().qqq_linear_workspace_bytes(M, N, K))


def new_linear_workspace(M: int, N: int, K: int, device="cuda") -> torch.Tensor:
    """Zero-filled workspace for the qqq_linear_* calls (zeroed once here)."""
    return torch.zeros((max(qqq_linear_workspace_bytes(M, N, K), 16),), dtype=torch.uint8, device=device)


def _fp16_rows(a_fp16):
    if a_fp16.dtype != torch.float16 or a_fp16.dim() != 2 or a_fp16.stride(1) != 1:
        raise ValueError("a_fp16 must be a 2-D fp16 tensor with unit inner stride")
    if not a_fp16.is_cuda:
        raise ValueError("libqqq takes device tensors only")
    M, K = a_fp16.shape
    lda = a_fp16.stride(0) if M > 1 else max(K, a_fp16.stride(0))
    return M, K, lda


def qqq_linear_w4a8_perchannel(a_fp16, w_packed, s_w, workspace, y=None, acc_out=None):
    M, K, lda = _fp16_rows(a_fp16)
    N = s_w.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=a_fp16.device)
    _check(lib().qqq_linear_w4a8_perchannel(
        ctypes.c_void_p(a_fp16.data_ptr()), lda, _ptr(w_packed, torch.uint8), _ptr(s_w, torch.float16),
        _ptr(y, torch.float16), _ptr(acc_out, torch.int32), M, N, K, _ptr(workspace, torch.uint8),
        workspace.numel(), _stream()))
    return y


def qqq_linear_w4a8_perchannel_static(a_fp16, w_packed, s_w, y, acc_out=None):
    """qqq_linear_w4a8_perchannel on the library's static device scratch: no workspace, and the
    caller passes the output tensor too, so nothing is allocated on the way."""
    M, K, lda = _fp16_rows(a_fp16)
    N = s_w.shape[0]
    _check(lib().qqq_linear_w4a8_perchannel_static(
        ctypes.c_void_p(a_fp16.data_ptr()), lda, _ptr(w_packed, torch.uint8), _ptr(s_w, torch.float16),
        _ptr(y, torch.float16), _ptr(acc_out, torch.int32), M, N, K, _stream()))
    return y


def qqq_linear_w4a8_pergroup(a_fp16, w_packed, s_g, s_w, workspace, sg_max=0, y=None, acc_out=None,
                             group=GROUP):
    M, K, lda = _fp16_rows(a_fp16)
    N = s_w.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=a_fp16.device)
    _check(lib().qqq_linear_w4a8_pergroup(
        ctypes.c_void_p(a_fp16.data_ptr()), lda, _ptr(w_packed, torch.uint8), _ptr(s_g, torch.int8),
        _ptr(s_w, torch.float16), group, sg_max, _ptr(y, torch.float16), _ptr(acc_out, torch.int32),
        M, N, K, _ptr(workspace, torch.uint8), workspace.numel(), _stream()))
    return y


# ---- offline stage (include/qqq_calib.h): adaptive smoothing and Hessian-based compensation

def _fp16_matrix(t):
    if t.dtype != torch.float16 or t.dim() != 2 or not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous 2-D fp16 device tensor")
    return t.shape


def qqq_adaptive_smoothing(x_fp16, w_fp16, grid_points=20):
    """Sec. 3.1 on one layer: X [M,K], W [N,K] fp16 -> dict(xs, ws, s, sigmas, losses, best); best is a
    device tensor (no synchronisation here)."""
    (M, K), (N, K2) = _fp16_matrix(x_fp16), _fp16_matrix(w_fp16)
    if K != K2:
        raise ValueError("X and W disagree on K")
    dev = x_fp16.device
    xs, ws = torch.empty_like(x_fp16), torch.empty_like(w_fp16)
    s = torch.empty((K,), dtype=torch.float32, device=dev)
    sigmas = torch.empty((grid_points,), dtype=torch.float32, device=dev)
    losses = torch.empty((grid_points,), dtype=torch.float64, device=dev)
    best = torch.empty((1,), dtype=torch.int32, device=dev)
    nbytes = int(lib().qqq_smoothing_workspace_bytes(M, N, K))
    work = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=dev)
    _check(lib().qqq_adaptive_smoothing(_ptr(x_fp16), _ptr(w_fp16), M, N, K, grid_points, _ptr(xs), _ptr(ws),
                                        _ptr(s), _ptr(sigmas), _ptr(losses), _ptr(best), _ptr(work),
                                        work.numel(), _stream()))
    return {"xs": xs, "ws": ws, "s": s, "sigmas": sigmas, "losses": losses, "best": best}


def qqq_channel_absmax(x_fp16):
    M, K = _fp16_matrix(x_fp16)
    out = torch.empty((K,), dtype=torch.float32, device=x_fp16.device)
    _check(lib().qqq_channel_absmax(_ptr(x_fp16), M, K, _ptr(out), _stream()))
    return out


def qqq_smooth_apply(x_fp16, w_fp16, absmax, sigma):
    """sigma: 1-element fp32 device tensor.  -> (xs, ws, s)."""
    (M, K), (N, _) = _fp16_matrix(x_fp16), _fp16_matrix(w_fp16)
    xs, ws = torch.empty_like(x_fp16), torch.empty_like(w_fp16)
    s = torch.empty((K,), dtype=torch.float32, device=x_fp16.device)
    _check(lib().qqq_smooth_apply(_ptr(x_fp16), _ptr(w_fp16), _ptr(absmax, torch.float32), _ptr(sigma, torch.float32),
                                  M, N, K, _ptr(xs), _ptr(ws), _ptr(s), _stream()))
    return xs, ws, s


def qqq_fp16_gemm_nt(x_fp16, w_fp16):
    (M, K), (N, _) = _fp16_matrix(x_fp16), _fp16_matrix(w_fp16)
    y = torch.empty((M, N), dtype=torch.float32, device=x_fp16.device)
    _check(lib().qqq_fp16_gemm_nt(_ptr(x_fp16), _ptr(w_fp16), M, N, K, _ptr(y), _stream()))
    return y


def qqq_hessian(x_fp16):
    M, K = _fp16_matrix(x_fp16)
    H = torch.empty((K, K), dtype=torch.float64, device=x_fp16.device)
    _check(lib().qqq_hessian(_ptr(x_fp16), M, K, _ptr(H), _stream()))
    return H


def qqq_gptq_quantize_w4_perchannel(w_fp16, H, percdamp=0.01):
    """Sec. 3.2 on one layer: W [N,K] fp16, H [K,K] fp64 -> (w_nat int32 [N,K/8], s_w fp16 [N])."""
    N, K = _fp16_matrix(w_fp16)
    dev = w_fp16.device
    w_nat = torch.empty((N, K // 8), dtype=torch.int32, device=dev)
    s_w = torch.empty((N,), dtype=torch.float16, device=dev)
    nbytes = int(lib().qqq_gptq_workspace_bytes(N, K))
    work = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=dev)
    _check(lib().qqq_gptq_quantize_w4_perchannel(_ptr(w_fp16), _ptr(H, torch.float64), N, K, float(percdamp),
                                                 _ptr(w_nat, torch.int32), _ptr(s_w, torch.float16), _ptr(work),
                                                 work.numel(), _stream()))
    return w_nat, s_w


def qqq_gptq_quantize_w4_pergroup(w_fp16, H, percdamp=0.01, want_int=True):
    """Sec. 3.2 with the group-128 quantiser of Sec. 3.3.2 on one layer: W [N,K] fp16, H [K,K] fp64 ->
    (w_nat int32 [N,K/8], s_wg fp16 [K/128,N], s_star fp16 [K/128,N], s_int int8 [K/128,N] or None, s_wc fp16 [N])."""
    N, K = _fp16_matrix(w_fp16)
    dev = w_fp16.device
    G = K // GROUP
    w_nat = torch.empty((N, K // 8), dtype=torch.int32, device=dev)
    s_wg = torch.empty((G, N), dtype=torch.float16, device=dev)
    s_star = torch.empty((G, N), dtype=torch.float16, device=dev)
    s_int = torch.empty((G, N), dtype=torch.int8, device=dev) if want_int else None
    s_wc = torch.empty((N,), dtype=torch.float16, device=dev)
    nbytes = int(lib().qqq_gptq_workspace_bytes(N, K))
    work = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=dev)
    _check(lib().qqq_gptq_quantize_w4_pergroup(_ptr(w_fp16), _ptr(H, torch.float64), N, K, GROUP, float(percdamp),
                                               _ptr(w_nat, torch.int32), _ptr(s_wg, torch.float16),
                                               _ptr(s_star, torch.float16), _ptr(s_int, torch.int8),
                                               _ptr(s_wc, torch.float16), _ptr(work), work.numel(), _stream()))
    return w_nat, s_wg, s_star, s_int, s_wc


def last_route() -> str:
    """The kernels the most recent GEMM / linear call of this thread enqueued (include/qqq_tuning.h)."""
    return lib().qqq_last_route().decode()


def count_sg_violations(s_g: torch.Tensor, sg_max: int) -> int:
    """Entries of the integer group-scale table [K/128, N] outside 0..sg_max (diagnostic; synchronises)."""
    G, N = s_g.shape
    out = torch.empty((1,), dtype=torch.int32, device=s_g.device)
    _check(lib().qqq_debug_count_sg_violations(_ptr(s_g, torch.int8), N, G * GROUP, sg_max,
                                               _ptr(out, torch.int32), _stream()))
    return int(out.item())


def probe_stream_read(buf: torch.Tensor, nbytes: int, workgroups: int, sink: torch.Tensor, offset: int = 0):
    """One launch of the streaming-read ceiling probe over buf[offset : offset + nbytes] (uint8 tensor)."""
    _check(lib().qqq_probe_stream_read(ctypes.c_void_p(buf.data_ptr() + offset), nbytes, workgroups,
                                       _ptr(sink, torch.int32), _stream()))


def probe_mfma_i8(a_pool: torch.Tensor, b_pool: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor):
    """One launch of the int8 MFMA ceiling probe (a_pool 128 KiB, b_pool 32 KiB of int8 operand values)."""
    if a_pool.numel() != 4 * 4 * 512 * 16 or b_pool.numel() != 2 * 2 * 512 * 16:
        raise ValueError("operand pools must hold 4*4*512 and 2*2*512 16-byte values")
    _check(lib().qqq_probe_mfma_i8(_ptr(a_pool, torch.int8), _ptr(b_pool, torch.int8), iters, workgroups,
                                   _ptr(sink, torch.int32), _stream()))


PROBE_A_READS, PROBE_W_READS, PROBE_CONVERT, PROBE_DMA, PROBE_FORM_32X32X32 = 1, 2, 4, 8, 16
PROBE_LOOP_STAGE = 51200


def probe_prefill_loop(src: torch.Tensor, region_bytes: int, steps: int, parts: int, workgroups: int,
                       sink: torch.Tensor):
    """One launch of the prefill k-loop probe: src is a uint8 tensor of workgroups * region_bytes bytes."""
    if src.numel() < workgroups * region_bytes:
        raise ValueError("src must hold workgroups * region_bytes bytes")
    _check(lib().qqq_probe_prefill_loop(_ptr(src, torch.uint8), region_bytes, steps, parts, workgroups,
                                        _ptr(sink, torch.int32), _stream()))


def set_fused_quant(enable: int) -> int:
    return lib().qqq_set_fused_quant(enable)


def set_kernel_override(family: int) -> int:
    return lib().qqq_set_kernel_override(family)


def set_group_mode_override(mode: int) -> int:
    return lib().qqq_set_group_mode_override(mode)


def set_skinny_tuning(channel_tiles: int, k_slices: int, waves: int = 0, depth: int = 0) -> int:
    return lib().qqq_set_skinny_tuning(channel_tiles, k_slices, waves, depth)


def set_prefill_tuning(waves: int) -> int:
    return lib().qqq_set_prefill_tuning(waves)



def set_prefill_ksplit(k_splits: int) -> int:
    """Diagnostic: K splits of the per-tile prefill kernel for 64 < M <= 512 (0 = automatic)."""
    return lib().qqq_set_prefill_ksplit(k_splits)
