"""CPU-only checks of the C-ABI boundary: the library loads, exports every function that
the headers under include/ declare, and rejects bad arguments on the host before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", h) for h in ("qqq.h", "qqq_tuning.h", "qqq_calib.h")]


@pytest.fixture(scope="module")
def L():
    from paper_2406_09904_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2406_09904_amd import build
        build.build()
    return binding.lib()


def declared_functions():
    names = set()
    for h in HEADERS:
        src = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(qqq_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_product_header_carries_no_knobs():
    src = re.sub(r"/\*.*?\*/", "", open(HEADERS[0]).read(), flags=re.S)
    assert "qqq_set_" not in src and "qqq_debug_" not in src and "qqq_last_route" not in src


def test_header_functions_are_exported(L):
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), n
    from paper_2406_09904_amd import binding
    assert sorted(binding.SYMBOLS) == names


def test_size_queries(L):
    assert L.qqq_packed_w4_bytes(4096, 4096) == 4096 * 4096 // 2
    assert L.qqq_packed_w4_bytes(4096, 4100) == 0          # K % 128
    assert L.qqq_packed_w4_bytes(4100, 4096) == 0          # N % 16
    assert L.qqq_packed_w4_bytes(16, 131072 + 128) == 0    # K beyond the int32-safe limit
    ws = L.qqq_gemm_workspace_bytes(16, 4096, 4096)
    assert ws >= 16 * 4096 * 4 + 4096 // 16 * 4
    assert L.qqq_gemm_workspace_bytes(1, 4097, 4096) == 0
    # linear workspace = GEMM workspace + fp32 token scales + int8 activations (256-byte aligned parts)
    lw = L.qqq_linear_workspace_bytes(16, 4096, 4096)
    assert lw >= ws + 16 * 4 + 16 * 4096 and lw <= ws + 16 * 4 + 16 * 4096 + 512
    assert L.qqq_linear_workspace_bytes(1, 4096, 4097) == 0
    assert L.qqq_version() >= 100


def test_host_side_argument_errors(L):
    bad = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails validation first
    assert L.qqq_quant_act(None, 4, 128, 128, None, None, None) == 1
    assert L.qqq_quant_act(bad, 4, 100, 128, bad, bad, None) == 2      # K % 8
    assert L.qqq_quant_act(bad, 4, 128, 64, bad, bad, None) == 2       # lda < K
    assert L.qqq_quant_act(bad, 0, 128, 128, bad, bad, None) == 0      # M == 0: no-op
    assert L.qqq_pack_w4(None, 16, 128, None, None) == 1
    assert L.qqq_pack_w4(bad, 17, 128, bad, None) == 2
    assert L.qqq_pack_w4(bad, 16, 128, bad, None) == 2                 # in place
    a = (bad, bad, bad, bad, bad, None)
    assert L.qqq_gemm_w4a8_perchannel(*a, 4, 100, 128, bad, 1 << 20, None) == 2
    assert L.qqq_gemm_w4a8_perchannel(*a, 4, 128, 200, bad, 1 << 20, None) == 2
    assert L.qqq_gemm_w4a8_perchannel(None, bad, bad, bad, bad, None, 4, 128, 128, bad, 1 << 20, None) == 1
    assert L.qqq_gemm_w4a8_perchannel(*a, 4, 128, 128, bad, 16, None) == 3    # workspace too small
    assert L.qqq_gemm_w4a8_perchannel(*a, 4, 128, 128, None, 0, None) == 1    # split-K needs one
    assert L.qqq_gemm_w4a8_perchannel(ctypes.c_void_p(0x1001), bad, bad, bad, bad, None, 4, 128, 128,
                                      bad, 1 << 20, None) == 2                # misaligned
    assert L.qqq_gemm_w4a8_perchannel(*a, 0, 128, 128, None, 0, None) == 0    # M == 0
    g = (bad, bad, bad, bad, bad)
    assert L.qqq_gemm_w4a8_pergroup(*g, 64, 0, bad, None, 4, 128, 128, bad, 1 << 20, None) == 2
    assert L.qqq_gemm_w4a8_pergroup(*g, 128, 200, bad, None, 4, 128, 128, bad, 1 << 20, None) == 2
    assert L.qqq_gemm_w4a8_pergroup(bad, bad, bad, None, bad, 128, 0, bad, None, 4, 128, 128, bad,
                                    1 << 20, None) == 1
    assert L.qqq_gemm_w4a8_pergroup(*g, 128, 0x200, bad, None, 4, 128, 128, bad, 1 << 20, None) == 2
    assert L.qqq_gemm_w4a8_pergroup(*g, 128, 0x100 | 128, bad, None, 4, 128, 128, bad, 1 << 20, None) == 2
    assert b"workspace" in L.qqq_last_error() or len(L.qqq_last_error()) > 0
    # real-valued fp16 group scales: same validation
    assert L.qqq_gemm_w4a8_pergroup_f16scale(*g, 64, bad, None, 4, 128, 128, bad, 1 << 20, None) == 2
    assert L.qqq_gemm_w4a8_pergroup_f16scale(bad, bad, bad, None, bad, 128, bad, None, 4, 128, 128, bad,
                                             1 << 20, None) == 1
    assert L.qqq_gemm_w4a8_pergroup_f16scale(bad, bad, bad, ctypes.c_void_p(0x1002), bad, 128, bad, None,
                                             4, 128, 128, bad, 1 << 20, None) == 2     # misaligned scales
    # one-call linear layer: fp16 rows in, same validation order (shape, null, alignment, workspace)
    lin = (bad, bad, bad, None)                       # w_packed, s_w, y, acc_out
    assert L.qqq_linear_w4a8_perchannel(bad, 128, *lin, 4, 100, 128, bad, 1 << 20, None) == 2
    assert L.qqq_linear_w4a8_perchannel(bad, 64, *lin, 4, 128, 128, bad, 1 << 20, None) == 2   # lda < K
    assert L.qqq_linear_w4a8_perchannel(bad, 132, *lin, 4, 128, 128, bad, 1 << 20, None) == 2  # lda % 8
    assert L.qqq_linear_w4a8_perchannel(None, 128, *lin, 4, 128, 128, bad, 1 << 20, None) == 1
    assert L.qqq_linear_w4a8_perchannel(bad, 128, *lin, 4, 128, 128, None, 0, None) == 1
    assert L.qqq_linear_w4a8_perchannel(bad, 128, *lin, 4, 128, 128, bad, 16, None) == 3
    assert L.qqq_linear_w4a8_perchannel(bad, 128, *lin, 0, 128, 128, None, 0, None) == 0       # M == 0
    assert L.qqq_linear_w4a8_pergroup(bad, 128, bad, bad, bad, 64, 0, bad, None, 4, 128, 128, bad,
                                      1 << 20, None) == 2                                      # group
    assert L.qqq_linear_w4a8_pergroup(bad, 128, bad, bad, bad, 128, 128, bad, None, 4, 128, 128, bad,
                                      1 << 20, None) == 2                                      # sg_max
    # errors of the GEMM half are found before the quantiser is enqueued (two-kernel route, M*K > 8192):
    # without a GPU a launch attempt would come back as error 4, the validation says 1 / 2
    assert L.qqq_linear_w4a8_perchannel(bad, 256, None, bad, bad, None, 64, 128, 256, bad, 1 << 24, None) == 1
    assert L.qqq_linear_w4a8_perchannel(bad, 256, bad, bad, ctypes.c_void_p(0x1004), None, 64, 128, 256, bad,
                                        1 << 24, None) == 2
    assert L.qqq_linear_w4a8_pergroup(bad, 256, bad, None, bad, 128, 15, bad, None, 64, 128, 256, bad,
                                      1 << 24, None) == 1
    # diagnostics
    assert L.qqq_debug_count_sg_violations(None, 128, 128, 15, bad, None) == 1
    assert L.qqq_debug_count_sg_violations(bad, 130, 128, 15, bad, None) == 2
    assert isinstance(L.qqq_last_route(), bytes)
    # offline stage
    assert L.qqq_smoothing_workspace_bytes(64, 128, 256) > 64 * 128 * 4
    assert L.qqq_smoothing_workspace_bytes(64, 100, 256) == 0
    assert L.qqq_adaptive_smoothing(bad, bad, 64, 128, 200, 8, bad, bad, bad, bad, bad, bad, bad, 1 << 30, None) == 2
    assert L.qqq_adaptive_smoothing(bad, bad, 64, 128, 256, 0, bad, bad, bad, bad, bad, bad, bad, 1 << 30, None) == 2
    assert L.qqq_adaptive_smoothing(None, bad, 64, 128, 256, 8, bad, bad, bad, bad, bad, bad, bad, 1 << 30, None) == 1
    assert L.qqq_adaptive_smoothing(bad, bad, 64, 128, 256, 8, bad, bad, bad, bad, bad, bad, bad, 16, None) == 3
    assert L.qqq_channel_absmax(bad, 4, 100, bad, None) == 2
    assert L.qqq_smooth_apply(bad, bad, bad, None, 4, 4, 128, bad, bad, bad, None) == 1
    assert L.qqq_fp16_gemm_nt(bad, bad, 4, 4, 24, bad, None) == 2
    assert L.qqq_hessian(bad, 4, 20000, bad, None) == 2
    assert L.qqq_gptq_workspace_bytes(64, 256) >= 256 * 256 * 8 + 64 * 256 * 8
    assert L.qqq_gptq_quantize_w4_perchannel(bad, bad, 64, 256, ctypes.c_double(-1.0), bad, bad, bad, 1 << 30, None) == 2
    assert L.qqq_gptq_quantize_w4_perchannel(bad, None, 64, 256, ctypes.c_double(0.01), bad, bad, bad, 1 << 30, None) == 1
    assert L.qqq_gptq_quantize_w4_perchannel(bad, bad, 64, 256, ctypes.c_double(0.01), bad, bad, bad, 64, None) == 3
    # the entry point on the library's static scratch: same order, plus its size limit; nothing
    # below gets as far as asking the runtime for the scratch address
    st = (bad, bad, bad, None)
    assert L.qqq_linear_w4a8_perchannel_static(bad, 128, *st, 4, 100, 128, None) == 2
    assert L.qqq_linear_w4a8_perchannel_static(bad, 8192, *st, 4096, 28672, 8192, None) == 3
    assert b"static scratch" in L.qqq_last_error()
    assert L.qqq_linear_w4a8_perchannel_static(bad, 64, *st, 4, 128, 128, None) == 2            # lda < K
    assert L.qqq_linear_w4a8_perchannel_static(None, 128, *st, 4, 128, 128, None) == 1
    assert L.qqq_linear_w4a8_perchannel_static(ctypes.c_void_p(0x1008), 128, *st, 4, 128, 128, None) == 2
    assert L.qqq_linear_w4a8_perchannel_static(bad, 128, *st, 0, 128, 128, None) == 0           # M == 0


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2406_09904_amd import binding
    with pytest.raises(ValueError):
        binding.qqq_quant_act(torch.zeros((2, 128), dtype=torch.float16))
