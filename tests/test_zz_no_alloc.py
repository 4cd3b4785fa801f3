"""GPU test of the entry point that allocates nothing (qqq_linear_w4a8_perchannel_static: the
library's static device scratch instead of a caller workspace), called through the C ABI.

Its output must equal that of qqq_linear_w4a8_perchannel bit for bit (int32 accumulators and fp16
outputs), and both must meet the oracle's bar (accumulators exact, fp16 within 1 ulp).  Calls in a
row share the scratch array and each keeps the previous call's contents: the sequence below goes
from a prefill shape that fills the array with quantised activations, pre-pass scratch and K-split
slabs to smaller decode shapes whose zero-on-entry part lies where that scratch was.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import binding as qqq
from paper_2406_09904_amd import synth
from tests.util import f16_bits, to_dev, ulp_distance

pytestmark = pytest.mark.gpu

# (M, K, N): the first is the largest input; the later ones are smaller inputs with a LARGER
# zero-on-entry part (more channels), then a few-row fused decode call, then the first shape again
SEQUENCE = [(192, 2048, 256), (16, 4096, 4096), (3, 1024, 512), (40, 512, 1024), (192, 2048, 256)]


def _inputs(M, K, N, seed):
    wl = synth.Workload("noalloc", "perchannel", M, K, N, seed=seed)
    return wl.activations(), wl.w_nat(), wl.s_w()


def test_static_scratch_matches_workspace_call_and_oracle():
    L = qqq.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for step, (M, K, N) in enumerate(SEQUENCE):
        print("no-alloc step %d: M=%d K=%d N=%d" % (step, M, K, N), flush=True)
        a, w_nat, s_w = _inputs(M, K, N, 4100 + step)
        d_a = to_dev(a.view(np.uint16), torch)
        d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
        d_sw = to_dev(s_w.view(np.uint16), torch)
        # reference: the existing entry point with a caller workspace
        ws = qqq.new_linear_workspace(M, N, K)
        acc_ref = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y_ref = qqq.qqq_linear_w4a8_perchannel(d_a, d_w, d_sw, ws, acc_out=acc_ref)
        # the static-scratch entry point, straight through the C ABI: plain pointers and sizes
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        acc = torch.full((M, N), -12345, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        rc = L.qqq_linear_w4a8_perchannel_static(
            ctypes.c_void_p(d_a.data_ptr()), K, ctypes.c_void_p(d_w.data_ptr()),
            ctypes.c_void_p(d_sw.data_ptr()), ctypes.c_void_p(y.data_ptr()),
            ctypes.c_void_p(acc.data_ptr()), M, N, K, stream)
        assert rc == 0, L.qqq_last_error().decode()
        torch.cuda.synchronize()
        assert torch.equal(acc, acc_ref), "step %d: accumulators differ from the workspace call" % step
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), "step %d: outputs differ" % step
        o_q, o_sa = orc.quant_act(a.view(np.uint16))
        o_acc, _, o_y = orc.gemm_perchannel(o_q, o_sa, w_nat, s_w.view(np.uint16))
        assert np.array_equal(acc.cpu().numpy(), o_acc), "step %d: accumulators differ from the oracle" % step
        assert ulp_distance(f16_bits(y), o_y).max() <= 1, "step %d: fp16 outputs off by more than 1 ulp" % step


def test_static_scratch_rejects_oversize_and_bad_arguments():
    L = qqq.lib()
    d = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    p = ctypes.c_void_p(d.data_ptr())
    need = L.qqq_linear_workspace_bytes(4096, 28672, 8192)
    assert need > (16 << 20)
    # beyond the static maximum: an error, nothing enqueued, the buffers are never touched
    assert L.qqq_linear_w4a8_perchannel_static(p, 8192, p, p, p, None, 4096, 28672, 8192, None) == 3
    assert b"static scratch" in L.qqq_last_error()
    assert L.qqq_linear_w4a8_perchannel_static(p, 1024, p, p, p, None, 4, 100, 1024, None) == 2
    assert L.qqq_linear_w4a8_perchannel_static(None, 1024, p, p, p, None, 4, 128, 1024, None) == 1
    assert L.qqq_linear_w4a8_perchannel_static(p, 1000, p, p, p, None, 4, 128, 1024, None) == 2
    assert L.qqq_linear_w4a8_perchannel_static(p, 1024, p, p, p, None, 0, 128, 1024, None) == 0
    torch.cuda.synchronize()
