"""GPU parity on the paper's own GEMM-study layer, N=8192, K=21760 (Sec. 4.4, the shape of Fig. 8),
for M in {1, 64, 128, 1024} and all three variants (per-channel, integer per-group, the paper's
real-valued fp16 per-group scale), with automatic kernel selection as bench.py --token-sweep times it.

The oracle's full product for M <= 128; for M = 1024 whole rows over all N columns (the first, the
last and one interior block of 64 rows plus 32 seeded random rows) and sampled entries elsewhere.
int32 accumulators bit-exact, fp16 outputs within 1 fp16 ulp.
"""
import functools

import numpy as np
import pytest
import torch

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import binding as qqq
from paper_2406_09904_amd import synth
from tests.util import f16_bits, ulp_distance

pytestmark = pytest.mark.gpu

N, K = 8192, 21760


@functools.lru_cache(maxsize=1)
def _layer():
    w_nat = synth.random_w_nat(N, K, 77)
    d_w = qqq.qqq_pack_w4(torch.from_numpy(w_nat.view(np.int32)).cuda(), K)
    s_w = synth.weight_scales_fp16(N, 78, 0.001, 0.005)
    sg_i = synth.group_scales(K, N, 79, 1, 15)
    sg_f = synth.group_scales_f16(K, N, 80)
    return w_nat, d_w, s_w, sg_i, sg_f


@pytest.mark.parametrize("M", [1, 64, 128, 1024])
@pytest.mark.parametrize("variant", ["perchannel", "pergroup", "pergroup_f16scale"])
def test_paper_gemm_study_shape(M, variant):
    w_nat, d_w, s_w, sg_i, sg_f = _layer()
    a = synth.activations_fp16(M, K, 81 + M)
    d_q, d_sa = qqq.qqq_quant_act(torch.from_numpy(a).cuda())
    d_sw = torch.from_numpy(s_w).cuda()
    ws = qqq.new_workspace(M, N, K)
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    if variant == "perchannel":
        y = qqq.qqq_gemm_w4a8_perchannel(d_q, d_sa, d_w, d_sw, ws, acc_out=acc)
    elif variant == "pergroup":
        y = qqq.qqq_gemm_w4a8_pergroup(d_q, d_sa, d_w, torch.from_numpy(sg_i).cuda(), d_sw, ws, sg_max=15,
                                       acc_out=acc)
    else:
        y = qqq.qqq_gemm_w4a8_pergroup_f16scale(d_q, d_sa, d_w, torch.from_numpy(sg_f).cuda(), d_sw, ws,
                                                acc_out=acc)
    torch.cuda.synchronize()
    assert not qqq.split_k_part(ws, M, N, K).any().item(), "workspace not returned to zero"

    o_q, o_sa = orc.quant_act(a.view(np.uint16))
    assert np.array_equal(d_q.cpu().numpy(), o_q) and np.array_equal(d_sa.cpu().numpy(), o_sa)
    g = synth.rng(900 + M)
    if M <= 128:
        rows = np.arange(M)
    else:
        mid = 64 * int(g.integers(1, M // 64 - 1))
        rows = np.unique(np.concatenate([np.arange(64), np.arange(mid, mid + 64), np.arange(M - 64, M),
                                         g.integers(0, M, 32)]))
    r_q, r_sa = np.ascontiguousarray(o_q[rows]), np.ascontiguousarray(o_sa[rows])
    sw_bits = s_w.view(np.uint16)
    if variant == "perchannel":
        f_acc, _, f_y = orc.gemm_perchannel(r_q, r_sa, w_nat, sw_bits)
    elif variant == "pergroup":
        f_acc, _, f_y = orc.gemm_pergroup(r_q, r_sa, w_nat, sg_i, sw_bits)
    else:
        f_acc, _, f_y = orc.gemm_pergroup_f16(r_q, r_sa, w_nat, sg_f.view(np.uint16), sw_bits)
    t_rows = torch.from_numpy(rows).cuda()
    assert np.array_equal(acc[t_rows].cpu().numpy(), f_acc), "int32 accumulators differ"
    assert ulp_distance(f16_bits(y[t_rows]), f_y).max() <= 1, "fp16 outputs differ by more than 1 ulp"
    assert np.abs(f_acc).max() > 0

    if M > 128:   # the rows the oracle did not take in full: sampled entries, one by one
        im, jn = g.integers(0, M, 3000), g.integers(0, N, 3000)
        if variant == "pergroup_f16scale":
            o_acc, o_y = orc.gemm_samples_f16(o_q, o_sa, w_nat, sg_f.view(np.uint16), sw_bits, im, jn)
        else:
            o_acc, o_y = orc.gemm_samples(o_q, o_sa, w_nat, sg_i if variant == "pergroup" else None,
                                          sw_bits, im, jn)
        t_im, t_jn = torch.from_numpy(im).cuda(), torch.from_numpy(jn).cuda()
        assert np.array_equal(acc[t_im, t_jn].cpu().numpy().astype(np.int64), o_acc)
        assert ulp_distance(f16_bits(y[t_im, t_jn]), o_y).max() <= 1
