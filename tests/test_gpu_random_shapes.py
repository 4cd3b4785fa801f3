"""GPU parity on a seeded random walk over shapes and entry points: the launcher picks the kernel
(decode kernel with 16/32/64-channel groups and K slices, 64..512-wide prefill tiles, K split with
the reduce kernel, persistent kernel, biased / FMA / saturating / real-valued conversions, fused or
two-kernel one-call path) from the shape, so the walk crosses every boundary of those choices.
Sampled outputs against the oracle one by one: int32 accumulators bit-exact, fp16 within 1 ulp, the
workspace's zero part left zero.
"""
import numpy as np
import pytest
import torch

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import binding as qqq
from paper_2406_09904_amd import synth
from tests.util import f16_bits, to_dev, ulp_distance

pytestmark = pytest.mark.gpu

ROWS = [1, 2, 3, 5, 9, 16, 17, 23, 31, 33, 40, 47, 50, 63, 64, 65, 90, 128, 130, 200, 257, 400, 513, 700, 1025, 1500]
VARIANTS = ["pc", "pg16", "pg127", "real", "lin_pc", "lin_pg"]


def one_case(g, seed, big):
    M = int(g.choice(ROWS))
    if big:
        N = int(g.choice([2048, 4096, 8192, 11008, 13824]))
        K = int(g.choice([1024, 2048, 4096, 5120, 8192, 11008]))
    else:
        N = 16 * int(g.integers(1, 700))
        K = 128 * int(g.integers(1, 60))
    variant = str(g.choice(VARIANTS))
    w = synth.random_w_nat(N, K, seed)
    s_w = synth.weight_scales_fp16(N, seed + 1, 0.001, 0.01)
    a16 = synth.activations_fp16(M, K, seed + 2)
    a_q, s_a = orc.quant_act(a16.view(np.uint16))
    d_w = qqq.qqq_pack_w4(to_dev(w, torch), K)
    d_sw = to_dev(s_w.view(np.uint16), torch)
    d_a16, d_aq, d_sa = to_dev(a16.view(np.uint16), torch), to_dev(a_q, torch), to_dev(s_a, torch)
    acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ns = min(2000, M * N)
    im, jn = g.integers(0, M, ns), g.integers(0, N, ns)
    linear = variant.startswith("lin")
    ws = qqq.new_linear_workspace(M, N, K) if linear else qqq.new_workspace(M, N, K)
    if variant in ("pc", "lin_pc"):
        o_acc, o_y = orc.gemm_samples(a_q, s_a, w, None, s_w.view(np.uint16), im, jn)
        y = (qqq.qqq_linear_w4a8_perchannel(d_a16, d_w, d_sw, ws, acc_out=acc) if linear else
             qqq.qqq_gemm_w4a8_perchannel(d_aq, d_sa, d_w, d_sw, ws, acc_out=acc))
    elif variant == "real":
        s16 = synth.group_scales_f16(K, N, seed + 3).view(np.uint16)
        o_acc, o_y = orc.gemm_samples_f16(a_q, s_a, w, s16, s_w.view(np.uint16), im, jn)
        y = qqq.qqq_gemm_w4a8_pergroup_f16scale(d_aq, d_sa, d_w, to_dev(s16, torch), d_sw, ws, acc_out=acc)
    else:
        hi, sg_max = (127, 0) if variant == "pg127" else (16, 16)
        s_g = synth.group_scales(K, N, seed + 3, 0, hi)
        o_acc, o_y = orc.gemm_samples(a_q, s_a, w, s_g, s_w.view(np.uint16), im, jn)
        d_sg = to_dev(s_g, torch)
        y = (qqq.qqq_linear_w4a8_pergroup(d_a16, d_w, d_sg, d_sw, ws, sg_max=sg_max, acc_out=acc) if linear else
             qqq.qqq_gemm_w4a8_pergroup(d_aq, d_sa, d_w, d_sg, d_sw, ws, sg_max=sg_max, acc_out=acc))
    torch.cuda.synchronize()
    what = "%s M=%d N=%d K=%d" % (variant, M, N, K)
    assert np.array_equal(acc.cpu().numpy()[im, jn].astype(np.int64), o_acc), what + ": accumulators differ"
    assert ulp_distance(f16_bits(y)[im, jn], o_y).max() <= 1, what + ": fp16 output off by more than 1 ulp"
    assert not qqq.split_k_part(ws, M, N, K).any().item(), what + ": workspace zero part not zero"


@pytest.mark.parametrize("block", range(4))
def test_random_small_layers(block):
    g = synth.rng(977 + block)
    for i in range(12):
        one_case(g, 5000 + 100 * block + i, big=False)


@pytest.mark.parametrize("block", range(4))
def test_random_llm_sized_layers(block):
    g = synth.rng(1977 + block)
    for i in range(6):
        one_case(g, 7000 + 100 * block + i, big=True)
