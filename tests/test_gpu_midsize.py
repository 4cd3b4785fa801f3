"""GPU parity for mid-size M (65..1024 rows), where the prefill path picks narrower tiles so that
enough workgroups exist, against the CPU oracle: every tile shape forced on ragged shapes, the
automatic choice on shapes that select each of them, and K split over several workgroups per tile
(raw int32 tiles summed by a second kernel), forced and chosen automatically.
"""
import numpy as np
import pytest
import torch

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import binding as qqq
from paper_2406_09904_amd import synth
from tests.util import f16_bits, to_dev, ulp_distance

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset():
    yield
    qqq.set_prefill_tuning(0)
    qqq.set_prefill_ksplit(0)
    qqq.set_group_mode_override(0)


def run(variant, a_q, s_a, w_nat, s_w, K, s_g=None, sg_max=0):
    M, N = a_q.shape[0], w_nat.shape[0]
    d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
    d_sw = to_dev(s_w.view(np.uint16), torch)
    ws = qqq.new_workspace(M, N, K)
    acc = torch.full((M, N), -12345, dtype=torch.int32, device="cuda")
    d_a, d_sa = to_dev(a_q, torch), to_dev(s_a, torch)
    if variant == "pc":
        y = qqq.qqq_gemm_w4a8_perchannel(d_a, d_sa, d_w, d_sw, ws, acc_out=acc)
    elif variant in ("pg", "pgb"):
        if variant == "pgb":   # the biased integer route, also where the automatic choice would skip its pre-pass
            qqq.set_group_mode_override(5)
        y = qqq.qqq_gemm_w4a8_pergroup(d_a, d_sa, d_w, to_dev(s_g, torch), d_sw, ws, sg_max=sg_max, acc_out=acc)
        if variant == "pgb":
            assert "mode=5" in qqq.last_route(), qqq.last_route()
            qqq.set_group_mode_override(0)
    else:
        y = qqq.qqq_gemm_w4a8_pergroup_f16scale(d_a, d_sa, d_w, to_dev(s_g, torch), d_sw, ws, acc_out=acc)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), f16_bits(y)


def reference(variant, a_q, s_a, w, s_w, K, N, seed, hi=16):
    if variant == "pc":
        s_g = None
        o_acc, _, o_y = orc.gemm_perchannel(a_q, s_a, w, s_w.view(np.uint16))
    elif variant in ("pg", "pgb"):
        s_g = synth.group_scales(K, N, seed, 1, hi)
        o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w, s_g, s_w.view(np.uint16))
    else:
        s_g = synth.group_scales_f16(K, N, seed).view(np.uint16)
        o_acc, _, o_y = orc.gemm_pergroup_f16(a_q, s_a, w, s_g, s_w.view(np.uint16))
    return s_g, o_acc, o_y


def inputs(M, K, N, seed):
    return (synth.int8_activations(M, K, seed), synth.token_scales(M, seed + 1),
            synth.random_w_nat(N, K, seed + 2), synth.weight_scales_fp16(N, seed + 3, 0.001, 0.01))


def check(acc, y, o_acc, o_y):
    assert np.array_equal(acc, o_acc), "int32 accumulators differ: %d of %d" % (
        int((acc != o_acc).sum()), acc.size)
    assert ulp_distance(y, o_y).max() <= 1


# 27 / 37: the 64x128 shape with its six-stage and its three-stage ring (17 picks by workgroup count)
@pytest.mark.parametrize("tune", [15, 16, 17, 27, 37])
@pytest.mark.parametrize("variant,hi,sg_max", [("pc", 0, 0), ("pg", 16, 16), ("pgb", 16, 16), ("pg", 127, 0), ("real", 0, 0)])
def test_forced_narrow_tiles_on_ragged_shapes(tune, variant, hi, sg_max):
    for (M, K, N) in ((150, 640, 784), (65, 128, 16), (333, 256, 400)):   # ragged in M and N
        a_q, s_a, w, s_w = inputs(M, K, N, M + K + N)
        s_g, o_acc, o_y = reference(variant, a_q, s_a, w, s_w, K, N, 7, hi or 16)
        qqq.set_prefill_tuning(tune)
        check(*run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=sg_max), o_acc, o_y)


# automatic choice: 64x128 tiles, 128x128, 128x256, and the large tile
@pytest.mark.parametrize("M,K,N", [(96, 1024, 4096), (128, 640, 13824), (200, 512, 11008),
                                   (512, 384, 13824), (1024, 256, 8192), (1000, 256, 2064)])
@pytest.mark.parametrize("variant", ["pc", "pg", "pgb", "real"])
def test_automatic_choice(M, K, N, variant):
    a_q, s_a, w, s_w = inputs(M, K, N, M + K + N + 1)
    s_g, o_acc, o_y = reference(variant, a_q, s_a, w, s_w, K, N, 9, 15)
    check(*run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=15), o_acc, o_y)


@pytest.mark.parametrize("tune,k_splits", [(15, 2), (16, 3), (17, 2), (17, 5), (10, 2), (17, 8)])
@pytest.mark.parametrize("variant,hi,sg_max", [("pc", 0, 0), ("pg", 16, 16), ("pgb", 16, 16), ("pg", 127, 0), ("real", 0, 0)])
def test_forced_k_split(tune, k_splits, variant, hi, sg_max):
    """K ranges of unequal length (k-steps not divisible by the split), ragged M and N, every
    conversion route; the biased per-group route puts its whole correction into the first split."""
    for (M, K, N) in ((100, 1408, 528), (65, 2560, 144)):
        a_q, s_a, w, s_w = inputs(M, K, N, M + K + N + 2)
        s_g, o_acc, o_y = reference(variant, a_q, s_a, w, s_w, K, N, 11, hi or 16)
        qqq.set_prefill_tuning(tune)
        qqq.set_prefill_ksplit(k_splits)
        check(*run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=sg_max), o_acc, o_y)


def test_k_split_equals_unsplit_bit_for_bit_and_caps():
    M, K, N = 300, 1024, 656
    a_q, s_a, w, s_w = inputs(M, K, N, 5)
    qqq.set_prefill_tuning(17)
    qqq.set_prefill_ksplit(1)
    acc1, y1 = run("pc", a_q, s_a, w, s_w, K)
    qqq.set_prefill_ksplit(3)                                  # 3 * 300 <= 1024
    acc3, y3 = run("pc", a_q, s_a, w, s_w, K)
    qqq.set_prefill_ksplit(64)                                 # capped at 1024 / M = 3 and at K / 128
    acc64, y64 = run("pc", a_q, s_a, w, s_w, K)
    assert np.array_equal(acc1, acc3) and np.array_equal(y1, y3)
    assert np.array_equal(acc1, acc64) and np.array_equal(y1, y64)
    assert qqq.set_prefill_ksplit(-1) == 64                    # negative values only query


@pytest.mark.parametrize("variant", ["pc", "pg"])
def test_automatic_k_split_on_a_long_k_narrow_n_layer(variant):
    """M=128, K=21760, N=2048: 32 tiles of 64x128 for 256 CUs, 170 k-steps: the cost model splits K.
    Sampled outputs against the oracle plus the unsplit kernel bit for bit."""
    M, K, N = 128, 21760, 2048
    a_q, s_a, w, s_w = inputs(M, K, N, 6)
    s_g = synth.group_scales(K, N, 12, 1, 15) if variant == "pg" else None
    acc, y = run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=15)
    qqq.set_prefill_ksplit(1)
    acc1, y1 = run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=15)
    assert np.array_equal(acc, acc1) and np.array_equal(y, y1)
    g = synth.rng(13)
    im, jn = g.integers(0, M, 4000), g.integers(0, N, 4000)
    o_acc, o_y = orc.gemm_samples(a_q, s_a, w, s_g, s_w.view(np.uint16), im, jn)
    assert np.array_equal(acc[im, jn].astype(np.int64), o_acc)
    assert ulp_distance(y[im, jn], o_y).max() <= 1


@pytest.mark.parametrize("variant,hi,sg_max", [("pc", 0, 0), ("pg", 16, 16), ("pgb", 16, 16), ("pg", 127, 0), ("real", 0, 0)])
def test_forced_persistent_kernel(variant, hi, sg_max):
    """The persistent kernel (one workgroup per CU walking its tiles) on shapes with fewer tiles than
    CUs, ragged edges, K at its minimum of three k-steps; every element against the oracle.  The
    real-valued route is not carried by it and must fall back to the per-tile kernel."""
    for (M, K, N) in ((300, 512, 1040), (130, 384, 528), (257, 1152, 2064)):
        a_q, s_a, w, s_w = inputs(M, K, N, M + K + N + 3)
        s_g, o_acc, o_y = reference(variant, a_q, s_a, w, s_w, K, N, 17, hi or 16)
        qqq.set_prefill_tuning(13)
        check(*run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=sg_max), o_acc, o_y)


def test_automatic_choice_of_the_persistent_kernel_with_the_biased_route():
    """More 128x512 tiles than CUs (9 x 32 = 288) and a short K: per-group with s_g <= 16 and a
    workspace takes the persistent kernel with the biased conversion; every element against the oracle."""
    M, K, N = 1100, 512, 16384
    a_q, s_a, w, s_w = inputs(M, K, N, 21)
    s_g, o_acc, o_y = reference("pg", a_q, s_a, w, s_w, K, N, 19, 16)
    check(*run("pg", a_q, s_a, w, s_w, K, s_g=s_g, sg_max=16), o_acc, o_y)


@pytest.mark.parametrize("M,K,N", [(1100, 512, 16400), (1100, 384, 44048), (2065, 640, 13824)])
@pytest.mark.parametrize("variant,hi,sg_max", [("pc", 0, 0), ("pg", 16, 16), ("pg", 127, 0)])
def test_persistent_kernel_with_more_tiles_than_cus(M, K, N, variant, hi, sg_max):
    """More 128x512 tiles than CUs, so every workgroup of the persistent kernel walks several tiles
    and its DMA cursor crosses tile borders (297, 783 = three per CU, and 459 tiles), ragged in M
    and N, K down to the kernel's minimum of three k-steps: automatic selection (whatever the cost
    model picks for the shape) and the persistent kernel forced; every element against the oracle.
    The automatic choice of the persistent kernel itself is checked at the benchmark's full sizes."""
    a_q, s_a, w, s_w = inputs(M, K, N, M + K + N + 5)
    s_g, o_acc, o_y = reference(variant, a_q, s_a, w, s_w, K, N, 23, hi or 16)
    check(*run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=sg_max), o_acc, o_y)
    print("automatic route for %s M=%d K=%d N=%d: %s" % (variant, M, K, N, qqq.last_route()), flush=True)
    qqq.set_prefill_tuning(13)
    check(*run(variant, a_q, s_a, w, s_w, K, s_g=s_g, sg_max=sg_max), o_acc, o_y)
    assert "prefill persistent" in qqq.last_route(), qqq.last_route()


@pytest.mark.parametrize("tune,k_splits", [(10, 1), (13, 1), (15, 1), (16, 1), (17, 1), (27, 1), (37, 1), (15, 2), (17, 3)])
def test_wide_biased_route_through_every_prefill_kernel(tune, k_splits):
    """Integer scales up to 18 with codes in [-7,7] (what the front-end emits): the byte-wise integer route forms
    (7 - code) * s_g and the kernels carry the negated sums; forced through every tile shape, the persistent kernel
    and K splits on ragged shapes, every element against the oracle."""
    for (M, K, N) in ((150, 640, 784), (65, 384, 16), (333, 1408, 400)):
        g = synth.rng(900 + M + tune)
        w_nat = synth.codes_to_w_nat(g.integers(-7, 8, (N, K)).astype(np.int8))
        s_g = g.integers(1, 19, (K // 128, N)).astype(np.int8)
        s_g[0, :] = 18
        a_q = synth.int8_activations(M, K, 901 + M)
        s_a = synth.token_scales(M, 902 + M)
        s_w = synth.weight_scales_fp16(N, 903 + M, 0.001, 0.01)
        o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w.view(np.uint16))
        qqq.set_prefill_tuning(tune)
        qqq.set_prefill_ksplit(k_splits)
        qqq.set_group_mode_override(5)
        d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
        acc = torch.full((M, N), -12345, dtype=torch.int32, device="cuda")
        y = qqq.qqq_gemm_w4a8_pergroup(to_dev(a_q, torch), to_dev(s_a, torch), d_w, to_dev(s_g, torch),
                                       to_dev(s_w.view(np.uint16), torch), qqq.new_workspace(M, N, K),
                                       sg_max=18 | qqq.SG_SYMMETRIC_CODES, acc_out=acc)
        torch.cuda.synchronize()
        assert "mode=8" in qqq.last_route(), qqq.last_route()
        check(acc.cpu().numpy(), f16_bits(y), o_acc, o_y)
