"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: int8 codes, fp32 token scales, packed words and int32 accumulators bit-exact; fp16 outputs
within 1 fp16 ulp of the oracle's fp32-rounded result.  Inputs are seeded and synthetic.
"""
import numpy as np
import pytest
import torch

from oracle import qqq_oracle as orc
from paper_2406_09904_amd import binding as qqq
from paper_2406_09904_amd import synth
from tests.util import f16_bits, to_dev, ulp_distance

pytestmark = pytest.mark.gpu

MODES = {"linear": 1, "clamp": 2, "fused": 3}


@pytest.fixture(autouse=True)
def _reset_overrides():
    yield
    qqq.set_kernel_override(0)
    qqq.set_group_mode_override(0)


def run_gemm(a_q, s_a, w_nat, s_w, K, s_g=None, sg_max=0, family=0, group_mode=0):
    """-> (acc int32 np, y bits np, workspace bytes np) from the HIP library."""
    M = a_q.shape[0]
    N = w_nat.shape[0]
    d_a, d_sa = to_dev(a_q, torch), to_dev(s_a, torch)
    d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
    d_sw = to_dev(s_w.view(np.uint16), torch)
    ws = qqq.new_workspace(M, N, K)
    acc = torch.full((M, N), -12345, dtype=torch.int32, device="cuda")
    qqq.set_kernel_override(family)
    qqq.set_group_mode_override(group_mode)
    if s_g is None:
        y = qqq.qqq_gemm_w4a8_perchannel(d_a, d_sa, d_w, d_sw, ws, acc_out=acc)
    else:
        y = qqq.qqq_gemm_w4a8_pergroup(d_a, d_sa, d_w, to_dev(s_g, torch), d_sw, ws, sg_max=sg_max,
                                       acc_out=acc)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), f16_bits(y), qqq.split_k_part(ws, M, N, K).cpu().numpy()


def check(acc, y, ws, o_acc, o_y):
    assert np.array_equal(acc, o_acc), "int32 accumulators differ: %d of %d" % (
        int((acc != o_acc).sum()), acc.size)
    d = ulp_distance(y, o_y)
    assert d.max() <= 1, "fp16 output off by %d ulp" % int(d.max())
    assert not ws.any(), "workspace not returned to zero"


# ----------------------------------------------------------------------------- pack
@pytest.mark.parametrize("N,K", [(16, 128), (48, 384), (272, 1024), (4096, 4096)])
def test_pack_unpack_roundtrip(N, K):
    w = synth.random_w_nat(N, K, N + K)
    d = to_dev(w, torch)
    p = qqq.qqq_pack_w4(d, K)
    assert p.numel() == N * K // 2
    back = qqq.qqq_unpack_w4(p, N, K)
    assert torch.equal(back, d)
    # packing permutes nibbles, never changes them: same nibble histogram
    pb, wb = p.cpu().numpy(), w.view(np.uint8)
    hist = lambda b: np.bincount(np.concatenate([(b & 0xF).ravel(), (b >> 4).ravel()]), minlength=16)
    assert np.array_equal(hist(pb), hist(wb))
    # position-encoding codes: code = f(n,k); unpack(pack) must restore every position
    n_idx, k_idx = np.meshgrid(np.arange(N), np.arange(K), indexing="ij")
    codes = ((n_idx * 7 + k_idx * 3 + (k_idx >> 4)) % 16) - 8
    w2 = synth.codes_to_w_nat(codes)
    d2 = to_dev(w2, torch)
    assert torch.equal(qqq.qqq_unpack_w4(qqq.qqq_pack_w4(d2, K), N, K), d2)


# ----------------------------------------------------------------------------- quant_act
@pytest.mark.parametrize("M,K", [(1, 128), (3, 4096), (16, 8192), (37, 5120), (5, 11008),
                                 (2, 8), (4, 20000), (300, 1024)])
def test_quant_act_bit_exact(M, K):
    a = synth.activations_fp16(M, K, 1000 + M + K)
    if M >= 3:
        a[1, :] = 0
        a[2, :] = np.float16(65504.0)
        a[2, ::2] = np.float16(-65504.0)
    o_q, o_s = orc.quant_act(a.view(np.uint16))
    d_q, d_s = qqq.qqq_quant_act(to_dev(a.view(np.uint16), torch))
    torch.cuda.synchronize()
    assert np.array_equal(d_s.cpu().numpy().view(np.uint32), o_s.view(np.uint32))
    assert np.array_equal(d_q.cpu().numpy(), o_q)


def test_quant_act_edge_rows_and_row_stride():
    K = 1024
    a = np.zeros((8, K), np.float16)
    a[0, 5] = np.float16(-3.0)                        # single non-zero
    a[1, :] = np.float16(2.0 ** -24)                  # smallest subnormal
    a[2, :] = (np.arange(K) % 255 - 127).astype(np.float16)     # exact multiples of s = 1
    a[3, :] = (np.arange(K) % 255 - 127).astype(np.float16) * np.float16(0.5) + np.float16(0.25)
    a[3, 0] = np.float16(63.5)                        # s = 0.5 -> x/s has .5 ties everywhere
    a[4, :] = synth.activations_fp16(1, K, 5)[0] * np.float16(1e-3)
    a[5, :] = np.float16(6.1e-5)                      # around the fp16 normal/subnormal edge
    a[6, ::7] = np.float16(1.5)
    o_q, o_s = orc.quant_act(a.view(np.uint16))
    d_q, d_s = qqq.qqq_quant_act(to_dev(a.view(np.uint16), torch))
    assert np.array_equal(d_q.cpu().numpy(), o_q) and np.array_equal(d_s.cpu().numpy(), o_s)
    assert o_s[7] == 0 and not o_q[7].any()
    # a strided view (lda > K): rows of a wider matrix
    wide = synth.activations_fp16(6, 2 * K, 6)
    d_wide = to_dev(wide.view(np.uint16), torch)
    d_q, d_s = qqq.qqq_quant_act(d_wide[:, :K])
    o_q, o_s = orc.quant_act(np.ascontiguousarray(wide[:, :K]).view(np.uint16))
    assert np.array_equal(d_q.cpu().numpy(), o_q) and np.array_equal(d_s.cpu().numpy(), o_s)


def test_quant_act_every_fp16_value_under_many_scales():
    """Each row holds every finite fp16 pattern not above the row's |max| (larger ones zeroed): all
    quotients x/s the quantiser can meet for that scale, exact ties and their neighbours included."""
    every = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    every = every[((every >> 10) & 0x1F) != 31]                 # finite only
    vals = every.view(np.float16).astype(np.float64)
    amaxes = [127.0, 63.5, 1.0, 254.0, 0.0124, 3.1416, 65504.0, 6.1e-5, 2.0 ** -24, 1016.0, 100.0, 0.333,
              7.0, 127.0 * 2.0 ** -10, 5.96e-6, 2049.0]
    a = np.zeros((len(amaxes), every.size), np.uint16)
    for r, am in enumerate(amaxes):
        am16 = float(np.float16(am))
        a[r] = np.where(np.abs(vals) <= am16, every, 0)
    o_q, o_s = orc.quant_act(a)
    d_q, d_s = qqq.qqq_quant_act(to_dev(a, torch))
    torch.cuda.synchronize()
    assert np.array_equal(d_s.cpu().numpy().view(np.uint32), o_s.view(np.uint32))
    bad = d_q.cpu().numpy() != o_q
    assert not bad.any(), "%d codes differ, first at %s" % (int(bad.sum()), np.argwhere(bad)[:3])


# ----------------------------------------------------------------------------- GEMM, small shapes
SKINNY = [(1, 16, 128), (1, 64, 4096), (3, 48, 384), (16, 272, 1024), (16, 4096, 1024),
          (17, 64, 512), (33, 96, 640), (64, 128, 2048), (8, 1024, 5120)]
PREFILL = [(65, 16, 128), (100, 272, 384), (128, 256, 1024), (200, 528, 640), (300, 1024, 512),
           (129, 4096, 256)]


def gemm_inputs(M, N, K, seed, sg_hi):
    a_q = synth.int8_activations(M, K, seed)
    s_a = synth.token_scales(M, seed + 1)
    w_nat = synth.random_w_nat(N, K, seed + 2)
    s_w = synth.weight_scales_fp16(N, seed + 3, 0.001, 0.02)
    s_g = synth.group_scales(K, N, seed + 4, 0, sg_hi)
    return a_q, s_a, w_nat, s_w, s_g


@pytest.mark.parametrize("M,N,K", SKINNY + PREFILL)
def test_perchannel_parity(M, N, K):
    a_q, s_a, w_nat, s_w, _ = gemm_inputs(M, N, K, 7 * M + N + K, 15)
    o_acc, _, o_y = orc.gemm_perchannel(a_q, s_a, w_nat, s_w.view(np.uint16))
    check(*run_gemm(a_q, s_a, w_nat, s_w, K), o_acc, o_y)


@pytest.mark.parametrize("M,N,K", [(5, 64, 1024), (16, 272, 1024), (40, 128, 512)])
def test_perchannel_parity_small_m_through_prefill_kernel(M, N, K):
    a_q, s_a, w_nat, s_w, _ = gemm_inputs(M, N, K, 11 * M + N + K, 15)
    o_acc, _, o_y = orc.gemm_perchannel(a_q, s_a, w_nat, s_w.view(np.uint16))
    check(*run_gemm(a_q, s_a, w_nat, s_w, K, family=2), o_acc, o_y)


@pytest.mark.parametrize("mode", ["linear", "clamp", "fused"])
@pytest.mark.parametrize("M,N,K", SKINNY[1:] + PREFILL[1:])
def test_pergroup_parity_small_scales(M, N, K, mode):
    # s_g in 0..16: the clamp can never fire, all three conversions must give the same integers
    a_q, s_a, w_nat, s_w, s_g = gemm_inputs(M, N, K, 13 * M + N + K, 16)
    o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w.view(np.uint16))
    check(*run_gemm(a_q, s_a, w_nat, s_w, K, s_g=s_g, sg_max=16, group_mode=MODES[mode]), o_acc, o_y)


@pytest.mark.parametrize("M,N,K", [(1, 64, 4096), (16, 272, 1024), (64, 128, 2048),
                                   (100, 272, 384), (300, 1024, 512)])
def test_pergroup_parity_saturating_scales(M, N, K):
    # s_g up to 127: code*s leaves int8 and must saturate exactly like the oracle
    a_q, s_a, w_nat, s_w, s_g = gemm_inputs(M, N, K, 17 * M + N + K, 127)
    o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w.view(np.uint16))
    check(*run_gemm(a_q, s_a, w_nat, s_w, K, s_g=s_g, sg_max=0), o_acc, o_y)
    check(*run_gemm(a_q, s_a, w_nat, s_w, K, s_g=s_g, sg_max=127), o_acc, o_y)


def test_automatic_mode_selection_matches():
    M, N, K = 16, 256, 1024
    a_q, s_a, w_nat, s_w, s_g = gemm_inputs(M, N, K, 99, 15)
    o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w.view(np.uint16))
    check(*run_gemm(a_q, s_a, w_nat, s_w, K, s_g=s_g, sg_max=15), o_acc, o_y)
    M = 130
    a_q, s_a, w_nat, s_w, s_g = gemm_inputs(M, N, K, 98, 15)
    o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w.view(np.uint16))
    check(*run_gemm(a_q, s_a, w_nat, s_w, K, s_g=s_g, sg_max=15), o_acc, o_y)


# ----------------------------------------------------------------------------- degenerate / extreme
@pytest.mark.parametrize("M", [5, 150])
def test_one_hot_weights_select_columns(M):
    N, K = 256, 512
    pi = synth.rng(21).permutation(K)[:N]
    codes = np.zeros((N, K), np.int64)
    codes[np.arange(N), pi] = 1
    w_nat = synth.codes_to_w_nat(codes)
    a_q = synth.int8_activations(M, K, 22)
    one = np.ones(M, np.float32)
    s_w = np.ones(N, np.float16)
    acc, y, ws = run_gemm(a_q, one, w_nat, s_w, K)
    assert np.array_equal(acc, a_q[:, pi].astype(np.int32))
    # s_a = s_w = 1 and |acc| <= 127: Y is acc exactly
    assert np.array_equal(y.view(np.float16).astype(np.int32), acc)


@pytest.mark.parametrize("M", [2, 70])
def test_extreme_values_and_int32_limit(M):
    N = 32
    one, s_w = np.ones(M, np.float32), np.ones(N, np.float16)
    K = 131072 if M == 2 else 8192
    a = np.full((M, K), 127, np.int8)
    a[1] = -127
    w = synth.codes_to_w_nat(np.full((N, K), -8))
    acc, _, ws = run_gemm(a, one, w, s_w, K)
    assert np.all(acc[0] == -1016 * K) and np.all(acc[1] == 1016 * K) and not ws.any()
    s16 = np.full((K // 128, N), 16, np.int8)
    for mode in (1, 2, 3):
        acc, _, ws = run_gemm(a, one, w, s_w, K, s_g=s16, sg_max=16, group_mode=mode)
        assert np.all(acc[0] == -16256 * K) and np.all(acc[1] == 16256 * K) and not ws.any()
    if K <= 8192:
        s127 = np.full((K // 128, N), 127, np.int8)
        acc, _, ws = run_gemm(a, one, w, s_w, K, s_g=s127, sg_max=0)
        assert np.all(acc[0] == -128 * 127 * K) and np.all(acc[1] == 128 * 127 * K)


def test_zero_token_and_fp16_overflow_rows():
    M, N, K = 4, 64, 256
    a_q, s_a, w_nat, s_w, _ = gemm_inputs(M, N, K, 5, 15)
    a_q[1] = 0
    s_a[1] = 0.0
    s_a[2] = 1.0e4           # drives |Y| beyond the fp16 range: must become +-inf like the oracle
    o_acc, _, o_y = orc.gemm_perchannel(a_q, s_a, w_nat, s_w.view(np.uint16))
    acc, y, ws = run_gemm(a_q, s_a, w_nat, s_w, K)
    check(acc, y, ws, o_acc, o_y)
    assert not y[1].view(np.float16).any()
    assert np.isinf(y[2].view(np.float16)).any()


def test_repeatable_and_workspace_reuse():
    # integer split-K is order independent: 20 launches on one workspace give identical bits
    M, N, K = 16, 4096, 4096
    a_q, s_a, w_nat, s_w, s_g = gemm_inputs(M, N, K, 31, 15)
    d_a, d_sa = to_dev(a_q, torch), to_dev(s_a, torch)
    d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
    d_sw, d_sg = to_dev(s_w.view(np.uint16), torch), to_dev(s_g, torch)
    ws = qqq.new_workspace(M, N, K)
    ref_acc = ref_y = None
    for it in range(20):
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y = qqq.qqq_gemm_w4a8_pergroup(d_a, d_sa, d_w, d_sg, d_sw, ws, sg_max=15, acc_out=acc)
        if ref_acc is None:
            ref_acc, ref_y = acc, y
        else:
            assert torch.equal(acc, ref_acc) and torch.equal(y.view(torch.int16), ref_y.view(torch.int16))
    assert not ws.any().item()
    o_acc, _, o_y = orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w.view(np.uint16))
    assert np.array_equal(ref_acc.cpu().numpy(), o_acc)
    assert ulp_distance(f16_bits(ref_y), o_y).max() <= 1


def test_device_side_errors_leave_outputs_untouched():
    M, N, K = 4, 64, 256
    a_q, s_a, w_nat, s_w, _ = gemm_inputs(M, N, K, 6, 15)
    d_a, d_sa = to_dev(a_q, torch), to_dev(s_a, torch)
    d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
    d_sw = to_dev(s_w.view(np.uint16), torch)
    y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    small = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(qqq.QQQError) as e:
        qqq.qqq_gemm_w4a8_perchannel(d_a, d_sa, d_w, d_sw, small, y=y)
    assert e.value.code == 3
    torch.cuda.synchronize()
    assert torch.all(y == 7.0).item()
    qqq.set_kernel_override(1)
    big_a = torch.zeros((100, K), dtype=torch.int8, device="cuda")
    with pytest.raises(qqq.QQQError) as e:
        qqq.qqq_gemm_w4a8_perchannel(big_a, torch.zeros(100, device="cuda"), d_w, d_sw,
                                     qqq.new_workspace(100, N, K))
    assert e.value.code == 2


# ----------------------------------------------------------------------------- whole path
@pytest.mark.parametrize("variant,M,K,N", [("perchannel", 16, 4096, 4096), ("pergroup", 1, 4096, 11008),
                                           ("perchannel", 200, 1024, 512)])
def test_whole_path_quant_then_gemm(variant, M, K, N):
    wl = synth.Workload("t", variant, M, K, N, seed=4242 + M)
    a, w_nat, s_w = wl.activations(), wl.w_nat(), wl.s_w()
    o_q, o_sa = orc.quant_act(a.view(np.uint16))
    d_q, d_sa = qqq.qqq_quant_act(to_dev(a.view(np.uint16), torch))
    d_w = qqq.qqq_pack_w4(to_dev(w_nat, torch), K)
    ws = qqq.new_workspace(M, N, K)
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    d_sw = to_dev(s_w.view(np.uint16), torch)
    if variant == "perchannel":
        o_acc, _, o_y = orc.gemm_perchannel(o_q, o_sa, w_nat, s_w.view(np.uint16))
        y = qqq.qqq_gemm_w4a8_perchannel(d_q, d_sa, d_w, d_sw, ws, acc_out=acc)
    else:
        s_g = wl.s_g()
        o_acc, _, o_y = orc.gemm_pergroup(o_q, o_sa, w_nat, s_g, s_w.view(np.uint16))
        y = qqq.qqq_gemm_w4a8_pergroup(d_q, d_sa, d_w, to_dev(s_g, torch), d_sw, ws, sg_max=15,
                                       acc_out=acc)
    torch.cuda.synchronize()
    assert np.array_equal(d_q.cpu().numpy(), o_q)
    assert np.array_equal(d_sa.cpu().numpy(), o_sa)
    check(acc.cpu().numpy(), f16_bits(y), ws.cpu().numpy(), o_acc, o_y)


def test_route_report_and_sg_max_check():
    """The library says which kernels a call enqueued, and the diagnostic scan counts the group
    scales that break an sg_max promise."""
    M, K, N = 2, 1024, 512
    wl = synth.Workload("route", "pergroup", M, K, N, seed=77)
    a = torch.from_numpy(wl.activations()).cuda()
    d_w = qqq.qqq_pack_w4(torch.from_numpy(wl.w_nat().view(np.int32)).cuda(), K)
    s_g = wl.s_g()
    d_sg, d_sw = torch.from_numpy(s_g).cuda(), torch.from_numpy(wl.s_w()).cuda()
    qqq.qqq_linear_w4a8_pergroup(a, d_w, d_sg, d_sw, qqq.new_linear_workspace(M, N, K), sg_max=15)
    assert "decode" in qqq.last_route() and "fused=1" in qqq.last_route(), qqq.last_route()
    a_q, s_a = qqq.qqq_quant_act(a)
    assert qqq.last_route() == "quant_act"
    qqq.qqq_gemm_w4a8_pergroup(a_q, s_a, d_w, d_sg, d_sw, qqq.new_workspace(M, N, K), sg_max=15)
    assert "decode" in qqq.last_route() and "fused=0" in qqq.last_route(), qqq.last_route()
    assert qqq.count_sg_violations(d_sg, 15) == 0
    assert qqq.count_sg_violations(d_sg, 7) == int((s_g > 7).sum())
    bad = s_g.copy()
    bad[3, 17] = -1
    bad[0, 0] = 127
    assert qqq.count_sg_violations(torch.from_numpy(bad).cuda(), 16) == 2
    torch.cuda.synchronize()
