"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This module holds NO arithmetic of the method: it only draws random arrays with the
shapes and value distributions of the benchmark workloads (LLaMA-shaped linear layers
with channel-wise activation outliers, uniform int4 codes, small positive scales) and
lays int4 codes out in the natural interchange format (eight 4-bit two's-complement
codes per 32-bit word, nibble i of word j holding W[n, 8j+i]).  Both sides consume the
arrays; neither side's code is used to produce them.  numpy only.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20240609
GROUP = 128


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def activations_fp16(M: int, K: int, seed: int, dist: str = "normal",
                     outlier_frac: float = 0.01, outlier_scale: float = 20.0) -> np.ndarray:
    """fp16 [M,K]; a fixed seeded set of floor(outlier_frac*K) channels is scaled for every token."""
    g = rng(seed)
    if dist == "normal":
        a = g.standard_normal((M, K), dtype=np.float32)
    elif dist == "laplace":
        a = g.laplace(0.0, 1.0, (M, K)).astype(np.float32)
    else:
        raise ValueError(dist)
    n_out = int(outlier_frac * K)
    if n_out:
        ch = rng(seed ^ 0x5EED).choice(K, size=n_out, replace=False)
        a[:, ch] *= np.float32(outlier_scale)
    return a.astype(np.float16)


def int8_activations(M: int, K: int, seed: int, lo: int = -127, hi: int = 127) -> np.ndarray:
    """int8 [M,K] uniform in [lo,hi]: already-quantised activations for GEMM-only cases."""
    return rng(seed).integers(lo, hi + 1, size=(M, K), dtype=np.int8)


def token_scales(M: int, seed: int, lo: float = 0.01, hi: float = 0.2) -> np.ndarray:
    return rng(seed).uniform(lo, hi, size=(M,)).astype(np.float32)


def random_w_nat(N: int, K: int, seed: int) -> np.ndarray:
    """uint32 [N,K/8]: uniformly random words = int4 codes uniform in [-8,7]."""
    assert K % 8 == 0
    return rng(seed).integers(0, 1 << 32, size=(N, K // 8), dtype=np.uint32)


def codes_to_w_nat(codes: np.ndarray) -> np.ndarray:
    """int codes [N,K] in [-8,7] -> uint32 [N,K/8] natural interchange format."""
    codes = np.asarray(codes)
    N, K = codes.shape
    assert K % 8 == 0
    assert codes.min() >= -8 and codes.max() <= 7
    nib = (codes.astype(np.int64) & 0xF).astype(np.uint32).reshape(N, K // 8, 8)
    out = np.zeros((N, K // 8), np.uint32)
    for i in range(8):
        out |= nib[:, :, i] << np.uint32(4 * i)
    return out


def weight_scales_fp16(N: int, seed: int, lo: float, hi: float) -> np.ndarray:
    return rng(seed).uniform(lo, hi, size=(N,)).astype(np.float16)


def group_scales(K: int, N: int, seed: int, lo: int = 1, hi: int = 15) -> np.ndarray:
    """int8 [K/128, N] integer group scales uniform in [lo,hi]."""
    assert K % GROUP == 0
    return rng(seed).integers(lo, hi + 1, size=(K // GROUP, N), dtype=np.int8)


def group_scales_f16(K: int, N: int, seed: int, lo: float = 0.5, hi: float = 15.5) -> np.ndarray:
    """fp16 [K/128, N] real-valued fused group scales s*_Wg = s_Wg / s_Wc, uniform in [lo,hi]
    (|code * s| stays inside int8 for hi <= 15.875)."""
    assert K % GROUP == 0
    return rng(seed).uniform(lo, hi, size=(K // GROUP, N)).astype(np.float16)


def weights_fp16(N: int, K: int, seed: int, outlier_frac: float = 0.001,
                 outlier_scale: float = 8.0) -> np.ndarray:
    """fp16 [N,K] stand-in for a trained linear layer: N(0, sigma_n^2) with a per-output-channel
    sigma_n log-uniform in [0.01, 0.04], and floor(outlier_frac*K) input channels scaled up."""
    g = rng(seed)
    sigma = np.exp(g.uniform(np.log(0.01), np.log(0.04), size=(N, 1))).astype(np.float32)
    w = g.standard_normal((N, K), dtype=np.float32) * sigma
    n_out = int(outlier_frac * K)
    if n_out:
        ch = rng(seed ^ 0xC01).choice(K, size=n_out, replace=False)
        w[:, ch] *= np.float32(outlier_scale)
    return w.astype(np.float16)


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: variant, shape and the distributions of its inputs."""
    name: str
    variant: str          # "perchannel" | "pergroup"
    M: int
    K: int
    N: int
    act_dist: str = "normal"
    outlier_frac: float = 0.01
    outlier_scale: float = 20.0
    sw_lo: float = 0.005
    sw_hi: float = 0.02
    sg_lo: int = 1
    sg_hi: int = 15
    seed: int = BASE_SEED

    def activations(self) -> np.ndarray:
        return activations_fp16(self.M, self.K, self.seed + 1, self.act_dist,
                                self.outlier_frac, self.outlier_scale)

    def w_nat(self) -> np.ndarray:
        return random_w_nat(self.N, self.K, self.seed + 2)

    def s_w(self) -> np.ndarray:
        return weight_scales_fp16(self.N, self.seed + 3, self.sw_lo, self.sw_hi)

    def s_g(self) -> np.ndarray:
        return group_scales(self.K, self.N, self.seed + 4, self.sg_lo, self.sg_hi)

    def s_g_f16(self) -> np.ndarray:
        """Real-valued fp16 fused scales for the same layer (the paper's own per-group form)."""
        return group_scales_f16(self.K, self.N, self.seed + 5, 0.5, float(self.sg_hi) + 0.5)


def _pc(name, M, K, N, cfg):
    return Workload(name, "perchannel", M, K, N, seed=BASE_SEED + 100 * cfg)


def _pg(name, M, K, N, cfg, **kw):
    return Workload(name, "pergroup", M, K, N, sw_lo=0.001, sw_hi=0.005,
                    seed=BASE_SEED + 100 * cfg, **kw)


def workloads() -> dict:
    """The benchmark configurations by name (LLaMA-shaped single linear layers)."""
    w = {}
    w["cfg1_pc_m16_k4096_n4096"] = _pc("cfg1_pc_m16_k4096_n4096", 16, 4096, 4096, 1)
    w["cfg2_pg_m1_k4096_n11008"] = _pg("cfg2_pg_m1_k4096_n11008", 1, 4096, 11008, 2)
    for M in (1, 8, 32, 128, 512, 2048):
        nm = "cfg3_pc_m%d_k5120_n13824" % M
        w[nm] = _pc(nm, M, 5120, 13824, 3)
    w["cfg4_pg_m4096_k11008_n4096"] = _pg("cfg4_pg_m4096_k11008_n4096", 4096, 11008, 4096, 4,
                                          act_dist="laplace", outlier_frac=0.005,
                                          outlier_scale=50.0)
    for M in (1, 16, 256, 4096):
        nm = "cfg5_pc_m%d_k8192_n28672" % M
        w[nm] = _pc(nm, M, 8192, 28672, 5)
        nm = "cfg5_pg_m%d_k8192_n28672" % M
        w[nm] = _pg(nm, M, 8192, 28672, 5)
    return w
