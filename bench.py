#!/usr/bin/env python3
"""Benchmark of the W4A8 hot path (quantise activations -> W4A8 GEMM) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-sweep]
                  [--no-cpu-baseline] [--eager]

A step is one pass of the whole hot path over one batch of seeded synthetic input that is
already resident in HBM: per-token int8 quantisation of the fp16 activations, then the W4A8 GEMM
of the workload's variant, through the library's one-call entry point qqq_linear_w4a8_* (for a
few decode rows that is one fused kernel, otherwise qqq_quant_act's kernel followed by the GEMM
kernel; weights were repacked once, offline, outside the timed region).  Packed
weights (and group scales) exist in R copies whose total exceeds four times the 256 MiB
last-level cache and consecutive steps rotate through them, so every step streams its weights
from HBM rather than from cache.  The K timed steps are captured once into a HIP graph and
replayed, which removes Python's launch overhead from microsecond-scale kernels (--eager
disables that).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "W4A8 GEMM TOPS and % roofline (HBM at M<=16, int8 MFMA at M>=1024)"
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_I8_PEAK_TOPS = 5033.0     # dense int8 MFMA: 256 CU x 4 SIMD x 2048 op/clk x 2.4 GHz
PRIMARY = "cfg2_pg_m1_k4096_n11008"
SWEEP = ["cfg1_pc_m16_k4096_n4096", "cfg3_pc_m1_k5120_n13824", "cfg3_pc_m8_k5120_n13824",
         "cfg3_pc_m2048_k5120_n13824", "cfg4_pg_m4096_k11008_n4096",
         "cfg5_pc_m1_k8192_n28672", "cfg5_pg_m16_k8192_n28672", "cfg5_pc_m4096_k8192_n28672",
         "cfg5_pg_m4096_k8192_n28672"]


def algorithmic_bytes(M, N, K, pergroup):
    """What the method itself must move once: packed int4 weights, group scales, fp16 channel
    scales, int8 activations, fp32 token scales, fp16 output."""
    return N * K // 2 + (K // 128 * N if pergroup else 0) + 2 * N + M * K + 4 * M + 2 * M * N


def quant_bytes(M, K):
    return 2 * M * K + M * K + 4 * M


def fused_bytes(M, N, K, pergroup):
    """Algorithmic bytes of the fused decode kernel: fp16 activations in, no int8 round trip."""
    return N * K // 2 + (K // 128 * N if pergroup else 0) + 2 * N + 2 * M * K + 2 * M * N


def is_fused(M, K):
    """Shapes for which qqq_linear_* runs the single fused kernel (see include/qqq.h)."""
    return M <= 4 and M * K <= 8192


class Case:
    """Device-resident inputs of one workload plus the launch closures."""

    def __init__(self, wl, torch, qqq, rotate_bytes=1 << 30, max_copies=64):
        import numpy as np
        self.wl = wl
        self.pg = wl.variant == "pergroup"
        M, K, N = wl.M, wl.K, wl.N
        self.a = torch.from_numpy(wl.activations()).cuda()
        w_nat = torch.from_numpy(wl.w_nat().view(np.int32)).cuda()
        packed = qqq.qqq_pack_w4(w_nat, K)
        del w_nat
        per_copy = packed.numel() + (K // 128 * N if self.pg else 0)
        self.copies = int(max(1, min(max_copies, -(-rotate_bytes // per_copy))))
        self.w = [packed] + [packed.clone() for _ in range(self.copies - 1)]
        self.s_w = torch.from_numpy(wl.s_w()).cuda()
        if self.pg:
            sg = torch.from_numpy(wl.s_g()).cuda()
            self.s_g = [sg] + [sg.clone() for _ in range(self.copies - 1)]
        self.a_q = torch.empty((M, K), dtype=torch.int8, device="cuda")
        self.s_a = torch.empty((M,), dtype=torch.float32, device="cuda")
        self.y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        self.ws = qqq.new_workspace(M, N, K)
        self.lws = qqq.new_linear_workspace(M, N, K)
        self.qqq = qqq
        self.ops = 2 * M * N * K
        self.bytes = algorithmic_bytes(M, N, K, self.pg)
        self.fused = is_fused(M, K)
        # the GEMM-only timing reads a_q/s_a: fill them with the workload's real codes first (MFMA
        # power, hence clock and speed, depends on the operand values)
        self.quant()
        torch.cuda.synchronize()

    def quant(self):
        self.qqq.qqq_quant_act(self.a, self.a_q, self.s_a)

    def gemm(self, i):
        r = i % self.copies
        if self.pg:
            self.qqq.qqq_gemm_w4a8_pergroup(self.a_q, self.s_a, self.w[r], self.s_g[r], self.s_w,
                                            self.ws, sg_max=self.wl.sg_hi, y=self.y)
        else:
            self.qqq.qqq_gemm_w4a8_perchannel(self.a_q, self.s_a, self.w[r], self.s_w, self.ws,
                                              y=self.y)

    def step(self, i):
        r = i % self.copies
        if self.pg:
            self.qqq.qqq_linear_w4a8_pergroup(self.a, self.w[r], self.s_g[r], self.s_w, self.lws,
                                              sg_max=self.wl.sg_hi, y=self.y)
        else:
            self.qqq.qqq_linear_w4a8_perchannel(self.a, self.w[r], self.s_w, self.lws, y=self.y)


def timed(torch, fn, steps, warmup, use_graph):
    """fn(i) enqueues one unit of work on the current stream.  Returns average ms per unit over
    exactly `steps` units, measured with events on that stream between two synchronisations."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    graph = None
    if use_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(steps):
                    fn(warmup + i)
            graph.replay()           # one untimed replay: graph upload
            torch.cuda.synchronize()
        except Exception as ex:      # capture unsupported: fall back to eager launches
            print("bench: graph capture failed (%s); timing eager launches" % ex, file=sys.stderr)
            graph = None
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    e0.record()
    if graph is not None:
        graph.replay()
    else:
        for i in range(steps):
            fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps, graph is not None


def roofline_for(case, step_ms, gemm_ms):
    """Roofline of the step's dominant kernel: the fused kernel (= the whole step) where
    qqq_linear_* fuses, the GEMM kernel otherwise."""
    wl = case.wl
    if case.fused:
        kernel, kernel_ms = "linear_w4a8_%s (fused quant_act + gemm)" % wl.variant, step_ms
        nbytes = fused_bytes(wl.M, wl.N, wl.K, case.pg)
    else:
        kernel, kernel_ms, nbytes = "gemm_w4a8_%s" % wl.variant, gemm_ms, case.bytes
    t_mem = nbytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = case.ops / (MFMA_I8_PEAK_TOPS * 1e12)
    if t_mem >= t_mfma:
        achieved = nbytes / (kernel_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4)}
    else:
        achieved = case.ops / (kernel_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_I8_PEAK_TOPS,
                "unit": "TOP/s", "frac": round(achieved / MFMA_I8_PEAK_TOPS, 4)}
    roof["kernel"] = kernel
    roof["kernel_us"] = round(kernel_ms * 1e3, 3)
    roof["algorithmic_bytes"] = nbytes
    return roof


def load_traffic(name):
    """HBM bytes per GEMM launch from the rocprofv3 --pmc summaries under profiles/, if present."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f).get(name)
        return int(rec["fetch_bytes"]) + int(rec["write_bytes"]) if rec else None
    except (OSError, ValueError, KeyError, TypeError):
        return None


def measure(case, torch, steps, warmup, use_graph):
    step_ms, graphed = timed(torch, case.step, steps, warmup, use_graph)
    gemm_ms, _ = timed(torch, case.gemm, steps, warmup, use_graph)
    quant_ms, _ = timed(torch, lambda i: case.quant(), steps, warmup, use_graph)
    return step_ms, gemm_ms, quant_ms, graphed


def real_scale_lines(wls, torch, qqq, args, use_graph):
    """The per-group GEMM with the paper's real-valued fp16 fused scale (Sec. 3.3.2 as printed) on
    the two per-group layer shapes: GEMM kernel only, same rotation of weight copies."""
    import numpy as np
    lines = []
    for name in ("cfg2_pg_m1_k4096_n11008", "cfg4_pg_m4096_k11008_n4096"):
        wl = wls[name]
        big = wl.M >= 1024
        c = Case(wl, torch, qqq, rotate_bytes=(1 << 28) if big else (1 << 30))
        c.quant()
        sg16 = torch.from_numpy(wl.s_g_f16()).cuda()
        sgs = [sg16] + [sg16.clone() for _ in range(c.copies - 1)]

        def gemm(i, c=c, sgs=sgs):
            r = i % c.copies
            qqq.qqq_gemm_w4a8_pergroup_f16scale(c.a_q, c.s_a, c.w[r], sgs[r], c.s_w, c.ws, y=c.y)

        st = max(5, min(args.steps, 20 if big else 100))
        ms, _ = timed(torch, gemm, st, min(args.warmup, 5), use_graph)
        nbytes = c.bytes + wl.K // 128 * wl.N       # fp16 scales: one more byte per group scale
        t_mem = nbytes / (HBM_PEAK_GBS * 1e9)
        t_mfma = c.ops / (MFMA_I8_PEAK_TOPS * 1e12)
        if t_mem >= t_mfma:
            ach = nbytes / (ms * 1e-3) / 1e9
            roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4)}
        else:
            ach = c.ops / (ms * 1e-3) / 1e12
            roof = {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_I8_PEAK_TOPS,
                    "unit": "TOP/s", "frac": round(ach / MFMA_I8_PEAK_TOPS, 4)}
        lines.append({"shape_of": name, "entry": "qqq_gemm_w4a8_pergroup_f16scale", "steps": st,
                      "gemm_us": round(ms * 1e3, 3), "tops": round(c.ops / (ms * 1e-3) / 1e12, 3),
                      "roofline": roof})
        del c, sgs, sg16
        torch.cuda.empty_cache()
    return lines


def conversion_ablation(torch, qqq, wls, use_graph):
    """Per-group prefill GEMM on the cfg4 shape with each way of turning int4 code x group scale into
    int8 (Sec. 3.3.2; the paper's Fig. 9 ablates FastFP16toINT8 against the conventional conversion
    instruction).  Same kernel family and tile shape; only the conversion differs.  The per-channel
    GEMM on the same shape is the no-conversion reference."""
    wl = wls["cfg4_pg_m4096_k11008_n4096"]
    c = Case(wl, torch, qqq, rotate_bytes=1 << 28)
    sg16 = torch.from_numpy(wl.s_g_f16()).cuda()
    rows = []

    def t(fn):
        ms, _ = timed(torch, fn, 20, 5, use_graph)
        return round(ms * 1e3, 1)

    def pg(i):
        qqq.qqq_gemm_w4a8_pergroup(c.a_q, c.s_a, c.w[i % c.copies], c.s_g[i % c.copies], c.s_w, c.ws,
                                   sg_max=15, y=c.y)

    def pg_any(i):
        qqq.qqq_gemm_w4a8_pergroup(c.a_q, c.s_a, c.w[i % c.copies], c.s_g[i % c.copies], c.s_w, c.ws,
                                   sg_max=0, y=c.y)

    def real(i):
        qqq.qqq_gemm_w4a8_pergroup_f16scale(c.a_q, c.s_a, c.w[i % c.copies], sg16, c.s_w, c.ws, y=c.y)

    def pc(i):
        qqq.qqq_gemm_w4a8_perchannel(c.a_q, c.s_a, c.w[i % c.copies], c.s_w, c.ws, y=c.y)

    qqq.set_prefill_tuning(10)                      # one kernel and tile shape for every line
    rows.append({"route": "per-channel (FastINT4toINT8, no group scale)", "gemm_us": t(pc)})
    rows.append({"route": "integer scale <= 16: packed 16-bit multiply + bias removal (default)",
                 "gemm_us": t(pg)})
    qqq.set_group_mode_override(3)
    rows.append({"route": "integer scale <= 16: fp16 FMA with folded constants + byte permute",
                 "gemm_us": t(pg)})
    qqq.set_group_mode_override(0)
    rows.append({"route": "integer scale, any: fp16 multiply, clamp, add, byte permute", "gemm_us": t(pg_any)})
    rows.append({"route": "real-valued scale: FastINT4toFP16 + FMA(128+1024) + permute + XOR (paper)",
                 "gemm_us": t(real)})
    qqq.set_group_mode_override(4)
    rows.append({"route": "real-valued scale: fp16 multiply + conventional round/convert + packing",
                 "gemm_us": t(real)})
    qqq.set_group_mode_override(0)
    qqq.set_prefill_tuning(0)
    for r in rows:
        r["tops"] = round(c.ops / (r["gemm_us"] * 1e-6) / 1e12, 1)
    return {"shape": {"M": wl.M, "K": wl.K, "N": wl.N}, "kernel": "gemm_prefill_dma_kernel, 128x512 tile",
            "rows": rows}


def front_end_lines(torch, qqq, synth, use_graph):
    """Offline weight front-end (fp16 weights -> int4 codes + scales, then the repack) on the two
    largest benchmark layers.  HBM-bound streaming passes; algorithmic bytes per weight: 2 in,
    0.5 out for the quantiser (plus the scale tables), 0.5 in + 0.5 out for the repack."""
    import numpy as np
    rows = []
    for name, N, K in (("cfg5 layer", 28672, 8192), ("cfg4 layer", 4096, 11008)):
        w = torch.from_numpy(synth.weights_fp16(N, K, 31).view(np.int16)).cuda().view(torch.float16)
        G = K // 128
        for variant in ("perchannel", "pergroup"):
            if variant == "perchannel":
                res = qqq.qqq_quantize_w4_perchannel(w)
                fn = lambda i, res=res: qqq.qqq_quantize_w4_perchannel(w, out=res)
                nbytes = N * K * 2.5 + N * 2
            else:
                res = qqq.qqq_quantize_w4_pergroup(w)
                fn = lambda i, res=res: qqq.qqq_quantize_w4_pergroup(w, out=res)
                nbytes = N * K * 2.5 + N * 2 + G * N * 5
            torch.cuda.synchronize()
            ms, _ = timed(torch, fn, 10, 2, use_graph)
            rows.append({"layer": name, "N": N, "K": K, "kernel": "quant_weight_kernel (%s)" % variant,
                         "us": round(ms * 1e3, 1), "bound": "hbm",
                         "achieved_gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "frac": round(nbytes / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9), 3)})
        w_nat, _ = qqq.qqq_quantize_w4_perchannel(w)
        out = qqq.qqq_pack_w4(w_nat, K)
        ms, _ = timed(torch, lambda i: qqq.qqq_pack_w4(w_nat, K, out=out), 10, 2, use_graph)
        rows.append({"layer": name, "N": N, "K": K, "kernel": "pack_w4", "us": round(ms * 1e3, 1), "bound": "hbm",
                     "achieved_gbs": round(N * K / (ms * 1e-3) / 1e9, 1),
                     "frac": round(N * K / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9), 3)})
        del w, w_nat, out
        torch.cuda.empty_cache()
    return rows


def token_sweep(torch, qqq, synth, use_graph):
    """The paper's own GEMM-study shape (Sec. 4.4: N=8192, K=21760) over a sweep of token counts:
    GEMM-kernel time of the per-channel, the integer per-group and the real-valued per-group
    variant, with the box's fp16 GEMM (torch.matmul, i.e. hipBLASLt/rocBLAS) timed in the same run
    as context for the speed-up ratios of Fig. 8.  Synthetic inputs as for the other workloads."""
    import numpy as np
    N, K = 8192, 21760
    rows = []
    w_nat = torch.from_numpy(synth.random_w_nat(N, K, 77).view(np.int32)).cuda()
    packed = qqq.qqq_pack_w4(w_nat, K)
    del w_nat
    copies = 12                                  # 12 x 85 MiB > 1 GiB: cold weights at small M
    ws_ = [packed] + [packed.clone() for _ in range(copies - 1)]
    s_w = torch.from_numpy(synth.weight_scales_fp16(N, 78, 0.001, 0.005)).cuda()
    sg_i = torch.from_numpy(synth.group_scales(K, N, 79, 1, 15)).cuda()
    sg_f = torch.from_numpy(synth.group_scales_f16(K, N, 80)).cuda()
    w16 = [torch.randn((N, K), dtype=torch.float16, device="cuda") * 0.02 for _ in range(3)]
    for M in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096):
        a = torch.from_numpy(synth.activations_fp16(M, K, 81 + M)).cuda()
        a_q, s_a = qqq.qqq_quant_act(a)
        y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        wsp = qqq.new_workspace(M, N, K)
        st = 50 if M <= 64 else (20 if M <= 1024 else 8)
        fns = {
            "perchannel_us": lambda i: qqq.qqq_gemm_w4a8_perchannel(a_q, s_a, ws_[i % copies], s_w, wsp, y=y),
            "pergroup_us": lambda i: qqq.qqq_gemm_w4a8_pergroup(a_q, s_a, ws_[i % copies], sg_i, s_w, wsp,
                                                                 sg_max=15, y=y),
            "pergroup_f16scale_us": lambda i: qqq.qqq_gemm_w4a8_pergroup_f16scale(
                a_q, s_a, ws_[i % copies], sg_f, s_w, wsp, y=y),
            "fp16_matmul_us": lambda i: torch.matmul(a, w16[i % 3].t(), out=y),
        }
        row = {"M": M}
        for key, fn in fns.items():
            ms, _ = timed(torch, fn, st, 3, use_graph)
            row[key] = round(ms * 1e3, 2)
        row["speedup_perchannel_vs_fp16"] = round(row["fp16_matmul_us"] / row["perchannel_us"], 2)
        row["speedup_pergroup_vs_fp16"] = round(row["fp16_matmul_us"] / row["pergroup_us"], 2)
        rows.append(row)
        print("token sweep M=%d: %s" % (M, row), file=sys.stderr, flush=True)
    return {"shape": {"N": N, "K": K}, "note": "GEMM kernel only, HIP graph replay, weight copies "
            "rotated (12 x 85 MiB); fp16_matmul is torch.matmul on fp16 weights (3 copies rotated)",
            "rows": rows}


def cpu_baseline(wl, budget_s=12.0):
    """The oracle, as it stands, on this machine's host cores: whole path on the workload (repeated
    until the time budget is used when one pass is short, on a row subset when one pass is long)."""
    import numpy as np
    from oracle import qqq_oracle as orc
    cores = os.cpu_count() or 1
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        pass
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env)) if int(env) > 0 else cores
    a, w_nat, s_w = wl.activations(), wl.w_nat(), wl.s_w().view(np.uint16)
    s_g = wl.s_g() if wl.variant == "pergroup" else None
    rows = wl.M
    macs_full = wl.M * wl.N * wl.K
    if macs_full > 4e9:                       # keep one pass to roughly ten seconds
        rows = max(1, int(wl.M * 4e9 / macs_full))
    a = np.ascontiguousarray(a[:rows])

    def one_pass():
        a_q, s_a = orc.quant_act(a.view(np.uint16))
        if s_g is None:
            orc.gemm_perchannel(a_q, s_a, w_nat, s_w)
        else:
            orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w)

    one_pass()                                # builds/loads the library, warms the page cache
    reps, t0 = 0, time.perf_counter()
    while True:
        one_pass()
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= 200:
            break
    tops = 2.0 * rows * wl.N * wl.K * reps / el / 1e12
    return {"value": round(tops, 6), "unit": "TOPS", "cores": cores, "kind": "oracle",
            "sample": "%d pass(es) of quant_act + %s GEMM on rows 0..%d of %s (all N=%d columns, "
                      "K=%d), %.1f s wall" % (reps, wl.variant, rows - 1, wl.name, wl.N, wl.K, el)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=PRIMARY)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time eager launches, no HIP graph")
    ap.add_argument("--conversion-ablation", action="store_true",
                    help="instead of the benchmark line: the int4->int8 conversion routes of the "
                         "per-group prefill GEMM on the cfg4 shape (Sec. 4.5.2, Fig. 9)")
    ap.add_argument("--front-end", action="store_true",
                    help="only the offline weight front-end lines (fp16 weights -> int4 codes + scales, repack)")
    ap.add_argument("--token-sweep", action="store_true",
                    help="instead of the benchmark line: the paper's N=8192, K=21760 token sweep")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2406_09904_amd import binding as qqq
    from paper_2406_09904_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qqq.lib()                                  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    wls = synth.workloads()
    if args.workload not in wls:
        print("unknown workload %s; choose from: %s" % (args.workload, ", ".join(wls)),
              file=sys.stderr)
        return 2

    use_graph = not args.eager
    if args.conversion_ablation:
        print(json.dumps({"conversion_ablation": conversion_ablation(torch, qqq, wls, use_graph)}), flush=True)
        return 0
    if args.front_end:
        print(json.dumps({"weight_front_end": front_end_lines(torch, qqq, synth, use_graph)}), flush=True)
        return 0
    if args.token_sweep:
        print(json.dumps({"token_sweep": token_sweep(torch, qqq, synth, use_graph)}), flush=True)
        return 0
    wl = wls[args.workload]
    case = Case(wl, torch, qqq)
    step_ms, gemm_ms, quant_ms, graphed = measure(case, torch, args.steps, args.warmup, use_graph)
    roof = roofline_for(case, step_ms, gemm_ms)
    roof["traffic"] = load_traffic(wl.name)
    out = {
        "metric": METRIC, "value": round(case.ops / (step_ms * 1e-3) / 1e12, 4), "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": wl.name, "variant": wl.variant, "M": wl.M, "K": wl.K, "N": wl.N,
                   "group": 128 if wl.variant == "pergroup" else None,
                   "step": "qqq_linear_w4a8_%s (%s)" % (
                       wl.variant, "one fused kernel" if case.fused else
                       "quant_act kernel + gemm kernel"),
                   "weight_copies_rotated": case.copies, "hip_graph": graphed,
                   "separate_quant_act_us": round(quant_ms * 1e3, 3),
                   "separate_gemm_us": round(gemm_ms * 1e3, 3)},
        "roofline": roof,
    }
    del case
    torch.cuda.empty_cache()

    if not args.no_sweep:
        sweep = []
        for name in SWEEP:
            if name == wl.name:
                continue
            w2 = wls[name]
            big = w2.M >= 1024
            c2 = Case(w2, torch, qqq, rotate_bytes=(1 << 28) if big else (1 << 30))
            st = max(5, min(args.steps, 20 if big else 100))
            s_ms, g_ms, q_ms, _ = measure(c2, torch, st, min(args.warmup, 5), use_graph)
            r2 = roofline_for(c2, s_ms, g_ms)
            r2["traffic"] = load_traffic(name)
            sweep.append({"workload": name, "steps": st, "ms_per_step": round(s_ms, 6),
                          "gemm_us": round(g_ms * 1e3, 3), "quant_act_us": round(q_ms * 1e3, 3),
                          "quant_act_gbs": round(quant_bytes(w2.M, w2.K) / (q_ms * 1e-3) / 1e9, 1),
                          "tops": round(c2.ops / (s_ms * 1e-3) / 1e12, 3),
                          "roofline": r2})
            del c2
            torch.cuda.empty_cache()
        out["sweep"] = sweep

    if not args.no_sweep:
        out["real_valued_group_scale"] = real_scale_lines(wls, torch, qqq, args, use_graph)

    if not args.no_sweep:
        out["weight_front_end"] = front_end_lines(torch, qqq, synth, use_graph)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
