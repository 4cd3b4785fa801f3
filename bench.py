#!/usr/bin/env python3
"""Benchmark of the W4A8 hot path (quantise activations -> W4A8 GEMM) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-sweep]
                  [--no-cpu-baseline] [--no-clock] [--eager]
                  [--ceilings | --token-sweep | --conversion-ablation | --front-end]

A step is one pass of the whole hot path over one batch of seeded synthetic input that is
already resident in HBM: per-token int8 quantisation of the fp16 activations, then the W4A8 GEMM
of the workload's variant, through the library's one-call entry point qqq_linear_w4a8_* (for a
few decode rows that is one fused kernel, otherwise qqq_quant_act's kernel followed by the GEMM
kernel; weights were repacked once, offline, outside the timed region).  The headline workload is
the largest single-GPU configuration (per-channel, M=4096 on the 28672 x 8192 layer); every other
configuration point of the benchmark is a line of the `sweep` array.

Cold-HBM protocol: packed weights (and group scales) exist in R copies whose total exceeds 1 GiB
(four times the 256 MiB last-level cache) and consecutive steps rotate through them; before every
timed replay a 512 MiB buffer is streamed through the chip (reads only), so a replay shorter than
one rotation starts cold too.
The K timed steps are captured once into a HIP graph (removes Python's launch overhead from
microsecond-scale kernels; --eager disables that), replayed untimed for about 30 ms so that the
clocks have left their idle state, and then replayed REPLAYS times, each replay timed with events on
the launch stream: ms_per_step is the median replay / K, min and max are reported beside it.  Prints ONE JSON line.
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
PRIMARY = "cfg5_pc_m4096_k8192_n28672"
# every configuration point of the benchmark (17), in the order of its five configurations
SWEEP = ["cfg1_pc_m16_k4096_n4096", "cfg2_pg_m1_k4096_n11008",
         "cfg3_pc_m1_k5120_n13824", "cfg3_pc_m8_k5120_n13824", "cfg3_pc_m32_k5120_n13824",
         "cfg3_pc_m128_k5120_n13824", "cfg3_pc_m512_k5120_n13824", "cfg3_pc_m2048_k5120_n13824",
         "cfg4_pg_m4096_k11008_n4096",
         "cfg5_pc_m1_k8192_n28672", "cfg5_pg_m1_k8192_n28672", "cfg5_pc_m16_k8192_n28672",
         "cfg5_pg_m16_k8192_n28672", "cfg5_pc_m256_k8192_n28672", "cfg5_pg_m256_k8192_n28672",
         "cfg5_pc_m4096_k8192_n28672", "cfg5_pg_m4096_k8192_n28672"]
REPLAYS = 5                    # timed replays of the captured graph (min / median / max reported)
FLUSH_BYTES = 512 << 20        # read before every timed replay: twice the last-level cache
WARM_MS = 30.0                 # untimed graph replays before the timed ones (clock ramp-up)
ORACLE_FULL_MACS = 2e11        # the oracle runs the whole product up to this size, a row subset beyond


def algorithmic_bytes(M, N, K, pergroup):
    """What the method itself must move once: packed int4 weights, group scales, fp16 channel
    scales, int8 activations, fp32 token scales, fp16 output."""
    return N * K // 2 + (K // 128 * N if pergroup else 0) + 2 * N + M * K + 4 * M + 2 * M * N


def quant_bytes(M, K):
    return 2 * M * K + M * K + 4 * M


def fused_bytes(M, N, K, pergroup):
    """Algorithmic bytes of the fused decode kernel: fp16 activations in, no int8 round trip."""
    return N * K // 2 + (K // 128 * N if pergroup else 0) + 2 * N + 2 * M * K + 2 * M * N


class Case:
    """Device-resident inputs of one workload plus the launch closures."""

    def __init__(self, wl, torch, qqq, rotate_bytes=1 << 30, max_copies=128):
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
        # the GEMM-only timing reads a_q/s_a: fill them with the workload's real codes first (MFMA
        # power, hence clock and speed, depends on the operand values)
        self.quant()
        # which kernels the library runs for this workload: asked, not re-derived
        self.gemm(0)
        self.gemm_route = qqq.last_route()
        self.step(0)
        self.step_route = qqq.last_route()
        self.fused = "fused=1" in self.step_route
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


_flush = None


def flush_cache(torch, qqq=None):
    """Streams a 512 MiB buffer through the chip with plain reads (the library's ceiling probe):
    whatever the 256 MiB last-level cache held is gone, and nothing dirty is left behind whose
    write-back would compete with the timed kernels (a rewritten buffer would do that)."""
    global _flush
    from paper_2406_09904_amd import binding
    if _flush is None:
        _flush = (torch.zeros((FLUSH_BYTES,), dtype=torch.uint8, device="cuda"),
                  torch.zeros((4,), dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
    binding.probe_stream_read(_flush[0], FLUSH_BYTES, 2048, _flush[1])


def timed(torch, fn, steps, warmup, use_graph, replays=REPLAYS):
    """fn(i) enqueues one unit of work on the current stream.  The `steps` units are captured once
    into a graph and replayed `replays` times (eager: re-issued), each replay preceded by a cache
    flush and timed with events on that stream between two synchronisations.  Returns
    ({"median","min","max"} in ms per unit, graph used?)."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    graph = None
    if use_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(steps):
                    fn(warmup + i)
            w0 = torch.cuda.Event(enable_timing=True)
            w1 = torch.cuda.Event(enable_timing=True)
            w0.record()
            graph.replay()           # untimed replay: graph upload
            w1.record()
            torch.cuda.synchronize()
            # more untimed replays until the chip has been busy for ~WARM_MS: after the host-side
            # set-up of a workload the clocks sit at idle, and the first milliseconds of work run slower
            more = int(min(200, WARM_MS / max(w0.elapsed_time(w1), 1e-3)))
            for _ in range(more):
                graph.replay()
            torch.cuda.synchronize()
        except Exception as ex:      # capture unsupported: fall back to eager launches
            print("bench: graph capture failed (%s); timing eager launches" % ex, file=sys.stderr)
            graph = None
            torch.cuda.synchronize()
    per = []
    for r in range(max(1, replays)):
        flush_cache(torch)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        if graph is not None:
            graph.replay()
        else:
            for i in range(steps):
                fn(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        per.append(e0.elapsed_time(e1) / steps)
    per.sort()
    return {"median": per[len(per) // 2], "min": per[0], "max": per[-1]}, graph is not None


def timed_ms(torch, fn, steps, warmup, use_graph):
    """Median ms per unit over three flushed replays (the secondary tables)."""
    return timed(torch, fn, steps, warmup, use_graph, replays=3)[0]["median"]


def roofline_for(case, step_ms, gemm_ms):
    """Roofline of the step's dominant kernel: the fused kernel (= the whole step) where
    qqq_linear_* fuses, the GEMM kernel (timed back to back alone) otherwise.  Bound: whichever of
    algorithmic bytes / 8 TB/s and 2MNK / 5.03 POP/s is the longer time."""
    wl = case.wl
    if case.fused:
        kernel, kernel_ms = case.step_route, step_ms
        nbytes = fused_bytes(wl.M, wl.N, wl.K, case.pg)
    else:
        kernel, kernel_ms, nbytes = case.gemm_route, gemm_ms, case.bytes
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
    # the benchmark's own targets: 70 % of HBM at M <= 16, 60 % of int8 MFMA peak at M >= 1024
    if wl.M <= 16:
        roof["target"] = {"frac": 0.70, "of": "hbm", "met": bool(roof["bound"] == "hbm" and roof["frac"] >= 0.70)}
    elif wl.M >= 1024:
        roof["target"] = {"frac": 0.60, "of": "mfma", "met": bool(roof["bound"] == "mfma" and roof["frac"] >= 0.60)}
    else:
        roof["target"] = None
    return roof


def load_profile_json(fname, name):
    try:
        with open(os.path.join(ROOT, "profiles", fname)) as f:
            return json.load(f).get(name)
    except (OSError, ValueError, TypeError):
        return None


def load_traffic(name):
    """HBM bytes per GEMM launch from the rocprofv3 --pmc summaries under profiles/, if present."""
    rec = load_profile_json("traffic.json", name)
    try:
        return int(rec["fetch_bytes"]) + int(rec["write_bytes"]) if rec else None
    except (KeyError, TypeError, ValueError):
        return None


def load_mfma_counters(name, kernel_us):
    """int8 MFMA utilisation of the dominant kernel from the SQ counter summaries under profiles/
    (SQ_INSTS_VALU_MFMA_MOPS_I8 * 512 operations per launch, SQ_VALU_MFMA_BUSY_CYCLES), where a
    run for this workload was recorded: counted operations / (this run's kernel time * nominal peak)."""
    rec = load_profile_json("mfma_counters.json", name)
    if not rec:
        return None
    try:
        out = {"counted_ops": int(rec["mops_i8"]) * 512,
               "util_vs_nominal": round(int(rec["mops_i8"]) * 512 / (kernel_us * 1e-6) / (MFMA_I8_PEAK_TOPS * 1e12), 4)}
        if "mfma_pipe_busy_frac" in rec:
            out["mfma_pipe_busy_frac_profiled"] = rec["mfma_pipe_busy_frac"]
        if "avg_clock_ghz" in rec:
            out["avg_clock_ghz_profiled"] = rec["avg_clock_ghz"]
        return out
    except (KeyError, TypeError, ValueError):
        return None


def measure(case, torch, steps, warmup, use_graph):
    step, graphed = timed(torch, case.step, steps, warmup, use_graph)
    gemm, _ = timed(torch, case.gemm, steps, warmup, use_graph)
    quant, _ = timed(torch, lambda i: case.quant(), steps, warmup, use_graph)
    return step, gemm, quant, graphed


def workload_line(case, torch, steps, warmup, use_graph):
    """One configuration point: step / GEMM / quantiser times, roofline of the dominant kernel."""
    wl = case.wl
    step, gemm, quant, graphed = measure(case, torch, steps, warmup, use_graph)
    roof = roofline_for(case, step["median"], gemm["median"])
    roof["traffic"] = load_traffic(wl.name)
    line = {"workload": wl.name, "variant": wl.variant, "M": wl.M, "K": wl.K, "N": wl.N,
            "steps": steps, "replays": REPLAYS, "weight_copies_rotated": case.copies, "hip_graph": graphed,
            "ms_per_step": round(step["median"], 6),
            "ms_per_step_min": round(step["min"], 6), "ms_per_step_max": round(step["max"], 6),
            "step_route": case.step_route, "gemm_route": case.gemm_route,
            "gemm_us": round(gemm["median"] * 1e3, 3), "gemm_us_min": round(gemm["min"] * 1e3, 3),
            "gemm_us_max": round(gemm["max"] * 1e3, 3),
            "quant_act_us": round(quant["median"] * 1e3, 3),
            "quant_act_gbs": round(quant_bytes(wl.M, wl.K) / (quant["median"] * 1e-3) / 1e9, 1),
            "tops": round(case.ops / (step["median"] * 1e-3) / 1e12, 3),
            "roofline": roof}
    if roof["bound"] == "mfma":
        line["mfma_util"] = load_mfma_counters(wl.name, roof["kernel_us"])
    return line


def sample_clock(torch, case):
    """Shader clock (rocm-smi) and socket power (amd-smi) while the workload's GEMM runs back to back
    for a few seconds, and once more when idle, plus the board's power limit.  None where the tools
    are missing or unreadable.  The int8 MFMA kernels run this GPU at its power limit, which is what
    sets their clock."""
    import re
    import subprocess

    def tool(args, pattern):
        try:
            r = subprocess.run(args, capture_output=True, text=True, timeout=20)
            m = re.search(pattern, r.stdout)
            return float(m.group(1)) if m else None
        except (OSError, subprocess.SubprocessError):
            return None

    def read():
        return (tool(["rocm-smi", "--showclocks"], r"sclk clock level:\s*\d+:\s*\((\d+)Mhz\)"),
                tool(["amd-smi", "metric", "--power"], r"SOCKET_POWER:\s*([0-9.]+)\s*W"))

    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(10):
                case.gemm(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        reps = int(max(1, min(200000, 5000.0 / max(e0.elapsed_time(e1), 1e-3))))
        for _ in range(reps):                       # ~5 s of queued work; the host does not wait
            graph.replay()
        time.sleep(1.2)
        busy = read()
        torch.cuda.synchronize()
    except Exception as ex:                         # noqa: BLE001 - a diagnostic, never fatal
        print("bench: clock sampling failed (%s)" % ex, file=sys.stderr)
        return None
    time.sleep(4.0)                                 # the power reading is an average over the last seconds
    idle = read()
    cap = tool(["rocm-smi", "--showmaxpower"], r"Max Graphics Package Power \(W\):\s*([0-9.]+)")
    return {"sclk_mhz_during_gemm": busy[0], "sclk_mhz_idle": idle[0], "nominal_mhz": 2400,
            "socket_power_w_during_gemm": busy[1], "socket_power_w_idle": idle[1], "power_limit_w": cap,
            "source": "rocm-smi --showclocks / amd-smi metric --power, one reading while %s's GEMM is replayed "
                      "back to back" % case.wl.name}


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
        ms = timed_ms(torch, gemm, st, min(args.warmup, 5), use_graph)
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
        ms = timed_ms(torch, fn, 20, 5, use_graph)
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

    def pg_sym18(i):
        qqq.qqq_gemm_w4a8_pergroup(c.a_q, c.s_a, c.w[i % c.copies], c.s_g[i % c.copies], c.s_w, c.ws,
                                   sg_max=18 | qqq.SG_SYMMETRIC_CODES, y=c.y)

    rows.append({"route": "integer scale <= 18, codes promised in [-7,7] (the front-end's output): packed 16-bit "
                          "multiply of 7 - code, bias and sign removal (default)", "gemm_us": t(pg_sym18)})
    qqq.set_group_mode_override(3)
    rows.append({"route": "integer scale <= 18, codes promised in [-7,7]: fp16 FMA route", "gemm_us": t(pg_sym18)})
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
            ms = timed_ms(torch, fn, 10, 2, use_graph)
            rows.append({"layer": name, "N": N, "K": K, "kernel": "quant_weight_kernel (%s)" % variant,
                         "us": round(ms * 1e3, 1), "bound": "hbm",
                         "achieved_gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "frac": round(nbytes / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9), 3)})
        w_nat, _ = qqq.qqq_quantize_w4_perchannel(w)
        out = qqq.qqq_pack_w4(w_nat, K)
        ms = timed_ms(torch, lambda i: qqq.qqq_pack_w4(w_nat, K, out=out), 10, 2, use_graph)
        rows.append({"layer": name, "N": N, "K": K, "kernel": "pack_w4", "us": round(ms * 1e3, 1), "bound": "hbm",
                     "achieved_gbs": round(N * K / (ms * 1e-3) / 1e9, 1),
                     "frac": round(N * K / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9), 3)})
        del w, w_nat, out
        torch.cuda.empty_cache()
    return rows


def offline_stage_lines(torch, qqq, synth):
    """The offline stage on one synthetic layer (include/qqq_calib.h): adaptive smoothing with a 16-point
    grid (Sec. 3.1) and Hessian-based compensation (Sec. 3.2).  Calibration-time code: wall time per
    call with events, eager launches (thousands of small kernels; no roofline is claimed for it)."""
    import numpy as np
    rows = []

    def wall(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return round(e0.elapsed_time(e1), 3)

    M, K, N = 512, 4096, 4096
    x = torch.from_numpy(synth.activations_fp16(M, K, 301)).cuda()
    w = torch.from_numpy(synth.weights_fp16(N, K, 302).view(np.int16)).cuda().view(torch.float16)
    rows.append({"call": "qqq_adaptive_smoothing", "M": M, "K": K, "N": N, "grid_points": 16,
                 "ms": wall(lambda: qqq.qqq_adaptive_smoothing(x, w, 16))})
    rows.append({"call": "qqq_hessian", "M": M, "K": K, "ms": wall(lambda: qqq.qqq_hessian(x))})
    K2, N2 = 1024, 4096
    x2 = torch.from_numpy(synth.activations_fp16(M, K2, 303)).cuda()
    w2 = torch.from_numpy(synth.weights_fp16(N2, K2, 304).view(np.int16)).cuda().view(torch.float16)
    H = qqq.qqq_hessian(x2)
    rows.append({"call": "qqq_gptq_quantize_w4_perchannel", "K": K2, "N": N2,
                 "ms": wall(lambda: qqq.qqq_gptq_quantize_w4_perchannel(w2, H, 0.01))})
    rows.append({"call": "qqq_gptq_quantize_w4_pergroup", "K": K2, "N": N2,
                 "ms": wall(lambda: qqq.qqq_gptq_quantize_w4_pergroup(w2, H, 0.01))})
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
            ms = timed_ms(torch, fn, st, 3, use_graph)
            row[key] = round(ms * 1e3, 2)
        row["speedup_perchannel_vs_fp16"] = round(row["fp16_matmul_us"] / row["perchannel_us"], 2)
        row["speedup_pergroup_vs_fp16"] = round(row["fp16_matmul_us"] / row["pergroup_us"], 2)
        rows.append(row)
        print("token sweep M=%d: %s" % (M, row), file=sys.stderr, flush=True)
    return {"shape": {"N": N, "K": K}, "note": "GEMM kernel only, HIP graph replay, weight copies "
            "rotated (12 x 85 MiB); fp16_matmul is torch.matmul on fp16 weights (3 copies rotated)",
            "rows": rows}


def host_cores():
    cores = os.cpu_count() or 1
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        pass
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        cores = min(cores, int(env))
    return cores


def oracle_rows(wl):
    """Rows the oracle takes for a workload: all of them up to ORACLE_FULL_MACS multiply-accumulates,
    else the first, one interior and the last 128-row tile plus 64 seeded random rows (all N columns)."""
    import numpy as np
    if float(wl.M) * wl.N * wl.K <= ORACLE_FULL_MACS:
        return np.arange(wl.M), "all %d rows" % wl.M
    g = np.random.default_rng(wl.seed + 11)
    interior = 128 * int(g.integers(1, wl.M // 128 - 1))
    rows = np.unique(np.concatenate([np.arange(0, 128), np.arange(interior, interior + 128),
                                     np.arange(wl.M - 128, wl.M), g.integers(0, wl.M, 64)]))
    return rows, "%d of %d rows (row tiles at 0, %d and %d plus 64 random rows)" % (
        len(rows), wl.M, interior, wl.M - 128)


def oracle_time(wl):
    """One pass of the oracle as it stands (gcc -O2 -fopenmp, int64 accumulation, no blocking) over
    the whole path of a workload on this machine's host cores: quant_act + the variant's GEMM + Dequant
    on the rows of oracle_rows(), all N columns.  Returns seconds and the sample description."""
    import numpy as np
    from oracle import qqq_oracle as orc
    rows, what = oracle_rows(wl)
    a = np.ascontiguousarray(wl.activations()[rows])
    w_nat, s_w = wl.w_nat(), wl.s_w().view(np.uint16)
    s_g = wl.s_g() if wl.variant == "pergroup" else None
    orc.lib()
    t0 = time.perf_counter()
    a_q, s_a = orc.quant_act(a.view(np.uint16))
    if s_g is None:
        orc.gemm_perchannel(a_q, s_a, w_nat, s_w)
    else:
        orc.gemm_pergroup(a_q, s_a, w_nat, s_g, s_w)
    return time.perf_counter() - t0, len(rows), what


def cpu_baseline(wls, names, headline):
    """The oracle timed on this machine's host cores beside the GPU numbers: one pass per configuration
    point (bounded: the two M=4096 points on the 28672 x 8192 layer run a stated row subset and their
    time is extrapolated by M / rows).  `value` is the headline workload's rate."""
    cores = host_cores()
    per = {}
    for name in names:
        wl = wls[name]
        sec, nrows, what = oracle_time(wl)
        macs = float(nrows) * wl.N * wl.K
        rec = {"seconds": round(sec, 3), "rows": nrows, "gmac_per_s": round(macs / sec / 1e9, 2),
               "extrapolated": nrows != wl.M}
        if nrows != wl.M:
            rec["seconds_full_extrapolated"] = round(sec * wl.M / nrows, 1)
        per[name] = rec
        print("oracle %s: %.2f s on %s" % (name, sec, what), file=sys.stderr, flush=True)
    wl = wls[headline]
    h = per[headline]
    _, what = oracle_rows(wl)
    return {"value": round(2.0 * h["rows"] * wl.N * wl.K / h["seconds"] / 1e12, 6), "unit": "TOPS",
            "cores": cores, "kind": "oracle",
            "sample": "one pass of quant_act + %s GEMM + Dequant of %s on %s, all N=%d columns, K=%d: %.1f s wall; "
                      "the whole workload would take about %.0f s (extrapolated by M/rows)" % (
                          wl.variant, wl.name, what, wl.N, wl.K, h["seconds"],
                          h.get("seconds_full_extrapolated", h["seconds"])),
            "per_workload": per}


def ceilings(torch, qqq, synth):
    """What this GPU gives plain kernels of the path's shape (include/qqq_tuning.h probes): a
    streaming read of the benchmark's weight sizes, an empty launch, and the int8 MFMA pipe with the
    prefill kernel's register dataflow on operand values of several kinds (the clock under MFMA
    load depends on them)."""
    import numpy as np
    out = {}
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    buf = torch.ones((2 << 30,), dtype=torch.uint8, device="cuda")
    rows = []
    for mib in (8, 23, 35, 117, 1024):
        nbytes = mib << 20
        nrot = buf.numel() // nbytes
        for wgs in (256, 512, 1024, 2048, 4096):
            steps = 100 if mib < 1024 else 6

            def fn(i, nbytes=nbytes, nrot=nrot, wgs=wgs):
                qqq.probe_stream_read(buf, nbytes, wgs, sink, offset=(i % nrot) * nbytes)

            ms = timed_ms(torch, fn, steps, 5, True)
            rows.append({"mib": mib, "workgroups": wgs, "us": round(ms * 1e3, 2),
                         "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1)})
    out["stream_read"] = rows
    ms = timed_ms(torch, lambda i: qqq.probe_stream_read(buf, 16, 1, sink), 200, 10, True)
    out["empty_launch_us"] = round(ms * 1e3, 2)
    del buf
    torch.cuda.empty_cache()
    # operand values: the headline workload's quantised activations, weights as the kernels feed them
    wl = synth.workloads()[PRIMARY]
    a_q, _ = qqq.qqq_quant_act(torch.from_numpy(wl.activations()[:64]).cuda())
    aq = a_q.cpu().numpy().reshape(-1)
    g = np.random.default_rng(1)
    na, nb = 4 * 4 * 512 * 16, 2 * 2 * 512 * 16
    codes = g.integers(-8, 8, nb).astype(np.int8)
    A = {"zero": np.zeros(na, np.int8), "workload activations": aq[:na].copy(),
         "uniform int8": g.integers(-127, 128, na).astype(np.int8)}
    B = {"zero": np.zeros(nb, np.int8), "16 x code (FastINT4toINT8)": (codes.astype(np.int16) * 16).astype(np.int8),
         "code + 8 (offset binary)": (codes + 8).astype(np.int8), "uniform int8": g.integers(-128, 128, nb).astype(np.int8)}
    rows = []
    for an, bn in (("zero", "zero"), ("workload activations", "16 x code (FastINT4toINT8)"),
                   ("workload activations", "code + 8 (offset binary)"), ("uniform int8", "uniform int8")):
        da, db = torch.from_numpy(A[an]).cuda(), torch.from_numpy(B[bn]).cuda()
        iters = 3000
        ms = timed_ms(torch, lambda i: qqq.probe_mfma_i8(da, db, iters, 256, sink), 1, 1, False)
        ops = 256 * 8 * iters * 4 * 8 * 65536.0
        rows.append({"activations": an, "weights": bn, "ms": round(ms, 3), "tops": round(ops / ms / 1e9, 1),
                     "frac_of_nominal": round(ops / ms / 1e9 / MFMA_I8_PEAK_TOPS, 4)})
    out["mfma_i8_only"] = rows
    # the prefill kernel's k-loop, part by part, on the headline workload's own bytes: activation
    # tiles (128 rows x 128 k) cut from its quantised activations, packed codes as they lie in memory
    w_packed = qqq.qqq_pack_w4(torch.from_numpy(wl.w_nat().view(np.int32)).cuda(), wl.K)
    a_all, _ = qqq.qqq_quant_act(torch.from_numpy(wl.activations()[:512]).cuda())
    wgs, stages = 256, 2
    a_tiles = a_all.view(4, 128, wl.K // 128, 128).permute(0, 2, 1, 3).reshape(-1, 16384)
    reps = (wgs * stages + a_tiles.shape[0] - 1) // a_tiles.shape[0]
    a_tiles = a_tiles.repeat(reps, 1)[:wgs * stages].contiguous().view(torch.uint8)
    w_bytes = w_packed.view(torch.uint8).reshape(-1)[:wgs * stages * 32768].view(wgs * stages, 32768)
    src = torch.zeros((wgs * stages, qqq.PROBE_LOOP_STAGE), dtype=torch.uint8, device="cuda")
    src[:, :16384] = a_tiles
    src[:, 16384:49152] = w_bytes
    region = stages * qqq.PROBE_LOOP_STAGE
    A, W, C, D = qqq.PROBE_A_READS, qqq.PROBE_W_READS, qqq.PROBE_CONVERT, qqq.PROBE_DMA
    rows = []
    steps = 3000
    for parts, name in ((0, "MFMAs only: operands stay in registers, conversion hoisted"),
                        (C, "+ int4 -> int8 conversion every k-step"),
                        (A, "+ activation fragments from LDS"),
                        (W | C, "+ packed codes from LDS and their conversion"),
                        (D, "+ DMA ring refill, wait and barrier"),
                        (A | W | C, "all LDS reads and the conversion"),
                        (A | W | C | D, "the whole k-loop"),
                        (qqq.PROBE_FORM_32X32X32, "32x32x32 form: MFMAs only"),
                        (qqq.PROBE_FORM_32X32X32 | A | W | C | D, "32x32x32 form: the whole k-loop")):
        ms = min(timed_ms(torch, lambda i, parts=parts: qqq.probe_prefill_loop(src, region, steps, parts, wgs, sink),
                          1, 1, False) for _ in range(3))
        ops = wgs * 8 * steps * 32 * 65536.0   # 128 x 64 x 128 multiply-accumulates per wave and k-step
        rows.append({"parts": name, "ms": round(ms, 3),
                     "frac_of_nominal": round(ops / ms / 1e9 / MFMA_I8_PEAK_TOPS, 4)})
    base = 1.0 / rows[0]["frac_of_nominal"]
    for r in rows:
        r["time_per_mac_vs_first_row"] = round(1.0 / r["frac_of_nominal"] / base, 3)
    # the same loop on constant bytes draws little power: the clock stays near nominal and the
    # fraction is the MFMA pipe's busy share, i.e. what the loop loses as a schedule
    src.fill_(0x12)
    for parts, name in ((0, "constant bytes: MFMAs only"), (A | W | C | D, "constant bytes: the whole k-loop")):
        ms = min(timed_ms(torch, lambda i, parts=parts: qqq.probe_prefill_loop(src, region, steps, parts, wgs, sink),
                          1, 1, False) for _ in range(3))
        rows.append({"parts": name, "ms": round(ms, 3),
                     "frac_of_nominal": round(wgs * 8 * steps * 32 * 65536.0 / ms / 1e9 / MFMA_I8_PEAK_TOPS, 4)})
    out["prefill_loop_parts"] = rows
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=PRIMARY)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time eager launches, no HIP graph")
    ap.add_argument("--conversion-ablation", action="store_true",
                    help="instead of the benchmark line: the int4->int8 conversion routes of the "
                         "per-group prefill GEMM on the cfg4 shape (Sec. 4.5.2, Fig. 9)")
    ap.add_argument("--front-end", action="store_true",
                    help="only the offline weight front-end lines (fp16 weights -> int4 codes + scales, repack)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark line: measured ceilings of this GPU (streaming read per "
                         "size and launch width, empty launch, int8 MFMA pipe per operand-value kind)")
    ap.add_argument("--no-clock", action="store_true", help="skip the rocm-smi clock reading")
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
    if args.ceilings:
        print(json.dumps({"ceilings": ceilings(torch, qqq, synth)}), flush=True)
        return 0
    wl = wls[args.workload]
    case = Case(wl, torch, qqq)
    head = workload_line(case, torch, args.steps, args.warmup, use_graph)
    clocks = None if args.no_clock else sample_clock(torch, case)
    roof = head["roofline"]
    out = {
        "metric": METRIC, "value": head["tops"], "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "ms_per_step_min": head["ms_per_step_min"],
        "ms_per_step_max": head["ms_per_step_max"], "replays": REPLAYS,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": wl.name, "variant": wl.variant, "M": wl.M, "K": wl.K, "N": wl.N,
                   "group": 128 if wl.variant == "pergroup" else None,
                   "step": "qqq_linear_w4a8_%s: %s" % (wl.variant, head["step_route"]),
                   "weight_copies_rotated": case.copies, "hip_graph": head["hip_graph"],
                   "cache_flush_before_each_replay_bytes": FLUSH_BYTES,
                   "separate_quant_act_us": head["quant_act_us"],
                   "separate_gemm_us": head["gemm_us"]},
        "roofline": roof,
        "clocks": clocks,
    }
    if "mfma_util" in head:
        out["mfma_util"] = head["mfma_util"]
    del case
    torch.cuda.empty_cache()

    names = [wl.name]
    if not args.no_sweep:
        sweep = []
        for name in SWEEP:
            if name == wl.name:
                sweep.append(dict(head, note="the headline line"))
                continue
            w2 = wls[name]
            c2 = Case(w2, torch, qqq)
            # graph length: for the short kernels a whole rotation of the weight copies and at least
            # 100 steps, so that what a replay pays once after the cache flush (address translation,
            # the first wave of workgroups) is spread over enough steps to read as per-step time
            st = max(5, min(args.steps, 20)) if w2.M >= 256 else max(args.steps, min(c2.copies, 128), 100)
            sweep.append(workload_line(c2, torch, st, min(args.warmup, 5), use_graph))
            print("bench %s: %.2f us/step, roofline %.3f (%s)" % (
                name, sweep[-1]["ms_per_step"] * 1e3, sweep[-1]["roofline"]["frac"],
                sweep[-1]["roofline"]["bound"]), file=sys.stderr, flush=True)
            del c2
            torch.cuda.empty_cache()
            names.append(name)
        out["sweep"] = sweep
        met = [l["workload"] for l in sweep if l["roofline"]["target"] and l["roofline"]["target"]["met"]]
        tgt = [l["workload"] for l in sweep if l["roofline"]["target"]]
        out["targets"] = {"met": len(met), "of": len(tgt), "met_workloads": met}
        out["real_valued_group_scale"] = real_scale_lines(wls, torch, qqq, args, use_graph)
        out["weight_front_end"] = front_end_lines(torch, qqq, synth, use_graph)
        out["offline_stage"] = offline_stage_lines(torch, qqq, synth)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wls, names, wl.name)
        if "sweep" in out:
            for l in out["sweep"]:
                l["oracle"] = out["cpu_baseline"]["per_workload"].get(l["workload"])
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
