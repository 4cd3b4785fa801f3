// Ceiling probes for the benchmark (bench.py --ceilings).  Not part of the W4A8 path: two plain
// kernels that measure what this GPU gives a kernel of the path's shape, so that the roofline
// fractions of the real kernels can be read against a measured ceiling next to the nominal one.
//   stream read : 128-bit coalesced loads of a contiguous buffer, nothing else (decode shapes)
//   int8 MFMA   : the prefill kernel's register dataflow (8 waves, 4 x 2 tiles of 32x32x32 per
//                 wave, two waves per SIMD) with no memory traffic in the loop; the operand
//                 VALUES come from the caller, because the chip's clock under MFMA load depends on them
//   prefill loop: the persistent prefill kernel's k-loop (per-channel) on caller-supplied bytes, in its
//                 v_mfma_i32_16x16x64_i8 form or in the 32x32x32 form for comparison, with its
//                 parts switched on one by one (LDS fragment reads, int4 -> int8 conversion, the DMA
//                 ring and its barrier).  Under MFMA load this GPU runs at its board power limit, so
//                 what each part costs is its energy, not its issue slots: the probe prices them
#include "qqq_prefill_common.h"

// The DMA helper names M0 as clobbered; the compiler remarks on clobber lists that name a reserved register.
#pragma clang diagnostic ignored "-Winline-asm"

namespace qqq {

template <int UNROLL>
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const uint4* __restrict__ p, size_t nvec,
                                                                uint32_t* sink) {
  uint32_t acc = 0;
  const size_t step = (size_t)gridDim.x * 256 * UNROLL;
  for (size_t i = (size_t)blockIdx.x * 256 * UNROLL + threadIdx.x; i < nvec; i += step) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t j = i + 256 * u;
      v[u] = (j < nvec) ? p[j] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) sink[0] = acc;  // keeps the loads alive; practically never true
}

constexpr int kPoolA = 4, kPoolB = 2;  // distinct operand sets the MFMAs rotate through

__global__ __launch_bounds__(512, 1) void probe_mfma_i8_kernel(int iters, const v4i* a_pool, const v4i* b_pool,
                                                              int32_t* sink) {
  v4i a[kPoolA][4], b[kPoolB][2];
#pragma unroll
  for (int i = 0; i < kPoolA; ++i)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) a[i][mt] = a_pool[(i * 4 + mt) * 512 + threadIdx.x];
#pragma unroll
  for (int i = 0; i < kPoolB; ++i)
#pragma unroll
    for (int c = 0; c < 2; ++c) b[i][c] = b_pool[(i * 2 + c) * 512 + threadIdx.x];
  v16i acc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < kPoolA; ++s)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
          acc[mt][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[s][mt], b[s % kPoolB][c], acc[mt][c], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[mt][c][v];
  if (s == 0x7fffffff && iters < 0) sink[0] = s;  // never true: iters >= 1
}

// One workgroup = the persistent kernel's 8 waves and 3-stage ring (50 KiB per stage: 16 KiB of
// activations, 8 x 4 KiB of packed codes, 2 KiB unused).  `region` bytes per workgroup (a multiple
// of the 50 KiB step) are walked cyclically by the DMA part; without it the ring keeps the
// region's first bytes.  PARTS: see qqq_tuning.h.
constexpr int kLoopAStage = 16384, kLoopWWave = 4096, kLoopStage = 51200;

template <int PARTS>
__global__ __launch_bounds__(512, 1) void probe_prefill_loop_kernel(int steps, const int8_t* src, uint32_t region,
                                                                   int32_t* sink) {
  constexpr bool kAReads = PARTS & QQQ_PROBE_A_READS, kWReads = PARTS & QQQ_PROBE_W_READS;
  constexpr bool kConvert = PARTS & (QQQ_PROBE_CONVERT | QQQ_PROBE_W_READS), kDma = PARTS & QQQ_PROBE_DMA;
  __shared__ __attribute__((aligned(1024))) int8_t lds[3 * kLoopStage];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int8_t* base = src + (size_t)blockIdx.x * region;
  for (int i = tid; i < 3 * kLoopStage / 4; i += 512) ((int*)lds)[i] = ((const int*)base)[i % (region / 4)];
  __syncthreads();
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  const uint32_t wave_u = (uint32_t)__builtin_amdgcn_readfirstlane(wave);
  uint32_t soff = 0;  // wave-uniform position of the DMA cursor in the region
  const uint32_t a_voff = (uint32_t)(2 * wave * 1024 + lane * 16);
  const uint32_t w_voff = (uint32_t)(kLoopAStage + wave * kLoopWWave + lane * 16);
  auto dma_piece = [&](int stage, int piece) {
    if constexpr (kDma) {
      const uint32_t dst = lds_base + (uint32_t)stage * kLoopStage +
                           (piece < 2 ? (2 * wave_u + piece) * 1024 : kLoopAStage + wave_u * kLoopWWave + (piece - 2) * 1024);
      const int8_t* b = base + soff + (piece < 2 ? piece : piece - 2) * 1024;
      const uint32_t voff = piece < 2 ? a_voff : w_voff;
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(b) : "memory", "m0");
    }
  };
  auto advance = [&]() {
    soff += kLoopStage;
    if (soff >= region) soff = 0;
  };
  auto wait_step = [&]() {  // as the kernel: all but the newest k-step's six loads have landed, then the barrier
    if constexpr (kDma) asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  };
  for (int st = 0; st < 2; ++st) {
#pragma unroll
    for (int piece = 0; piece < 6; ++piece) dma_piece(st, piece);
    advance();
  }
  wait_step();
  int stage = 0;
  int s = 0;
  if constexpr (!(PARTS & QQQ_PROBE_FORM_32X32X32)) {
    // the kernels' loop: 16 slots of four v_mfma_i32_16x16x64_i8, fragments three slots ahead, barrier
    // before the last three slots, scheduling barrier per slot
    const int r16 = lane & 15, kb = lane >> 4;
    int a_off[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) a_off[q] = r16 * 128 + (((4 * q + kb) ^ ((r16 >> 1) & 7)) << 4);
    const int w_off = kLoopAStage + wave * kLoopWWave + lane * 16;
    v4i acc[8][4];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[mt][c] = (v4i){0, 0, 0, 0};
    v4i wq[4];
    auto read_w = [&](const int8_t* sb) {
#pragma unroll
      for (int c = 0; c < 4; ++c) wq[c] = *(const v4i*)(sb + w_off + c * 1024);
    };
    auto read_a = [&](const int8_t* sb, int slot) {
      return *(const v4i*)(sb + a_off[slot >> 3] + (slot & 7) * 2048);
    };
    auto make_b = [&](int c, int q) {
      v4i pc = wq[c];
      // without this the conversion of loop-invariant codes is hoisted out of the loop
      if constexpr (kConvert && !kWReads) asm volatile("" : "+v"(pc));
      return q ? convert_b<kPerChannel>((uint32_t)pc[2], (uint32_t)pc[3], 0)
               : convert_b<kPerChannel>((uint32_t)pc[0], (uint32_t)pc[1], 0);
    };
    constexpr int kAhead = 3;
    v4i abuf[4], afix[4], b0[4], b1[4];
    read_w(lds);
#pragma unroll
    for (int i = 0; i < 4; ++i) afix[i] = read_a(lds, i);  // operands that stay in registers when A_READS is off
#pragma unroll
    for (int i = 0; i < kAhead; ++i) abuf[i] = read_a(lds, i);
#pragma unroll
    for (int c = 0; c < 4; ++c) b0[c] = make_b(c, 0);
    for (int t = 0; t < steps; ++t) {
      const int dstage = stage == 0 ? 2 : stage - 1;
      const int nstage = stage == 2 ? 0 : stage + 1;
      const int8_t* sb = lds + stage * kLoopStage;
      const int8_t* nb = lds + nstage * kLoopStage;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (i == 16 - kAhead) {
          advance();
          wait_step();
          if constexpr (kWReads) read_w(nb);
        }
        if constexpr (kAReads)
          abuf[(i + kAhead) & 3] = (i + kAhead < 16) ? read_a(sb, i + kAhead) : read_a(nb, i + kAhead - 16);
        if (i < 6) dma_piece(dstage, i);
        if (i >= 2 && i < 6) b1[i - 2] = make_b(i - 2, 1);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc[i & 7][c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(kAReads ? abuf[i & 3] : afix[i & 3], i < 8 ? b0[c] : b1[c],
                                                                acc[i & 7][c], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) b0[c] = make_b(c, 0);
      stage = nstage;
    }
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v) s += acc[mt][c][v];
  } else {
    // the same wave patch with 4 x 2 tiles of v_mfma_i32_32x32x32_i8 (the per-tile kernel's 4-wave loop,
    // compiler-scheduled), for comparison: twice the accumulator bytes per multiply-accumulate
    const int n32 = lane & 31, h = lane >> 5;
    int a_off[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) a_off[q] = n32 * 128 + (((2 * q + h) ^ ((n32 >> 1) & 7)) << 4);
    const int w_off = kLoopAStage + wave * kLoopWWave + (n32 >> 4) * 1024 + ((n32 & 15) + 16 * h) * 16;
    v16i acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0;
    v4i wq[2][2];
    auto read_w = [&](const int8_t* sb) {
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        wq[c][0] = *(const v4i*)(sb + w_off + c * 2048);
        wq[c][1] = *(const v4i*)(sb + w_off + c * 2048 + 512);
      }
    };
    auto read_a = [&](v4i (&a)[4], const int8_t* sb, int q) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) a[mt] = *(const v4i*)(sb + a_off[q] + mt * 4096);
    };
    auto make_b = [&](int c, int q) {
      v4i pc = wq[c][q & 1];
      if constexpr (kConvert && !kWReads) asm volatile("" : "+v"(pc));
      return convert_b<kPerChannel>((uint32_t)((q >> 1) ? pc[2] : pc[0]), (uint32_t)((q >> 1) ? pc[3] : pc[1]), 0);
    };
    auto mfma_col = [&](const v4i (&a)[4], const v4i b, int c) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) acc[mt][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mt], b, acc[mt][c], 0, 0, 0);
    };
    v4i a0[4], a1[4];
    read_w(lds);
    read_a(a0, lds, 0);
    read_a(a1, lds, 1);
    for (int t = 0; t < steps; ++t) {
      const int dstage = stage == 0 ? 2 : stage - 1;
      const int8_t* sb = lds + stage * kLoopStage;
      dma_piece(dstage, 0);
      if constexpr (kAReads) read_a(a1, sb, 1);
      mfma_col(a0, make_b(0, 0), 0);
      dma_piece(dstage, 1);
      mfma_col(a0, make_b(1, 0), 1);
      dma_piece(dstage, 2);
      if constexpr (kAReads) read_a(a0, sb, 2);
      mfma_col(a1, make_b(0, 1), 0);
      dma_piece(dstage, 3);
      mfma_col(a1, make_b(1, 1), 1);
      dma_piece(dstage, 4);
      if constexpr (kAReads) read_a(a1, sb, 3);
      mfma_col(a0, make_b(0, 2), 0);
      dma_piece(dstage, 5);
      advance();
      mfma_col(a0, make_b(1, 2), 1);
      const v4i b30 = make_b(0, 3), b31 = make_b(1, 3);
      wait_step();
      stage = (stage == 2) ? 0 : stage + 1;
      const int8_t* nb = lds + stage * kLoopStage;
      if constexpr (kAReads) read_a(a0, nb, 0);
      if constexpr (kWReads) read_w(nb);
      mfma_col(a1, b30, 0);
      mfma_col(a1, b31, 1);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[mt][c][v];
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the cursor's last loads may still be landing
  if (s == 0x7fffffff && steps < 0) sink[0] = s;  // never true: steps >= 1
}

template <int PARTS>
static void launch_loop_probe(int steps, const void* src, uint32_t region, int workgroups, int32_t* sink,
                              hipStream_t st) {
  hipLaunchKernelGGL(probe_prefill_loop_kernel<PARTS>, dim3((unsigned)workgroups), dim3(512), 0, st, steps,
                     (const int8_t*)src, region, sink);
}

}  // namespace qqq

using namespace qqq;

extern "C" {

int qqq_probe_stream_read(const void* buf, size_t bytes, int workgroups, uint32_t* sink, void* stream) {
  if (!buf || !sink) return set_error(QQQ_ERR_NULL, "probe_stream_read: null pointer argument");
  if (bytes < 16 || bytes % 16 != 0 || workgroups < 1 || workgroups > (1 << 20) ||
      (reinterpret_cast<uintptr_t>(buf) & 15u))
    return set_error(QQQ_ERR_SHAPE, "probe_stream_read: bytes must be a multiple of 16, the buffer 16-byte aligned, "
                     "1 <= workgroups <= 2^20");
  hipLaunchKernelGGL(probe_stream_read_kernel<4>, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)buf, bytes / 16, sink);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "probe_stream_read launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

int qqq_probe_mfma_i8(const void* a_pool, const void* b_pool, int iters, int workgroups, int32_t* sink,
                      void* stream) {
  if (!a_pool || !b_pool || !sink) return set_error(QQQ_ERR_NULL, "probe_mfma_i8: null pointer argument");
  if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > 65536 ||
      (reinterpret_cast<uintptr_t>(a_pool) & 15u) || (reinterpret_cast<uintptr_t>(b_pool) & 15u))
    return set_error(QQQ_ERR_SHAPE, "probe_mfma_i8: 1 <= iters <= 2^24, 1 <= workgroups <= 65536, pools 16-byte aligned");
  hipLaunchKernelGGL(probe_mfma_i8_kernel, dim3((unsigned)workgroups), dim3(512), 0, (hipStream_t)stream, iters,
                     (const v4i*)a_pool, (const v4i*)b_pool, sink);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "probe_mfma_i8 launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

int qqq_probe_prefill_loop(const void* src, size_t region_bytes, int steps, int parts, int workgroups,
                           int32_t* sink, void* stream) {
  if (!src || !sink) return set_error(QQQ_ERR_NULL, "probe_prefill_loop: null pointer argument");
  if (steps < 1 || steps > (1 << 24) || workgroups < 1 || workgroups > 65536 || region_bytes < (size_t)kLoopStage ||
      region_bytes % kLoopStage != 0 || region_bytes > (64u << 20) || (reinterpret_cast<uintptr_t>(src) & 15u))
    return set_error(QQQ_ERR_SHAPE, "probe_prefill_loop: 1 <= steps <= 2^24, 1 <= workgroups <= 65536, region a "
                     "multiple of 51200 bytes up to 64 MiB, src 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const uint32_t region = (uint32_t)region_bytes;
  constexpr int A = QQQ_PROBE_A_READS, W = QQQ_PROBE_W_READS, C = QQQ_PROBE_CONVERT, D = QQQ_PROBE_DMA,
                F = QQQ_PROBE_FORM_32X32X32;
  switch (parts) {
    case 0: launch_loop_probe<0>(steps, src, region, workgroups, sink, st); break;
    case C: launch_loop_probe<C>(steps, src, region, workgroups, sink, st); break;
    case A: launch_loop_probe<A>(steps, src, region, workgroups, sink, st); break;
    case A | C: launch_loop_probe<A | C>(steps, src, region, workgroups, sink, st); break;
    case W | C: launch_loop_probe<W | C>(steps, src, region, workgroups, sink, st); break;
    case D: launch_loop_probe<D>(steps, src, region, workgroups, sink, st); break;
    case A | W | C: launch_loop_probe<A | W | C>(steps, src, region, workgroups, sink, st); break;
    case A | W | C | D: launch_loop_probe<A | W | C | D>(steps, src, region, workgroups, sink, st); break;
    case F: launch_loop_probe<F>(steps, src, region, workgroups, sink, st); break;
    case F | A | W | C | D: launch_loop_probe<F | A | W | C | D>(steps, src, region, workgroups, sink, st); break;
    default: return set_error(QQQ_ERR_SHAPE, "probe_prefill_loop: unsupported combination of parts %d", parts);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "probe_prefill_loop launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

}  // extern "C"
