// Skinny (decode) W4A8 GEMM for M <= 64: HBM-bound streaming of the packed int4 weights.
//
// A workgroup of W waves owns one channel group (16*NT output channels) and one of S slices of
// K; its waves interleave over the slice's k-steps and their partial int32 tiles are summed in
// LDS.  With S == 1 the workgroup writes the result directly; otherwise partials meet in an int32
// workspace through device-scope atomics and the workgroup that arrives last at a channel group
// runs the epilogue and returns the workspace to zero.  Integer sums are exact in any order, so
// the result does not depend on the split.  Each wave keeps two batches of U k-steps of 128-bit
// loads in flight (the next batch is issued before the current one is consumed), which is what
// keeps enough bytes in flight to stream HBM from short launches.
//
// Per k-step (128 k) a lane loads 16 B of packed codes per 16-channel tile, converts them in
// registers to two int8 MFMA operands (Sec. 3.3.1 FastINT4toINT8, or Sec. 3.3.2's group-scale
// route) and issues two v_mfma_i32_16x16x64_i8 per row tile.  Activations are the other operand
// (rows >= M repeat row M-1; their outputs are never stored).  Dequant (Sec. 3.3) is fused at the end.
#include "qqq_internal.h"

namespace qqq {

template <int NT, int MT, int U>
struct Batch {
  uint4 w[U][NT];
  v4i a[U][MT][2];
  int sgs[U][4 * NT];  // wave-uniform: the k-step's 16*NT group-scale bytes
};

// The 16*NT group scales of one k-step of a wave's channel group are contiguous and the same for
// the whole wave, so they travel through the scalar (constant) path: no vector-memory
// instruction, which is the scarce issue slot of this kernel.  The compiler tracks the scalar
// loads' completion itself, so they stay in flight across the batch like the vector loads.
typedef const __attribute__((address_space(4))) int* const_int_ptr;

template <int NT>
__device__ __forceinline__ void load_group_scales(const int8_t* gp, int (&sgs)[4 * NT]) {
  const const_int_ptr sp = (const_int_ptr)(uintptr_t)gp;  // gp is wave-uniform
#pragma unroll
  for (int j = 0; j < 4 * NT; ++j) sgs[j] = sp[j];
}

// lane's scale for tile i: byte 16*i + n%16 of the wave's scale words
template <int NT>
__device__ __forceinline__ int pick_group_scale(const int (&sgs)[4 * NT], int i, int nl) {
  // word nl/4 through lane masks (and/or on scalar operands), then byte nl%4
  const int q = nl >> 2;
  const int m0 = -(int)(q == 0), m1 = -(int)(q == 1), m2 = -(int)(q == 2), m3 = -(int)(q == 3);
  const int d = (sgs[4 * i] & m0) | (sgs[4 * i + 1] & m1) | (sgs[4 * i + 2] & m2) | (sgs[4 * i + 3] & m3);
  return (d >> ((nl & 3) * 8)) & 0xFF;
}

// Issues the loads of one batch.  Every call issues the same instructions whatever the position:
// k-steps past the end of the slice are clamped to its last k-step and rows past M to row M-1
// (their products land in k-steps that consume_batch skips and in output rows that are never
// stored).  With no branch around a load the compiler can count the loads issued after a batch
// and waits only for that batch when it is consumed, leaving the next one in flight.
template <int MODE, int NT, int MT, int U>
__device__ __forceinline__ void load_batch(Batch<NT, MT, U>& b, const GemmParams& p, int tb,
                                           int tstride, int t1, int ng, uint32_t lane,
                                           const uint32_t (&aoff)[MT]) {
  const int ntiles = p.N >> 4;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    // wave-uniform bases (scalar registers) plus 32-bit lane offsets
    const int t = min(tb + tstride * u, t1 - 1);
    const uint4* wt = p.w + ((int64_t)t * ntiles + (int64_t)ng * NT) * 64;
    const int8_t* at = p.a_q + (int64_t)t * 128;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      // streamed once: non-temporal, so the weights do not evict the activations from L2
      const v4i raw = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(&wt[lane + 64u * i]));
      b.w[u][i] = make_uint4((uint32_t)raw[0], (uint32_t)raw[1], (uint32_t)raw[2], (uint32_t)raw[3]);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      b.a[u][mt][0] = *(const v4i*)(at + aoff[mt]);
      b.a[u][mt][1] = *(const v4i*)(at + aoff[mt] + 64u);  // second MFMA step of this k-step
    }
    if constexpr (MODE != kPerChannel)
      load_group_scales<NT>(p.s_g + (int64_t)t * p.N + (int64_t)ng * NT * 16, b.sgs[u]);
  }
  // keep every load of the batch ahead of the arithmetic that follows (the scheduler would
  // otherwise sink the scalar loads next to their first use and expose their latency)
  __builtin_amdgcn_sched_barrier(0);
}

template <int MODE, int NT, int MT, int U>
__device__ __forceinline__ void consume_batch(const Batch<NT, MT, U>& b, v4i (&acc)[MT][NT], int tb,
                                              int tstride, int t1, int nl) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (tb + tstride * u >= t1) break;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const uint32_t d[4] = {b.w[u][i].x, b.w[u][i].y, b.w[u][i].z, b.w[u][i].w};
      int o[8];
      int sg = 0;
      if constexpr (MODE != kPerChannel) sg = pick_group_scale<NT>(b.sgs[u], i, nl);
      if constexpr (MODE == kPerChannel || MODE == kGroupLinear) {
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_x16(d[j], o[2 * j], o[2 * j + 1]);
      } else if constexpr (MODE == kGroupClamp) {
        const _Float16 hs = (_Float16)(float)sg;
        const h2 s2 = {hs, hs};
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_group_clamp(d[j], s2, o[2 * j], o[2 * j + 1]);
      } else {
        const GroupFusedConsts g = make_group_fused(sg);
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_group_fused(d[j], g, o[2 * j], o[2 * j + 1]);
      }
      const v4i b0 = {o[0], o[1], o[2], o[3]}, b1 = {o[4], o[5], o[6], o[7]};
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        if constexpr (MODE == kGroupLinear) {
          // the group's partial sum of A*16*code, then (partial/16)*s_g: the same integer as
          // summing A*(code*s_g) because no product saturates when s_g <= 16
          v4i part =
              __builtin_amdgcn_mfma_i32_16x16x64_i8(b.a[u][mt][0], b0, (v4i){0, 0, 0, 0}, 0, 0, 0);
          part = __builtin_amdgcn_mfma_i32_16x16x64_i8(b.a[u][mt][1], b1, part, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[mt][i][r] += (part[r] >> 4) * sg;
        } else {
          acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b.a[u][mt][0], b0, acc[mt][i], 0, 0, 0);
          acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b.a[u][mt][1], b1, acc[mt][i], 0, 0, 0);
        }
      }
    }
  }
}

template <int MODE, int NT, int MT, int W, int U>
__global__ __launch_bounds__(W * 64) void gemm_skinny_kernel(const GemmParams p, const int NG,
                                                             const int S) {
  constexpr int kTiles = MT * NT;
  constexpr int kElems = kTiles * 256;          // int32 outputs of the workgroup
  constexpr int kThreads = W * 64;
  constexpr int kPer = (kElems + kThreads - 1) / kThreads;  // outputs per thread after the reduction
  __shared__ int red[W * kElems];
  __shared__ int s_last;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // the wave index through a scalar register: the k-loop's control flow and the group-scale
  // addresses are then wave-uniform for the compiler too
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nl = lane & 15, kc = lane >> 4;
  const int T = p.T, N = p.N, M = p.M;

  // consecutive workgroups take consecutive channel groups of the same K slice, so the
  // workgroups that run together sweep one contiguous window of the packed weights
  const int ng = blockIdx.x % NG, ks = blockIdx.x / NG;
  const int t0 = ks * T / S, t1 = (ks + 1) * T / S;  // ks < S <= T <= 1024: no overflow

  // this thread's output elements after the cross-wave sum: element e of [tile][r][lane]
  int row[kPer], col[kPer];
  float sa[kPer], sw[kPer];
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    const int e = tid + kThreads * j;
    const int le = e & 63, r = (e >> 6) & 3, tile = e >> 8;
    const int i = tile % NT, mt = tile / NT;
    col[j] = (ng * NT + i) * 16 + (le & 15);
    row[j] = (e < kElems) ? mt * 16 + 4 * (le >> 4) + r : M;  // M = "no output"
    sa[j] = 0.0f;
    sw[j] = 0.0f;
    if (row[j] < M) {  // scales fetched now so the epilogue does not wait on memory
      sa[j] = p.s_a[row[j]];
      sw[j] = (float)p.s_w[col[j]];
    }
  }

  v4i acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[mt][i] = (v4i){0, 0, 0, 0};

  if (t0 + wave < t1) {  // wave-uniform
    constexpr int kStep = W * U;  // k-steps between consecutive batches of one wave
    uint32_t aoff[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      aoff[mt] = (uint32_t)min(mt * 16 + nl, M - 1) * (uint32_t)p.K + (uint32_t)kc * 16u;
    Batch<NT, MT, U> b0, b1;
    int tb = t0 + wave;
    int more = (t1 - tb - 1) / kStep;  // batches after the first
    load_batch<MODE>(b0, p, tb, W, t1, ng, (uint32_t)lane, aoff);
    for (; more >= 2; more -= 2) {  // one basic block: load the next batch, consume the current
      load_batch<MODE>(b1, p, tb + kStep, W, t1, ng, (uint32_t)lane, aoff);
      consume_batch<MODE>(b0, acc, tb, W, t1, nl);
      load_batch<MODE>(b0, p, tb + 2 * kStep, W, t1, ng, (uint32_t)lane, aoff);
      consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl);
      tb += 2 * kStep;
    }
    if (more == 1) {
      load_batch<MODE>(b1, p, tb + kStep, W, t1, ng, (uint32_t)lane, aoff);
      consume_batch<MODE>(b0, acc, tb, W, t1, nl);
      consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl);
    } else {
      consume_batch<MODE>(b0, acc, tb, W, t1, nl);
    }
  }

  // ---- sum the waves' tiles in LDS: red[wave][tile][r][lane]
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        red[wave * kElems + ((mt * NT + i) * 4 + r) * 64 + lane] = acc[mt][i][r];
  __syncthreads();
  int val[kPer];
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    const int e = tid + kThreads * j;
    int v = 0;
    if (e < kElems) {
#pragma unroll
      for (int w = 0; w < W; ++w) v += red[w * kElems + e];
    }
    val[j] = v;
  }

  if (S > 1) {
#pragma unroll
    for (int j = 0; j < kPer; ++j)
      if (row[j] < M && val[j] != 0) atomicAdd(&p.ws_acc[(int64_t)row[j] * N + col[j]], val[j]);
    // Partial sums travel only through device-scope atomics, so the arrival counter below needs
    // just "my atomics have been performed" (vmcnt(0)), not a cache write-back/invalidate fence.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(&p.ws_cnt[ng], 1) == S - 1);
    __syncthreads();
    if (s_last == 0) return;
#pragma unroll
    for (int j = 0; j < kPer; ++j)
      if (row[j] < M) val[j] = atomicExch(&p.ws_acc[(int64_t)row[j] * N + col[j]], 0);
    if (tid == 0) atomicExch(&p.ws_cnt[ng], 0);
  }
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    if (row[j] < M) {
      int v = val[j];
      if constexpr (MODE == kPerChannel) v >>= 4;  // exact: the sum is a multiple of 16
      const int64_t o = (int64_t)row[j] * N + col[j];
      p.y[o] = dequant(v, sa[j], sw[j]);
      if (p.acc_out) p.acc_out[o] = v;
    }
  }
}

static int g_tune_nt = 0, g_tune_s = 0, g_tune_w = 0, g_tune_u = 0;
void set_skinny_tuning(int nt, int s, int w, int u) {
  g_tune_nt = nt;
  g_tune_s = s;
  g_tune_w = w;
  g_tune_u = u;
}

template <int MODE, int NT, int MT, int W, int U>
static int launch_one(const GemmParams& p, int S, hipStream_t st) {
  const int NG = p.N / (16 * NT);
  const int64_t grid = (int64_t)NG * S;
  hipLaunchKernelGGL((gemm_skinny_kernel<MODE, NT, MT, W, U>), dim3((unsigned)grid), dim3(W * 64), 0,
                     st, p, NG, S);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "skinny gemm launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

template <int MODE, int NT, int MT, int U>
static int launch_w(const GemmParams& p, int W, int S, hipStream_t st) {
  if constexpr (NT * MT <= 2) {  // 16 waves x 4 tiles of partial sums would not fit in LDS
    if (W >= 16) return launch_one<MODE, NT, MT, 16, U>(p, S, st);
  }
  if (W >= 8) return launch_one<MODE, NT, MT, 8, U>(p, S, st);
  return launch_one<MODE, NT, MT, 4, U>(p, S, st);
}

// Shape of the launch: channel tiles per workgroup (nt), waves per workgroup (w), K slices (s).
static void choose_split(const GemmParams& p, int mt, int& nt, int& w, int& s) {
  nt = 1;
  if (mt == 1) nt = (p.N % 64 == 0) ? 4 : (p.N % 32 == 0) ? 2 : 1;
  if (mt == 2) nt = (p.N % 32 == 0) ? 2 : 1;
  const int cus = num_cus();
  // Measured on MI355X: the widest channel group that still leaves about two workgroups for
  // every three CUs streams best, with 8 waves per workgroup and no K split (no atomics).
  while (nt > 1 && (int64_t)(p.N / (16 * nt)) * 3 < 2 * cus) nt >>= 1;
  w = (p.T >= 16) ? 8 : 4;
  s = 1;
  // Very narrow outputs: too few channel groups to occupy the chip, so slice K as well
  const int ng = p.N / (16 * nt);
  if (ng * 2 < cus) {
    s = (cus + ng - 1) / ng;
    const int max_s = p.T / (2 * w) > 0 ? p.T / (2 * w) : 1;
    if (s > max_s) s = max_s;
  }
}

template <int MODE>
static int launch_mode(const GemmParams& p, hipStream_t st) {
  const int mt = (p.M + 15) / 16;
  int nt, w, S;
  choose_split(p, mt, nt, w, S);
  if (g_tune_nt > 0 && mt * g_tune_nt <= 4 && p.N % (16 * g_tune_nt) == 0) nt = g_tune_nt;
  if (g_tune_s > 0 && g_tune_s <= p.T) S = g_tune_s;
  if (g_tune_w > 0) w = g_tune_w;
  if (mt <= 1) {
    // k-steps per batch of loads: two batches are in flight, so "deep" keeps 4 (NT=4), 8 (NT=2)
    // or 16 (NT=1) KiB per wave outstanding
    // (measured: the shallow setting streams better on every benchmark shape, so it is the default)
    const bool deep = g_tune_u > 1;
    if (nt == 4) return deep ? launch_w<MODE, 4, 1, 2>(p, w, S, st) : launch_w<MODE, 4, 1, 1>(p, w, S, st);
    if (nt == 2) return deep ? launch_w<MODE, 2, 1, 4>(p, w, S, st) : launch_w<MODE, 2, 1, 2>(p, w, S, st);
    return deep ? launch_w<MODE, 1, 1, 8>(p, w, S, st) : launch_w<MODE, 1, 1, 4>(p, w, S, st);
  }
  if (mt == 2) {
    if (nt >= 2) return launch_w<MODE, 2, 2, 1>(p, w, S, st);
    return launch_w<MODE, 1, 2, 2>(p, w, S, st);
  }
  return launch_w<MODE, 1, 4, 1>(p, w, S, st);
}

int launch_gemm_skinny(const GemmParams& p, int mode, hipStream_t st) {
  if (p.M > kSkinnyMaxM) return set_error(QQQ_ERR_SHAPE, "skinny kernel handles M <= %d", kSkinnyMaxM);
  switch (mode) {
    case kPerChannel: return launch_mode<kPerChannel>(p, st);
    case kGroupLinear: return launch_mode<kGroupLinear>(p, st);
    case kGroupClamp: return launch_mode<kGroupClamp>(p, st);
    case kGroupFused: return launch_mode<kGroupFused>(p, st);
  }
  return set_error(QQQ_ERR_SHAPE, "unknown mode %d", mode);
}

}  // namespace qqq
