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
  int sgv[U][(NT + 3) / 4];  // the words of the k-step's group scales that hold this lane's scales of tiles
                             // (lane/16) mod NT (and that plus 4 where a workgroup has eight tiles)
};

// The 16*NT group scales of one k-step of a wave's channel group are 4*NT contiguous words.  Lane
// (row kc = lane/16, channel nl = lane%16) requests the word that holds the scale of channel nl in
// tile kc mod NT: one vector-memory instruction for the wave, and every lane already holds one of
// the NT scales of its own channel.  When the batch is consumed each lane extracts its byte and the
// 16-lane rows are exchanged with the row-swap instructions (v_permlane32_swap swaps the upper
// half of one operand with the lower half of the other, v_permlane16_swap the odd rows of one with
// the even rows of the other), after which every lane holds all NT scales of its channel: three
// instructions for four tiles, no scalar broadcasts, no LDS crossbar.
// (The real-valued variant's scales are fp16: 8*NT words, two scales each.)
template <int NT, int MODE>
__device__ __forceinline__ int load_group_scales(const int8_t* gp, uint32_t lane, uint32_t tile0 = 0) {
  const uint32_t tile = tile0 + ((lane >> 4) & (uint32_t)((NT < 4 ? NT : 4) - 1)), nl = lane & 15u;
  const uint32_t word = MODE == kGroupReal ? 8u * tile + (nl >> 1) : 4u * tile + (nl >> 2);
  return reinterpret_cast<const int*>(gp)[word];
}

// sg[i] = scale of the lane's channel in tile i (int8 scale, or fp16 bit pattern)
template <int NT, int MODE>
__device__ __forceinline__ void spread_group_scales(int sgv, int nl, int (&sg)[NT]) {
  const uint32_t own = MODE == kGroupReal ? ((uint32_t)sgv >> ((nl & 1) * 16)) & 0xFFFFu
                                          : ((uint32_t)sgv >> ((nl & 3) * 8)) & 0xFFu;
  if constexpr (NT == 1) {
    sg[0] = (int)own;
  } else if constexpr (NT == 2) {  // rows hold tiles 0,1,0,1
    const auto t = __builtin_amdgcn_permlane16_swap(own, own, false, false);
    sg[0] = (int)t[0];
    sg[1] = (int)t[1];
  } else {                         // rows hold tiles 0,1,2,3
    static_assert(NT == 4, "channel tiles per word of scales");
    const auto h = __builtin_amdgcn_permlane32_swap(own, own, false, false);  // rows 0,1,0,1 | 2,3,2,3
    const auto lo = __builtin_amdgcn_permlane16_swap(h[0], h[0], false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(h[1], h[1], false, false);
    sg[0] = (int)lo[0];
    sg[1] = (int)lo[1];
    sg[2] = (int)hi[0];
    sg[3] = (int)hi[1];
  }
}

// Issues the loads of one batch.  Every call issues the same instructions whatever the position:
// k-steps past the end of the slice are clamped to its last k-step and rows past M to row M-1
// (their products land in k-steps that consume_batch skips and in output rows that are never
// stored).  With no branch around a load the compiler can count the loads issued after a batch
// and waits only for that batch when it is consumed, leaving the next one in flight.
// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for every
// global load in flight, and here the first weight batches are deliberately still on their way.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int MODE, int NT, int MT, int U>
__device__ __forceinline__ void load_batch_w(Batch<NT, MT, U>& b, const GemmParams& p, int tb,
                                             int tstride, int t1, int ng, uint32_t lane) {
  const int ntiles = p.N >> 4;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    // wave-uniform bases (scalar registers) plus 32-bit lane offsets
    const int t = min(tb + tstride * u, t1 - 1);
    const uint4* wt = p.w + ((int64_t)t * ntiles + (int64_t)ng * NT) * 64;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      // streamed once: non-temporal, so the weights do not evict the activations from L2
      const v4i raw = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(&wt[lane + 64u * i]));
      b.w[u][i] = make_uint4((uint32_t)raw[0], (uint32_t)raw[1], (uint32_t)raw[2], (uint32_t)raw[3]);
    }
    if constexpr (MODE != kPerChannel) {
#pragma unroll
      for (int q = 0; q < (NT + 3) / 4; ++q)
        b.sgv[u][q] = load_group_scales<NT, MODE>(
            p.s_g + ((int64_t)t * p.N + (int64_t)ng * NT * 16) * (MODE == kGroupReal ? 2 : 1), lane, 4u * q);
    }
  }
}

// abase: the global a_q, or the workgroup's LDS copy in the fused kernel
template <int NT, int MT, int U>
__device__ __forceinline__ void load_batch_a(Batch<NT, MT, U>& b, const int8_t* abase, int tb,
                                             int tstride, int t1, const uint32_t (&aoff)[MT][2]) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int t = min(tb + tstride * u, t1 - 1);
    const int8_t* at = abase + (int64_t)t * 128;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      b.a[u][mt][0] = *(const v4i*)(at + aoff[mt][0]);
      b.a[u][mt][1] = *(const v4i*)(at + aoff[mt][1]);
    }
  }
}

template <int MODE, int NT, int MT, int U>
__device__ __forceinline__ void load_batch(Batch<NT, MT, U>& b, const GemmParams& p,
                                           const int8_t* abase, int tb, int tstride, int t1, int ng,
                                           uint32_t lane, const uint32_t (&aoff)[MT][2]) {
  load_batch_w<MODE>(b, p, tb, tstride, t1, ng, lane);
  load_batch_a(b, abase, tb, tstride, t1, aoff);
  // keep every load of the batch ahead of the arithmetic that follows (the scheduler would
  // otherwise interleave them with the conversion and shorten the time they are in flight)
  __builtin_amdgcn_sched_barrier(0);
}

// Row-major activation fetch.  An MFMA operand wants lane (row l%16, k-block l/16): taken straight from
// memory that is 16 different rows per quarter wave, 16 cache-line look-ups for 256 bytes, and from
// nine rows on it shows (8 -> 16 distinct rows: +1.0 us on a 20 us launch).  With `tr` set the batch
// was loaded row-major instead (lane l: row l/8 of the first or second eight rows, 16-byte chunk l%8:
// whole 128-byte lines per eight lanes) and each fragment pair takes a round trip through the
// wave's own 2 KiB of LDS into operand order: chunk c of row r sits in slot c ^ ((r/2)%8), which
// makes both the row-major writes and the operand-order reads conflict-free.  One wave's LDS
// accesses are served in order, so no barrier is involved.
struct ATranspose {
  int8_t* tr;            // the wave's 2 KiB, or nullptr: fragments are already in operand order
  uint32_t woff[2], roff[2];
};
__device__ __forceinline__ ATranspose make_a_transpose(int8_t* tr, uint32_t lane) {
  ATranspose t;
  t.tr = tr;
  const uint32_t r = lane >> 3, c = lane & 7, nl = lane & 15, kc = lane >> 4;
  t.woff[0] = r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
  t.woff[1] = (r + 8) * 128 + ((c ^ (((r + 8) >> 1) & 7)) << 4);
  t.roff[0] = nl * 128 + ((kc ^ ((nl >> 1) & 7)) << 4);
  t.roff[1] = nl * 128 + (((4 + kc) ^ ((nl >> 1) & 7)) << 4);
  return t;
}

template <int MODE, int NT, int MT, int U>
__device__ __forceinline__ void consume_batch(const Batch<NT, MT, U>& b, v4i (&acc)[MT][NT], int tb,
                                              int tstride, int t1, int nl, const ATranspose& at) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (tb + tstride * u >= t1) break;
    v4i a[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      a[mt][0] = b.a[u][mt][0];
      a[mt][1] = b.a[u][mt][1];
      if (at.tr) {  // wave-uniform
        *(v4i*)(at.tr + at.woff[0]) = a[mt][0];
        *(v4i*)(at.tr + at.woff[1]) = a[mt][1];
        a[mt][0] = *(const v4i*)(at.tr + at.roff[0]);
        a[mt][1] = *(const v4i*)(at.tr + at.roff[1]);
      }
    }
    int sgs[NT] = {};
    if constexpr (MODE != kPerChannel) {
      if constexpr (NT <= 4) {
        spread_group_scales<NT, MODE>(b.sgv[u][0], nl, sgs);
      } else {  // eight tiles: two words, four tiles each
        static_assert(NT == 8, "channel tiles per workgroup");
        int lo4[4], hi4[4];
        spread_group_scales<4, MODE>(b.sgv[u][0], nl, lo4);
        spread_group_scales<4, MODE>(b.sgv[u][1], nl, hi4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          sgs[i] = lo4[i];
          sgs[4 + i] = hi4[i];
        }
      }
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const uint32_t d[4] = {b.w[u][i].x, b.w[u][i].y, b.w[u][i].z, b.w[u][i].w};
      int o[8];
      const int sg = sgs[i];
      if constexpr (MODE == kPerChannel || MODE == kGroupLinear) {
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_x16(d[j], o[2 * j], o[2 * j + 1]);
      } else if constexpr (MODE == kGroupClamp) {
        const _Float16 hs = (_Float16)(float)sg;
        const h2 s2 = {hs, hs};
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_group_clamp(d[j], s2, o[2 * j], o[2 * j + 1]);
      } else if constexpr (MODE == kGroupReal) {
        const h2 s2 = as_h2((uint32_t)sg | ((uint32_t)sg << 16));
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_group_real(d[j], s2, o[2 * j], o[2 * j + 1]);
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
          v4i part = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][0], b0, (v4i){0, 0, 0, 0}, 0, 0, 0);
          part = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][1], b1, part, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 4; ++r)  // |part >> 4| <= 127*8*128 < 2^23 and 0 <= sg <= 16: the full-rate
            acc[mt][i][r] = __mul24(part[r] >> 4, sg) + acc[mt][i][r];  // 24-bit multiply(-add)
        } else {
          acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][0], b0, acc[mt][i], 0, 0, 0);
          acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][1], b1, acc[mt][i], 0, 0, 0);
        }
      }
    }
  }
}

// FUSED: the workgroup quantises the fp16 activation rows itself (Sec. 4.1: per-token absmax
// scale, division, round half to even) into LDS before the k-loop, with the arithmetic of the
// stand-alone pass, so a decode step is a single launch.  Every workgroup repeats the M*K
// conversions, which is only worth it for a few rows; the A operands then come from LDS.
template <int MODE, int NT, int MT, int W, int U, int FUSED>
__global__ __launch_bounds__(W * 64) void gemm_skinny_kernel(const GemmParams p, const int NG,
                                                             const int S) {
  constexpr int kTiles = MT * NT;
  constexpr int kElems = kTiles * 256;          // int32 outputs of the workgroup
  constexpr int kThreads = W * 64;
  constexpr int kPer = (kElems + kThreads - 1) / kThreads;  // outputs per thread after the reduction
  // one LDS buffer: the quantised activations during the k-loop (FUSED), the waves' partial
  // tiles after it
  constexpr int kRedInts = W * kElems;
  // FUSED: 0 = no, 1 = up to kFusedLdsSmall activations (M*K), 2 = up to kFusedLdsBytes
  constexpr int kFusedBytes = FUSED == 2 ? kFusedLdsBytes : kFusedLdsSmall;
  // (+ 16 bytes per row: see the fused prologue)
  constexpr int kFusedInts = kFusedBytes / 4 + 4 * kFusedMaxM;
  constexpr int kSmemInts = (FUSED && kFusedInts > kRedInts) ? kFusedInts : kRedInts;
  __shared__ __attribute__((aligned(16))) int smem[kSmemInts];
  int* const red = smem;
  __shared__ __attribute__((aligned(16))) int8_t a_tr[FUSED ? 16 : W * 2048];  // see ATranspose
  __shared__ int s_last;
  __shared__ uint32_t s_amax[kFusedMaxM][W];
  __shared__ float s_sa[kFusedMaxM];

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
  // The epilogue's scales are requested now, with clamped indices and no arithmetic on them (the
  // fp16 stays raw bits), so nothing here waits for memory and the epilogue does not either.
  float sa[kPer];
  uint32_t sw_bits[kPer];
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    const int e = tid + kThreads * j;
    const int le = e & 63, r = (e >> 6) & 3, tile = e >> 8;
    const int i = tile % NT, mt = tile / NT;
    col[j] = (ng * NT + i) * 16 + (le & 15);
    row[j] = (e < kElems) ? mt * 16 + 4 * (le >> 4) + r : M;  // M = "no output"
    sa[j] = 0.0f;
    if constexpr (!FUSED) sa[j] = p.s_a[min(row[j], M - 1)];
    sw_bits[j] = reinterpret_cast<const uint16_t*>(p.s_w)[min(col[j], N - 1)];
  }

  constexpr int kStep = W * U;  // k-steps between consecutive batches of one wave
  Batch<NT, MT, U> b0, b1;
  const int8_t* abase = p.a_q;
  if constexpr (FUSED) {
    // host guarantees M <= kFusedMaxM and M*K <= kFusedBytes
    constexpr int kVPT = kFusedBytes / 8 / kThreads;  // 128-bit fp16 vectors per thread
    static_assert(kVPT >= 1 && kVPT * kThreads * 8 == kFusedBytes, "fused path sized for 8 waves");
    const int nvec = p.K >> 3;  // 128-bit vectors of 8 fp16 per row
    const int total = M * nvec;
    uint2* const aq_lds = reinterpret_cast<uint2*>(smem);
    {
      // The rows stay in registers between the |max| pass and the division.  Every thread issues
      // all kVPT loads (positions past the end re-read some earlier vector, spread over many
      // addresses) and then the first two batches of weights, with no branch in between: the
      // rows return first and are quantised while the weights are still on their way.
      uint4 v[kVPT];
      int vm[kVPT];
      const int wrap = (1 << (31 - __builtin_clz(total))) - 1;  // largest 2^k <= total, minus 1
#pragma unroll
      for (int j = 0; j < kVPT; ++j) {
        const int raw = tid + kThreads * j;
        const int idx = raw < total ? raw : (raw & wrap);
        vm[j] = idx / nvec;
        v[j] = p.a_fp16[(int64_t)vm[j] * p.lda_vec + (idx - vm[j] * nvec)];
      }
      load_batch_w<MODE>(b0, p, t0 + wave, W, t1, ng, (uint32_t)lane);
      __builtin_amdgcn_sched_barrier(0);  // request order = consumption order, as in the k-loop
      load_batch_w<MODE>(b1, p, t0 + wave + kStep, W, t1, ng, (uint32_t)lane);
      __builtin_amdgcn_sched_barrier(0);  // all requests are out before any arithmetic on the rows
      uint32_t am[kFusedMaxM];
#pragma unroll
      for (int m = 0; m < kFusedMaxM; ++m) am[m] = 0;
#pragma unroll
      for (int j = 0; j < kVPT; ++j) {
        const uint32_t bits = absmax_bits(v[j], 0);
#pragma unroll
        for (int m = 0; m < kFusedMaxM; ++m) am[m] = max(am[m], vm[j] == m ? bits : 0u);
      }
#pragma unroll
      for (int m = 0; m < kFusedMaxM; ++m) {
        am[m] = wave_max_u32(am[m]);
        if (lane == 0) s_amax[m][wave] = am[m];
      }
      lds_barrier();
      float amax[kFusedMaxM], sc[kFusedMaxM];
#pragma unroll
      for (int m = 0; m < kFusedMaxM; ++m) {
        uint32_t bits = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) bits = max(bits, s_amax[m][w]);
        amax[m] = half_bits_to_float(bits);
        sc[m] = amax[m] / 127.0f;
        if (tid == 0 && m < M) s_sa[m] = (amax[m] == 0.0f) ? 0.0f : sc[m];
      }
#pragma unroll
      for (int j = 0; j < kVPT; ++j) {
        const int idx = tid + kThreads * j;
        float a_m = amax[0], s_m = sc[0];
#pragma unroll
        for (int m = 1; m < kFusedMaxM; ++m) {
          a_m = (vm[j] == m) ? amax[m] : a_m;
          s_m = (vm[j] == m) ? sc[m] : s_m;
        }
        if (idx < total) {
          uint2 o = make_uint2(0, 0);
          if (a_m != 0.0f) {
            o.x = quant4(v[j].x, v[j].y, s_m);
            o.y = quant4(v[j].z, v[j].w, s_m);
          }
          // row m starts at byte m*(K+16): K is a multiple of all 64 banks, and an MFMA fragment read
          // takes the same 16 bytes of up to four different rows at once, which the pad spreads over the banks
          aq_lds[idx + 2 * vm[j]] = o;
        }
      }
    }
    lds_barrier();
#pragma unroll
    for (int j = 0; j < kPer; ++j)
      if (row[j] < M) sa[j] = s_sa[row[j]];
    abase = reinterpret_cast<const int8_t*>(smem);
  }

  v4i acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[mt][i] = (v4i){0, 0, 0, 0};

  if (t0 + wave < t1) {  // wave-uniform
    // up to eight rows (and from the fused kernel's LDS copy) the fragments are fetched in operand
    // order; beyond, row-major with the round trip through LDS
    const bool row_major = !FUSED && (MT > 1 || M > 8);
    const ATranspose at = make_a_transpose(row_major ? a_tr + wave * 2048 : nullptr, (uint32_t)lane);
    uint32_t aoff[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if (row_major) {
        aoff[mt][0] = (uint32_t)min(mt * 16 + (lane >> 3), M - 1) * (uint32_t)p.K + (uint32_t)(lane & 7) * 16u;
        aoff[mt][1] = (uint32_t)min(mt * 16 + 8 + (lane >> 3), M - 1) * (uint32_t)p.K + (uint32_t)(lane & 7) * 16u;
      } else {
        aoff[mt][0] = (uint32_t)min(mt * 16 + nl, M - 1) * ((uint32_t)p.K + (FUSED ? 16u : 0u)) + (uint32_t)kc * 16u;
        aoff[mt][1] = aoff[mt][0] + 64u;  // second MFMA step of this k-step
      }
    }
    int tb = t0 + wave;
    int more = (t1 - tb - 1) / kStep;  // batches after the first
    if constexpr (FUSED) {
      // the weights of the first two batches were requested before the prologue (the second is a
      // clamped repeat when the wave has a single batch and is then never consumed)
      load_batch_a(b0, abase, tb, W, t1, aoff);
      load_batch_a(b1, abase, tb + kStep, W, t1, aoff);
      __builtin_amdgcn_sched_barrier(0);
      for (; more >= 3; more -= 2) {  // one basic block: consume a batch, request the one after next
        consume_batch<MODE>(b0, acc, tb, W, t1, nl, at);
        load_batch<MODE>(b0, p, abase, tb + 2 * kStep, W, t1, ng, (uint32_t)lane, aoff);
        consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl, at);
        load_batch<MODE>(b1, p, abase, tb + 3 * kStep, W, t1, ng, (uint32_t)lane, aoff);
        tb += 2 * kStep;
      }
      consume_batch<MODE>(b0, acc, tb, W, t1, nl, at);
      if (more == 2) {
        load_batch<MODE>(b0, p, abase, tb + 2 * kStep, W, t1, ng, (uint32_t)lane, aoff);
        consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl, at);
        consume_batch<MODE>(b0, acc, tb + 2 * kStep, W, t1, nl, at);
      } else if (more == 1) {
        consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl, at);
      }
    } else {
      load_batch<MODE>(b0, p, abase, tb, W, t1, ng, (uint32_t)lane, aoff);
      for (; more >= 2; more -= 2) {  // one basic block: load the next batch, consume the current
        load_batch<MODE>(b1, p, abase, tb + kStep, W, t1, ng, (uint32_t)lane, aoff);
        consume_batch<MODE>(b0, acc, tb, W, t1, nl, at);
        load_batch<MODE>(b0, p, abase, tb + 2 * kStep, W, t1, ng, (uint32_t)lane, aoff);
        consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl, at);
        tb += 2 * kStep;
      }
      if (more == 1) {
        load_batch<MODE>(b1, p, abase, tb + kStep, W, t1, ng, (uint32_t)lane, aoff);
        consume_batch<MODE>(b0, acc, tb, W, t1, nl, at);
        consume_batch<MODE>(b1, acc, tb + kStep, W, t1, nl, at);
      } else {
        consume_batch<MODE>(b0, acc, tb, W, t1, nl, at);
      }
    }
  }

  // ---- sum the waves' tiles in LDS: red[wave][tile][r][lane]
  if constexpr (FUSED) __syncthreads();  // every wave is done reading the activations in smem
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
      p.y[o] = dequant(v, sa[j], half_bits_to_float(sw_bits[j]));
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

template <int MODE, int NT, int MT, int W, int U, int FUSED = 0>
static int launch_one(const GemmParams& p, int S, hipStream_t st) {
  const int NG = p.N / (16 * NT);
  const int64_t grid = (int64_t)NG * S;
  hipLaunchKernelGGL((gemm_skinny_kernel<MODE, NT, MT, W, U, FUSED>), dim3((unsigned)grid),
                     dim3(W * 64), 0, st, p, NG, S);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "skinny gemm launch: %s", hipGetErrorString(e));
  route_note("decode nt=%d mt=%d waves=%d depth=%d kslices=%d fused=%d mode=%d grid=%lld", NT, MT, W, U, S,
             FUSED ? 1 : 0, MODE, (long long)grid);
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
// 16-channel tiles per workgroup for N channels and mt row tiles (also read by the dispatch model)
int decode_channel_tiles(int64_t N, int mt, bool light_conversion) {
  int nt = (N % 64 == 0) ? 4 : (N % 32 == 0) ? 2 : 1;
  // (with several row tiles every workgroup re-reads all activations from L2, so the widest channel
  // group that keeps the CUs busy, rule below, also cuts those re-reads the most)
  // up to 32 rows: 128 channels where enough workgroups remain.  Every workgroup reads all activations
  // from L2 (from 9 rows on a third to two thirds of what it reads of the weights at 64 channels per
  // workgroup): cfg5 M=16 20.9 -> 20.0 us; with few rows it is level or slightly ahead
  // (only with the light conversions, per-channel and group scale on partial sums: the per-weight fp16 routes
  // need the second workgroup per CU to cover their arithmetic: real-valued scales, 8192 x 28672, M=1: 29.3 us
  // with 128 channels, 26.8 with 64)
  if (mt <= 2 && N % 128 == 0 && light_conversion) nt = 8;
  // Measured on MI355X: the widest channel group that still leaves about two workgroups for
  // every three CUs streams best, with 8 waves per workgroup and no K split (no atomics).
  while (nt > 1 && (N / (16 * nt)) * 3 < 2 * (int64_t)num_cus()) nt >>= 1;
  return nt;
}

static void choose_split(const GemmParams& p, int mt, bool light_conversion, int& nt, int& w, int& s) {
  nt = decode_channel_tiles(p.N, mt, light_conversion);
  const int cus = num_cus();
  w = (p.T >= 16) ? 8 : 4;
  // a workgroup with 32 KiB of weights or less (16 channels, K <= 4096) finishes sooner on 4 waves, each with
  // two batches of loads, than on 8 with one and twice the partial tiles to add (K = N = 4096, M=16: 4.85 -> 4.7 us
  // on average over a profiled run)
  if ((int64_t)16 * nt * p.K / 2 <= 32768) w = 4;
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
  choose_split(p, mt, MODE == kPerChannel || MODE == kGroupLinear, nt, w, S);
  if (g_tune_nt > 0 && p.N % (16 * g_tune_nt) == 0) nt = g_tune_nt;
  if (g_tune_s > 0 && g_tune_s <= p.T) S = g_tune_s;
  if (g_tune_w > 0) w = g_tune_w;
  if (p.a_fp16 != nullptr) {
    // fused activation quantisation: one row tile, 8 waves, default batch depth
    if (mt != 1 || p.M > kFusedMaxM || (int64_t)p.M * p.K > kFusedLdsBytes)
      return set_error(QQQ_ERR_SHAPE, "fused decode kernel: M=%d K=%d out of range", p.M, p.K);
    // two sizes of the quantising prologue: every thread loads (and holds) its share of the larger one
    if ((int64_t)p.M * p.K <= kFusedLdsSmall) {
      if (nt >= 4) return launch_one<MODE, 4, 1, 8, 1, 1>(p, S, st);
      if (nt == 2) return launch_one<MODE, 2, 1, 8, 2, 1>(p, S, st);
      return launch_one<MODE, 1, 1, 8, 4, 1>(p, S, st);
    }
    if (nt >= 4) return launch_one<MODE, 4, 1, 8, 1, 2>(p, S, st);
    if (nt == 2) return launch_one<MODE, 2, 1, 8, 2, 2>(p, S, st);
    return launch_one<MODE, 1, 1, 8, 4, 2>(p, S, st);
  }
  if (mt <= 1) {
    // k-steps per batch of loads: two batches are in flight, so "deep" keeps 4 (NT=4), 8 (NT=2)
    // or 16 (NT=1) KiB per wave outstanding
    // (measured: the shallow setting streams better on every benchmark shape, so it is the default)
    const bool deep = g_tune_u > 1;
    if (nt == 8) return launch_w<MODE, 8, 1, 1>(p, w, S, st);
    if (nt == 4) return deep ? launch_w<MODE, 4, 1, 2>(p, w, S, st) : launch_w<MODE, 4, 1, 1>(p, w, S, st);
    if (nt == 2) return deep ? launch_w<MODE, 2, 1, 4>(p, w, S, st) : launch_w<MODE, 2, 1, 2>(p, w, S, st);
    return deep ? launch_w<MODE, 1, 1, 8>(p, w, S, st) : launch_w<MODE, 1, 1, 4>(p, w, S, st);
  }
  if (mt == 2) {
    if (nt >= 8) return launch_w<MODE, 8, 2, 1>(p, w, S, st);
    if (nt >= 4) return launch_w<MODE, 4, 2, 1>(p, w, S, st);
    if (nt >= 2) return launch_w<MODE, 2, 2, 1>(p, w, S, st);
    return launch_w<MODE, 1, 2, 2>(p, w, S, st);
  }
  if (nt >= 4) return launch_w<MODE, 4, 4, 1>(p, 4, S, st);  // 16 tiles of accumulators: 4 waves fit LDS and registers
  if (nt >= 2) return launch_w<MODE, 2, 4, 1>(p, w, S, st);
  return launch_w<MODE, 1, 4, 1>(p, w, S, st);
}

int launch_gemm_skinny(const GemmParams& p, int mode, hipStream_t st) {
  if (p.M > kSkinnyMaxM) return set_error(QQQ_ERR_SHAPE, "skinny kernel handles M <= %d", kSkinnyMaxM);
  switch (mode) {
    case kPerChannel: return launch_mode<kPerChannel>(p, st);
    case kGroupLinear: return launch_mode<kGroupLinear>(p, st);
    case kGroupClamp: return launch_mode<kGroupClamp>(p, st);
    case kGroupFusedWide:
    case kGroupFused: return launch_mode<kGroupFused>(p, st);
    case kGroupReal: return launch_mode<kGroupReal>(p, st);
  }
  return set_error(QQQ_ERR_SHAPE, "unknown mode %d", mode);
}

}  // namespace qqq
