// Skinny (decode) W4A8 GEMM for M <= 64: HBM-bound streaming of the packed int4 weights.
//
// Work is the flat list of (channel group, k-step) units in the order the packed weights lie in
// memory; every workgroup takes one contiguous range of it (so every CU streams the same number
// of bytes whatever N and K are), its four waves interleave over the k-steps of the range, and
// partial int32 tiles are summed across waves in LDS.  A range that covers a channel group's
// whole K writes the result directly; otherwise partials meet in an int32 workspace through
// device-scope atomics and the workgroup that completes a channel group runs the epilogue and
// returns the workspace to zero.  Integer sums are exact in any order, so the result does not
// depend on the split.
//
// Per k-step (128 k) a lane loads 16 B of packed codes per 16-channel tile, converts them in
// registers to two int8 MFMA operands (Sec. 3.3.1 FastINT4toINT8, or Sec. 3.3.2's group-scale
// route) and issues two v_mfma_i32_16x16x64_i8 per row tile.  Activations are the other operand
// (rows >= M are zero registers, never loaded).  Dequant (Sec. 3.3) is fused at the end.
#include "qqq_internal.h"

namespace qqq {

template <int MODE, int NT, int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const GemmParams p, const int64_t units) {
  constexpr int kTiles = MT * NT;
  __shared__ int red[4 * kTiles * 256];
  __shared__ int s_last;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int nl = lane & 15, kc = lane >> 4;
  const int T = p.T, N = p.N, M = p.M;
  const int64_t K = p.K;

  const int64_t u0 = (int64_t)blockIdx.x * units / gridDim.x;
  const int64_t u1 = (int64_t)(blockIdx.x + 1) * units / gridDim.x;

  for (int64_t u = u0; u < u1;) {
    const int ng = (int)(u / T);
    const int tb = (int)(u - (int64_t)ng * T);
    const int te = (int)((u1 - u < (int64_t)(T - tb)) ? (tb + (u1 - u)) : T);

    v4i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < NT; ++i) acc[mt][i] = (v4i){0, 0, 0, 0};

    const uint4* wbase = p.w + ((int64_t)ng * NT * T) * 64 + lane;
    for (int t = tb + wave; t < te; t += 4) {
      uint4 wv[NT];
#pragma unroll
      for (int i = 0; i < NT; ++i) wv[i] = wbase[((int64_t)i * T + t) * 64];
      v4i a[MT][2];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + nl;
        a[mt][0] = (v4i){0, 0, 0, 0};
        a[mt][1] = (v4i){0, 0, 0, 0};
        if (m < M) {
          const v4i* ap = (const v4i*)(p.a_q + (int64_t)m * K + (int64_t)t * 128 + kc * 16);
          a[mt][0] = ap[0];
          a[mt][1] = ap[4];  // +64 bytes: second MFMA step of this k-step
        }
      }
      int sg[NT];
      if constexpr (MODE != kPerChannel) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
          sg[i] = (int)p.s_g[(int64_t)t * N + (int64_t)(ng * NT + i) * 16 + nl];
      }
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        v4i b0, b1;
        const uint32_t d[4] = {wv[i].x, wv[i].y, wv[i].z, wv[i].w};
        int o[8];
        if constexpr (MODE == kPerChannel || MODE == kGroupLinear) {
#pragma unroll
          for (int j = 0; j < 4; ++j) unpack_x16(d[j], o[2 * j], o[2 * j + 1]);
        } else if constexpr (MODE == kGroupClamp) {
          const _Float16 hs = (_Float16)(float)sg[i];
          const h2 s2 = {hs, hs};
#pragma unroll
          for (int j = 0; j < 4; ++j) unpack_group_clamp(d[j], s2, o[2 * j], o[2 * j + 1]);
        } else {
          const GroupFusedConsts g = make_group_fused(sg[i]);
#pragma unroll
          for (int j = 0; j < 4; ++j) unpack_group_fused(d[j], g, o[2 * j], o[2 * j + 1]);
        }
        b0 = (v4i){o[0], o[1], o[2], o[3]};
        b1 = (v4i){o[4], o[5], o[6], o[7]};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if constexpr (MODE == kGroupLinear) {
            // the group's partial sum of A*16*code, then (partial/16)*s_g: the same integer as
            // summing A*(code*s_g) because no product saturates when s_g <= 16
            v4i part = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][0], b0, (v4i){0, 0, 0, 0}, 0, 0, 0);
            part = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][1], b1, part, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mt][i][r] += (part[r] >> 4) * sg[i];
          } else {
            acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][0], b0, acc[mt][i], 0, 0, 0);
            acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][1], b1, acc[mt][i], 0, 0, 0);
          }
        }
      }
    }

    // ---- sum the four waves' tiles in LDS: red[wave][tile][r][lane]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          red[((wave * kTiles + mt * NT + i) * 4 + r) * 64 + lane] = acc[mt][i][r];
    __syncthreads();

    const bool full = (tb == 0 && te == T);
    int val[kTiles], row[kTiles], col[kTiles];
#pragma unroll
    for (int j = 0; j < kTiles; ++j) {
      const int e = tid + 256 * j;  // element of [tile][r][lane]
      val[j] = red[e] + red[e + kTiles * 256] + red[e + 2 * kTiles * 256] + red[e + 3 * kTiles * 256];
      const int le = e & 63, r = (e >> 6) & 3, tile = e >> 8;
      const int i = tile % NT, mt = tile / NT;
      col[j] = (ng * NT + i) * 16 + (le & 15);
      row[j] = mt * 16 + 4 * (le >> 4) + r;
    }

    bool finish = full;
    if (!full) {
#pragma unroll
      for (int j = 0; j < kTiles; ++j)
        if (row[j] < M && val[j] != 0) atomicAdd(&p.ws_acc[(int64_t)row[j] * N + col[j]], val[j]);
      __threadfence();
      __syncthreads();
      if (tid == 0) {
        const int done = atomicAdd(&p.ws_cnt[ng], te - tb) + (te - tb);
        s_last = (done == T);
      }
      __syncthreads();
      finish = (s_last != 0);
      if (finish) {
        __threadfence();
#pragma unroll
        for (int j = 0; j < kTiles; ++j)
          if (row[j] < M) val[j] = atomicExch(&p.ws_acc[(int64_t)row[j] * N + col[j]], 0);
        if (tid == 0) atomicExch(&p.ws_cnt[ng], 0);
      }
    }
    if (finish) {
#pragma unroll
      for (int j = 0; j < kTiles; ++j) {
        if (row[j] < M) {
          int v = val[j];
          if constexpr (MODE == kPerChannel) v >>= 4;  // exact: the sum is a multiple of 16
          const int64_t o = (int64_t)row[j] * N + col[j];
          p.y[o] = dequant(v, p.s_a[row[j]], (float)p.s_w[col[j]]);
          if (p.acc_out) p.acc_out[o] = v;
        }
      }
    }
    __syncthreads();  // red[] and s_last are reused by the next range
    u += te - tb;
  }
}

template <int MODE, int NT, int MT>
static int launch_one(const GemmParams& p, int blocks_per_cu, hipStream_t st) {
  const int64_t units = (int64_t)(p.N / (16 * NT)) * p.T;
  int64_t grid = (int64_t)num_cus() * blocks_per_cu;
  if (grid > units) grid = units;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL((gemm_skinny_kernel<MODE, NT, MT>), dim3((unsigned)grid), dim3(256), 0, st, p,
                     units);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "skinny gemm launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

template <int MODE>
static int launch_mode(const GemmParams& p, hipStream_t st) {
  const int mt = (p.M + 15) / 16;
  // channel tiles per unit: wider units reuse each activation fragment more, but need enough
  // units to give every workgroup several k-steps per wave
  const int64_t units1 = (int64_t)(p.N / 16) * p.T;
  const int64_t want = (int64_t)num_cus() * 4 * 8;
  if (mt <= 1) {
    if (p.N % 64 == 0 && units1 / 4 >= want) return launch_one<MODE, 4, 1>(p, 4, st);
    if (p.N % 32 == 0 && units1 / 2 >= want) return launch_one<MODE, 2, 1>(p, 4, st);
    return launch_one<MODE, 1, 1>(p, 4, st);
  }
  if (mt == 2) {
    if (p.N % 32 == 0 && units1 / 2 >= want) return launch_one<MODE, 2, 2>(p, 4, st);
    return launch_one<MODE, 1, 2>(p, 4, st);
  }
  return launch_one<MODE, 1, 4>(p, 4, st);
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
