// LDS-tiled W4A8 GEMM for M > 64 (prefill): bound by the int8 MFMA pipe.
//
// A workgroup of 4 waves computes a BM x BN = 128 x 256 tile of Y.  The waves split N (64 channels
// each) and share the activation tile through LDS, so every packed weight fragment is loaded
// from global memory straight into the registers of the one wave that needs it, converted to
// int8 once (Sec. 3.3.1 / 3.3.2 of the QQQ paper) and fed to 8 MFMAs.  The activation tile
// (128 rows x 128 k int8) is double-buffered in LDS with a 16-byte row pad that keeps the
// 128-bit operand reads free of bank conflicts.  One k-step = 128 k = one scale group.
#include "qqq_internal.h"

namespace qqq {

constexpr int kBM = 128, kBN = 256, kBK = 128;
constexpr int kLdsRow = kBK + 16;  // bytes per LDS row of A

template <int MODE>
__global__ __launch_bounds__(256) void gemm_prefill_kernel(const GemmParams p, const int tiles_m,
                                                           const int tiles_n) {
  __shared__ __attribute__((aligned(16))) int8_t lds_a[2][kBM * kLdsRow];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int nl = lane & 15, kc = lane >> 4;
  const int T = p.T, N = p.N, M = p.M;
  const int64_t K = p.K;

  // XCD-aware order: consecutive workgroup ids land on different XCDs (8 of them), so give each
  // XCD a contiguous run of tiles, m fastest, and neighbours in one L2 share their weight tile.
  const int nblk = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8;
    if (per > 0 && pid < per * 8) pid = (pid % 8) * per + pid / 8;
  }
  const int tm = pid % tiles_m, tn = pid / tiles_m;
  const int m0 = tm * kBM;
  const int nt0 = tn * (kBN / 16) + wave * 4;  // first of this wave's 4 channel tiles
  const int ntiles = N / 16;

  // global -> LDS copy assignment: 8 threads per row (16 B each), 32 rows per pass, 4 passes
  const int cr = tid >> 3, cc = tid & 7;
  v4i areg[4];
  auto load_a = [&](int t) {
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int m = m0 + ps * 32 + cr;
      areg[ps] = (v4i){0, 0, 0, 0};
      if (m < M) areg[ps] = *(const v4i*)(p.a_q + (int64_t)m * K + (int64_t)t * kBK + cc * 16);
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int ps = 0; ps < 4; ++ps)
      *(v4i*)(&lds_a[buf][(ps * 32 + cr) * kLdsRow + cc * 16]) = areg[ps];
  };
  uint4 wreg[4];
  int sgreg[4];
  auto load_w = [&](int t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      wreg[i] = make_uint4(0, 0, 0, 0);
      sgreg[i] = 0;
      if (nt0 + i < ntiles) {
        wreg[i] = p.w[((int64_t)t * ntiles + (nt0 + i)) * 64 + lane];
        if constexpr (MODE != kPerChannel)
          sgreg[i] = (int)p.s_g[(int64_t)t * N + (int64_t)(nt0 + i) * 16 + nl];
      }
    }
  };

  v4i acc[8][4];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[mt][i] = (v4i){0, 0, 0, 0};

  load_a(0);
  load_w(0);
  store_a(0);
  __syncthreads();

  for (int t = 0; t < T; ++t) {
    const int buf = t & 1;
    uint4 wcur[4];
    int sgcur[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      wcur[i] = wreg[i];
      sgcur[i] = sgreg[i];
    }
    if (t + 1 < T) {
      load_a(t + 1);
      load_w(t + 1);
    }
    if constexpr (MODE == kGroupLinear) {
      v4i a[8][2];
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          a[mt][j] = *(const v4i*)(&lds_a[buf][(mt * 16 + nl) * kLdsRow + j * 64 + kc * 16]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t d[4] = {wcur[i].x, wcur[i].y, wcur[i].z, wcur[i].w};
        int o[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_x16(d[j], o[2 * j], o[2 * j + 1]);
        const v4i b0 = {o[0], o[1], o[2], o[3]}, b1 = {o[4], o[5], o[6], o[7]};
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
          v4i part = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][0], b0, (v4i){0, 0, 0, 0}, 0, 0, 0);
          part = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt][1], b1, part, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[mt][i][r] += (part[r] >> 4) * sgcur[i];
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        v4i a[8];
#pragma unroll
        for (int mt = 0; mt < 8; ++mt)
          a[mt] = *(const v4i*)(&lds_a[buf][(mt * 16 + nl) * kLdsRow + j * 64 + kc * 16]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t d0 = j ? wcur[i].z : wcur[i].x, d1 = j ? wcur[i].w : wcur[i].y;
          int o[4];
          if constexpr (MODE == kPerChannel) {
            unpack_x16(d0, o[0], o[1]);
            unpack_x16(d1, o[2], o[3]);
          } else if constexpr (MODE == kGroupClamp) {
            const _Float16 hs = (_Float16)(float)sgcur[i];
            const h2 s2 = {hs, hs};
            unpack_group_clamp(d0, s2, o[0], o[1]);
            unpack_group_clamp(d1, s2, o[2], o[3]);
          } else {
            const GroupFusedConsts g = make_group_fused(sgcur[i]);
            unpack_group_fused(d0, g, o[0], o[1]);
            unpack_group_fused(d1, g, o[2], o[3]);
          }
          const v4i b = {o[0], o[1], o[2], o[3]};
#pragma unroll
          for (int mt = 0; mt < 8; ++mt)
            acc[mt][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt], b, acc[mt][i], 0, 0, 0);
        }
      }
    }
    if (t + 1 < T) store_a(buf ^ 1);
    __syncthreads();
  }

  // ---- fused Dequant epilogue: lane holds column nl of each tile, rows 4*kc + r
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (nt0 + i >= ntiles) continue;
    const int n = (nt0 + i) * 16 + nl;
    const float sw = (float)p.s_w[n];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + mt * 16 + 4 * kc + r;
        if (m < M) {
          int v = acc[mt][i][r];
          if constexpr (MODE == kPerChannel) v >>= 4;
          const int64_t o = (int64_t)m * N + n;
          p.y[o] = dequant(v, p.s_a[m], sw);
          if (p.acc_out) p.acc_out[o] = v;
        }
      }
    }
  }
}

template <int MODE>
static int launch_mode(const GemmParams& p, hipStream_t st) {
  const int tiles_m = (p.M + kBM - 1) / kBM;
  const int tiles_n = (p.N + kBN - 1) / kBN;
  const int64_t grid = (int64_t)tiles_m * tiles_n;
  if (grid > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "prefill: grid too large");
  hipLaunchKernelGGL((gemm_prefill_kernel<MODE>), dim3((unsigned)grid), dim3(256), 0, st, p,
                     tiles_m, tiles_n);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "prefill gemm launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

int launch_gemm_prefill(const GemmParams& p, int mode, hipStream_t st) {
  switch (mode) {
    case kPerChannel: return launch_mode<kPerChannel>(p, st);
    case kGroupLinear: return launch_mode<kGroupLinear>(p, st);
    case kGroupClamp: return launch_mode<kGroupClamp>(p, st);
    case kGroupFused: return launch_mode<kGroupFused>(p, st);
  }
  return set_error(QQQ_ERR_SHAPE, "unknown mode %d", mode);
}

}  // namespace qqq
