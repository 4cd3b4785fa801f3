// LDS-tiled W4A8 GEMM for M > 64 (prefill): bound by the int8 MFMA pipe.
//
// A workgroup of NW waves computes a 128 x (64*NW) tile of Y with v_mfma_i32_32x32x32_i8.  The
// waves split N (64 channels = two 32-wide MFMA column tiles each) and share the activation tile
// through LDS, so every packed weight fragment is loaded from global memory straight into the
// registers of the one wave that needs it, converted to int8 once (Sec. 3.3.1 / 3.3.2 of the QQQ
// paper) and fed to 4 MFMAs.  The activation tile (128 rows x 128 k int8) is double-buffered in
// LDS with a 16-byte row pad that keeps the 128-bit operand reads free of bank conflicts.
// One k-step = 128 k = one scale group = four MFMA k-steps of 32.
//
// Operand mapping of the 32x32x32 MFMA: lane l supplies row/column l%32 and the 16 k-bytes
// 16*(l/32)..+15 of the step.  In the packed layout a 32-channel tile is two adjacent 1 KiB
// chunks; lane (n32, h) takes the 16-byte pieces of chunk n32/16 at (n32%16, kc=h) and
// (n32%16, kc=h+2): the first holds its k-bytes for MFMA steps 0 and 2, the second for 1 and 3.
#include "qqq_internal.h"

namespace qqq {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBM = 128, kBK = 128;
constexpr int kLdsRow = kBK + 16;  // bytes per LDS row of A

template <int MODE>
__device__ __forceinline__ v4i make_b(uint32_t d0, uint32_t d1, int sg) {
  int o[4];
  if constexpr (MODE == kPerChannel) {
    unpack_x16(d0, o[0], o[1]);
    unpack_x16(d1, o[2], o[3]);
  } else if constexpr (MODE == kGroupClamp) {
    const _Float16 hs = (_Float16)(float)sg;
    const h2 s2 = {hs, hs};
    unpack_group_clamp(d0, s2, o[0], o[1]);
    unpack_group_clamp(d1, s2, o[2], o[3]);
  } else {
    const GroupFusedConsts g = make_group_fused(sg);
    unpack_group_fused(d0, g, o[0], o[1]);
    unpack_group_fused(d1, g, o[2], o[3]);
  }
  return (v4i){o[0], o[1], o[2], o[3]};
}

template <int MODE, int NW>
__global__ __launch_bounds__(NW * 64, 8 / NW) void gemm_prefill_kernel(const GemmParams p, const int tiles_m,
                                                               const int tiles_n) {
  constexpr int kThreads = NW * 64;
  constexpr int kBN = NW * 64;
  constexpr int kCopy = (kBM * kBK / 16) / kThreads;  // 16-byte pieces of the A tile per thread
  __shared__ __attribute__((aligned(16))) int8_t lds_a[2][kBM * kLdsRow];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n32 = lane & 31, h = lane >> 5;
  const int T = p.T, N = p.N, M = p.M;
  const int64_t K = p.K;
  const int ntiles = N >> 4;

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
  // this wave's two 32-channel tiles; nt16[c] = the 16-channel chunk this lane reads for tile c
  int nt16[2];
  bool nvalid[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    nt16[c] = tn * (kBN / 16) + wave * 4 + c * 2 + (n32 >> 4);
    nvalid[c] = nt16[c] < ntiles;
  }

  // global -> LDS copy assignment: 8 threads per row (16 B each)
  const int cr = tid >> 3, cc = tid & 7;
  v4i areg[kCopy];
  auto load_a = [&](int t) {
#pragma unroll
    for (int ps = 0; ps < kCopy; ++ps) {
      const int m = m0 + ps * (kThreads / 8) + cr;
      areg[ps] = (v4i){0, 0, 0, 0};
      if (m < M) areg[ps] = *(const v4i*)(p.a_q + (int64_t)m * K + (int64_t)t * kBK + cc * 16);
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int ps = 0; ps < kCopy; ++ps)
      *(v4i*)(&lds_a[buf][(ps * (kThreads / 8) + cr) * kLdsRow + cc * 16]) = areg[ps];
  };
  uint4 wreg[2][2];  // [tile][piece]
  int sgreg[2];
  auto load_w = [&](int t) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      wreg[c][0] = make_uint4(0, 0, 0, 0);
      wreg[c][1] = make_uint4(0, 0, 0, 0);
      sgreg[c] = 0;
      if (nvalid[c]) {
        const uint4* base = p.w + ((int64_t)t * ntiles + nt16[c]) * 64 + (n32 & 15);
        wreg[c][0] = base[16 * h];
        wreg[c][1] = base[16 * (h + 2)];
        if constexpr (MODE != kPerChannel)
          sgreg[c] = (int)p.s_g[(int64_t)t * N + (int64_t)nt16[c] * 16 + (n32 & 15)];
      }
    }
  };

  v16i acc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0;

  load_a(0);
  load_w(0);
  store_a(0);
  __syncthreads();

  for (int t = 0; t < T; ++t) {
    const int buf = t & 1;
    uint4 wcur[2][2];
    int sgcur[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      wcur[c][0] = wreg[c][0];
      wcur[c][1] = wreg[c][1];
      sgcur[c] = sgreg[c];
    }
    if (t + 1 < T) {
      load_a(t + 1);
      load_w(t + 1);
    }
    const int8_t* abase = &lds_a[buf][n32 * kLdsRow + h * 16];
#pragma unroll
    for (int s = 0; s < 4; ++s) {  // MFMA k-steps of 32
      v4i a[4];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) a[mt] = *(const v4i*)(abase + mt * 32 * kLdsRow + s * 32);
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        // step s uses piece s%2, dword pair s/2
        const uint4 pc = wcur[c][s & 1];
        const uint32_t d0 = (s >> 1) ? pc.z : pc.x, d1 = (s >> 1) ? pc.w : pc.y;
        const v4i b = make_b<MODE>(d0, d1, sgcur[c]);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
          acc[mt][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mt], b, acc[mt][c], 0, 0, 0);
      }
    }
    if (t + 1 < T) store_a(buf ^ 1);
    __syncthreads();
  }

  // ---- fused Dequant epilogue: lane holds column n32 of each tile; register v of a 32x32 tile is
  // row 8*(v/4) + 4*h + v%4
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    if (!nvalid[c]) continue;
    const int n = nt16[c] * 16 + (n32 & 15);
    const float sw = (float)p.s_w[n];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + mt * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (m < M) {
          int x = acc[mt][c][v];
          if constexpr (MODE == kPerChannel) x >>= 4;  // exact: the sum is a multiple of 16
          const int64_t o = (int64_t)m * N + n;
          p.y[o] = dequant(x, p.s_a[m], sw);
          if (p.acc_out) p.acc_out[o] = x;
        }
      }
    }
  }
}

static int g_prefill_waves = 0;
void set_prefill_tuning(int waves) { g_prefill_waves = waves; }
int get_prefill_tuning() { return g_prefill_waves; }
static int g_prefill_ksplit = 0;  // 0 = automatic
void set_prefill_ksplit(int s) { g_prefill_ksplit = s; }
int get_prefill_ksplit() { return g_prefill_ksplit; }

template <int MODE, int NW>
static int launch_one(const GemmParams& p, hipStream_t st) {
  const int tiles_m = (p.M + kBM - 1) / kBM;
  const int tiles_n = (p.N + NW * 64 - 1) / (NW * 64);
  const int64_t grid = (int64_t)tiles_m * tiles_n;
  if (grid > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "prefill: grid too large");
  hipLaunchKernelGGL((gemm_prefill_kernel<MODE, NW>), dim3((unsigned)grid), dim3(NW * 64), 0, st, p,
                     tiles_m, tiles_n);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "prefill gemm launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

template <int MODE>
static int launch_mode(const GemmParams& p, hipStream_t st) {
  int nw = 8;
  if (g_prefill_waves == 4) nw = 4;
  if (nw == 8) return launch_one<MODE, 8>(p, st);
  return launch_one<MODE, 4>(p, st);
}

int launch_gemm_prefill(const GemmParams& p, int mode, hipStream_t st) {
  switch (mode) {
    case kPerChannel: return launch_mode<kPerChannel>(p, st);
    case kGroupClamp: return launch_mode<kGroupClamp>(p, st);
    // applying the group scale to partial sums costs more VALU work than the MFMAs hide once
    // the tile has many rows, so both clamp-free requests use the per-weight fp16 FMA route here
    case kGroupLinear:
    case kGroupFused: return launch_mode<kGroupFused>(p, st);
  }
  return set_error(QQQ_ERR_SHAPE, "unknown mode %d", mode);
}

}  // namespace qqq
