// Offline weight front-end: symmetric round-to-nearest int4 codes and their scales from fp16
// weights (the inputs of Sec. 3.3.1's offline scale adjustment and of the offline boxes of
// Fig. 5 in the QQQ paper).  The row of an output channel is read once, the block maxima
// (channel: workgroup reduction; group of 128 = one 16-lane row of a wave) are reduced with
// data-parallel primitives, the row is divided by the stored fp16 scale, rounded half to
// even, clamped to [-7,7] and written eight codes per word in the natural nibble format.
// Per-group, the same pass finds the channel's largest dequantised magnitude, from which the
// fp16->int8 scale s_Wc and the fused scales s*_Wg = s_Wg / s_Wc follow.  A streaming pass:
// 2 B in, 0.5 B out per weight.
#include "qqq_internal.h"

namespace qqq {

namespace {

constexpr float kStarCap = 18.203125f;  // largest fp16 s with rne(7 * s) <= 127
constexpr int kWaves = 4;               // waves per workgroup, one channel per wave at a time

__device__ __forceinline__ uint32_t row16_max_u32(uint32_t v) {  // max over a 16-lane row, in every lane
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));
  return v;
}

// fp16 bits of amax / q (fp32 IEEE division, one rounding to fp16)
__device__ __forceinline__ uint16_t scale_bits(float amax, float q) {
  return __builtin_bit_cast(uint16_t, (_Float16)(amax / q));
}

// clamp(rne(w / s), -7, 7), the quotient being the correctly rounded fp32 one, computed without
// dividing in the common case: q~ = w * rcp(s) is within 2^-22 relative of w/s, and so is the
// rounded quotient (2^-24); for |q~| < 8 both are then within 2^-19 absolute of w/s, so unless q~
// lies within 2^-16 of a half-integer the two round to the same integer.  Beyond 8 in magnitude
// either rounding clamps to +-7.  Only near a tie the IEEE division decides.
__device__ __forceinline__ int rtn_code(uint32_t h16, float s, float rs) {
  const float w = half_bits_to_float(h16);
  const float q = w * rs;
  float r = __builtin_rintf(q);
  if (__builtin_fabsf(q - r) > 0.5f - 0x1p-16f) r = __builtin_rintf(w / s);
  return (int)__builtin_amdgcn_fmed3f(r, -7.0f, 7.0f);
}

// eight fp16 weights -> eight nibbles; *cmax = max |code|
template <bool CMAX>
__device__ __forceinline__ uint32_t quant8(uint4 v, float s, float rs, int* cmax) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  uint32_t out = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c0 = rtn_code(w[i] & 0xFFFFu, s, rs), c1 = rtn_code(w[i] >> 16, s, rs);
    if constexpr (CMAX) *cmax = max(*cmax, max(abs(c0), abs(c1)));
    out |= (uint32_t)(c0 & 0xF) << (8 * i) | (uint32_t)(c1 & 0xF) << (8 * i + 4);
  }
  return out;
}

struct GroupOut {
  uint16_t* s_wg;    // [G][N] or nullptr
  uint16_t* s_star;  // [G][N]
  int8_t* s_int;     // [G][N] or nullptr
  int G;
  int rows_log2;     // channels per workgroup = 1 << rows_log2, at least kWaves
};

__device__ __forceinline__ uint32_t block_max(uint32_t v, uint32_t* smem) {
  v = wave_max_u32(v);
  if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
  __syncthreads();
  const uint32_t r = max(max(smem[0], smem[1]), max(smem[2], smem[3]));
  __syncthreads();
  return r;
}

}  // namespace

// Per-channel: one workgroup per channel.
// VPT > 0: the row fits in VPT 128-bit vectors per thread and stays in registers.
// VPT == 0: any K; the row is read twice (the second read hits L2).
template <int VPT>
__global__ __launch_bounds__(256) void quant_weight_channel_kernel(const uint4* __restrict__ w, int64_t ldw_vec,
                                                                   int nvec, uint32_t* __restrict__ w_nat,
                                                                   uint16_t* __restrict__ s_w) {
  __shared__ uint32_t smem[4];
  const int64_t n = blockIdx.x;
  const uint4* row = w + n * ldw_vec;
  uint32_t* out = w_nat + n * (int64_t)nvec;
  constexpr int kIter = VPT > 0 ? VPT : 1;
  uint4 v[kIter];
  uint32_t amax_bits = 0;
  if constexpr (VPT > 0) {
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const int idx = threadIdx.x + 256 * j;
      v[j] = make_uint4(0, 0, 0, 0);
      if (idx < nvec) v[j] = row[idx];
      amax_bits = absmax_bits(v[j], amax_bits);
    }
  } else {
    for (int idx = threadIdx.x; idx < nvec; idx += 256) amax_bits = absmax_bits(row[idx], amax_bits);
  }
  amax_bits = block_max(amax_bits, smem);
  const uint16_t sb = scale_bits(half_bits_to_float(amax_bits), 7.0f);
  const float s = half_bits_to_float(sb);
  if (threadIdx.x == 0) s_w[n] = sb;
  const float rs = __builtin_amdgcn_rcpf(s);
  if (s == 0.0f) {  // uniform over the workgroup
    for (int idx = threadIdx.x; idx < nvec; idx += 256) out[idx] = 0u;
    return;
  }
  if constexpr (VPT > 0) {
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const int idx = threadIdx.x + 256 * j;
      if (idx < nvec) out[idx] = quant8<false>(v[j], s, rs, nullptr);
    }
  } else {
    for (int idx = threadIdx.x; idx < nvec; idx += 256) out[idx] = quant8<false>(row[idx], s, rs, nullptr);
  }
}

// Per-group: one wave per channel at a time, `rows` channels per workgroup.  A group of 128 is 16
// consecutive vectors, i.e. one 16-lane row of a wave, so its scale needs no memory of the rest of
// the channel: the wave streams the row once, four vectors per lane at a time, and leaves the group
// scales in LDS; the channel's s_Wc follows from a wave reduction at the end of the row.
// The scale tables are [G][N]: one channel owns one element of every table row.  The workgroup's
// LDS stage is [G][rows], and after a barrier the tables are written in runs of `rows` elements,
// the division s_Wg / s_Wc being done there.  STAGED == false (a table too tall for LDS): the
// wave reads its row a second time (from L2) and writes its table elements one by one.
template <bool STAGED>
__global__ __launch_bounds__(64 * kWaves) void quant_weight_group_kernel(const uint4* __restrict__ w,
                                                                         int64_t ldw_vec, int nvec, int64_t N,
                                                                         uint32_t* __restrict__ w_nat,
                                                                         uint16_t* __restrict__ s_wc,
                                                                         const GroupOut go) {
  extern __shared__ uint16_t stage[];  // [G][rows] s_Wg bits, then [rows] s_Wc bits
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rows = 1 << go.rows_log2;
  const int64_t n0 = (int64_t)blockIdx.x << go.rows_log2;
  auto emit = [&](int64_t at, uint16_t wg_bits, float wc) {
    const float sg = half_bits_to_float(wg_bits);
    uint16_t star = 0;
    if (wc != 0.0f) {
      const _Float16 h = (_Float16)(sg / wc);
      star = __builtin_bit_cast(uint16_t, (float)h > kStarCap ? (_Float16)kStarCap : h);
    }
    go.s_star[at] = star;
    if (go.s_wg) go.s_wg[at] = wg_bits;
    if (go.s_int) go.s_int[at] = (int8_t)fminf(fmaxf(__builtin_rintf(half_bits_to_float(star)), 1.0f), 18.0f);
  };
  for (int r = wave; r < rows; r += kWaves) {
    const int64_t n = n0 + r;
    if (n >= N) break;
    const uint4* row = w + n * ldw_vec;
    uint32_t* out = w_nat + n * (int64_t)nvec;
    uint32_t dmax_bits = 0;  // bits of max |code * s_Wg|, a non-negative float
#pragma unroll 1
    for (int i0 = 0; i0 < nvec; i0 += 256) {
      uint4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int idx = i0 + 64 * j + lane;
        v[j] = make_uint4(0, 0, 0, 0);
        if (idx < nvec) v[j] = row[idx];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int idx = i0 + 64 * j + lane;
        const uint32_t gmax = row16_max_u32(absmax_bits(v[j], 0));
        const uint16_t sgb = scale_bits(half_bits_to_float(gmax), 7.0f);
        const float sg = half_bits_to_float(sgb);
        int cmax = 0;
        uint32_t codes = 0;
        if (sg != 0.0f) codes = quant8<true>(v[j], sg, __builtin_amdgcn_rcpf(sg), &cmax);
        if (idx < nvec) out[idx] = codes;
        dmax_bits = max(dmax_bits, __builtin_bit_cast(uint32_t, (float)cmax * sg));
        if constexpr (STAGED)
          if ((lane & 15) == 0 && idx < nvec) stage[((idx >> 4) << go.rows_log2) + r] = sgb;
      }
    }
    dmax_bits = wave_max_u32(dmax_bits);
    const uint16_t wcb = scale_bits(__builtin_bit_cast(float, dmax_bits), 127.0f);
    if (lane == 0) s_wc[n] = wcb;
    if constexpr (STAGED) {
      if (lane == 0) stage[(go.G << go.rows_log2) + r] = wcb;
    } else {
      const float wc = half_bits_to_float(wcb);
      for (int i0 = 0; i0 < nvec; i0 += 64) {  // the group maxima again, from L2
        const int idx = i0 + lane;
        const uint4 vec = idx < nvec ? row[idx] : make_uint4(0, 0, 0, 0);
        const uint32_t gmax = row16_max_u32(absmax_bits(vec, 0));
        if ((lane & 15) == 0 && idx < nvec)
          emit((int64_t)(idx >> 4) * N + n, scale_bits(half_bits_to_float(gmax), 7.0f), wc);
      }
    }
  }
  if constexpr (STAGED) {
    __syncthreads();
    const int cells = go.G << go.rows_log2;
    for (int c = threadIdx.x; c < cells; c += 64 * kWaves) {
      const int r = c & (rows - 1);
      if (n0 + r < N)
        emit((int64_t)(c >> go.rows_log2) * N + n0 + r, stage[c], half_bits_to_float(stage[cells + r]));
    }
  }
}

int launch_quant_weight(const void* w, int64_t N, int64_t K, int64_t ldw, bool grouped, uint32_t* w_nat,
                        uint16_t* s_ch, uint16_t* s_wg, uint16_t* s_star, int8_t* s_int, hipStream_t st) {
  if (N == 0) return QQQ_OK;
  const uint4* wp = (const uint4*)w;
  const int64_t ldw_vec = ldw / 8;
  const int nvec = (int)(K / 8);
  if (!grouped) {
    const dim3 grid((unsigned)N), block(256);
    const int vpt = (nvec + 255) / 256;
#define QQQ_QW(V) \
  hipLaunchKernelGGL((quant_weight_channel_kernel<V>), grid, block, 0, st, wp, ldw_vec, nvec, w_nat, s_ch)
    if (vpt <= 1) QQQ_QW(1);
    else if (vpt <= 2) QQQ_QW(2);
    else if (vpt <= 4) QQQ_QW(4);
    else if (vpt <= 8) QQQ_QW(8);
    else if (vpt <= 16) QQQ_QW(16);
    else QQQ_QW(0);
#undef QQQ_QW
  } else {
    GroupOut go;
    go.s_wg = s_wg;
    go.s_star = s_star;
    go.s_int = s_int;
    go.G = (int)(K / QQQ_GROUP);
    // channels per workgroup: as many as keep about four workgroups per compute unit, at least one
    // per wave and at most 32 (one 64-byte run of fp16 per table row), with a stage of at most 48 KB
    auto stage_bytes = [&](int lg) { return (((size_t)go.G << lg) + ((size_t)1 << lg)) * 2; };
    int lg = 5;
    while (lg > 2 && (N >> lg) < 4 * (int64_t)num_cus()) --lg;
    while (lg > 2 && stage_bytes(lg) > 48u * 1024u) --lg;
    go.rows_log2 = lg;
    const bool staged = stage_bytes(lg) <= 48u * 1024u;
    const dim3 grid((unsigned)((N + (1 << lg) - 1) >> lg)), block(64 * kWaves);
    if (staged)
      hipLaunchKernelGGL((quant_weight_group_kernel<true>), grid, block, stage_bytes(lg), st, wp, ldw_vec, nvec, N,
                         w_nat, s_ch, go);
    else
      hipLaunchKernelGGL((quant_weight_group_kernel<false>), grid, block, 0, st, wp, ldw_vec, nvec, N, w_nat,
                         s_ch, go);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "quant_weight launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

}  // namespace qqq
