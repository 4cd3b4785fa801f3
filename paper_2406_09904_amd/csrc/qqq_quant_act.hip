// qqq_quant_act: per-token dynamic symmetric int8 quantisation of fp16 activations
// (Sec. 4.1 "Algorithm" of the QQQ paper; s_A of Fig. 3).  One workgroup per token: the row is
// read once into registers, |max| is reduced across the workgroup, and the row is divided by
// the scale, rounded half-to-even and written as int8.  A pure streaming pass: 2 B in, 1 B out.
#include "qqq_internal.h"

namespace qqq {

__device__ __forceinline__ uint32_t block_max_u32(uint32_t v, uint32_t* smem) {
  v = wave_max_u32(v);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) smem[wave] = v;
  __syncthreads();
  const int nw = blockDim.x >> 6;
  uint32_t r = 0;
  for (int i = 0; i < nw; ++i) r = max(r, smem[i]);
  return r;
}

// Optional by-product for the per-group prefill GEMM's biased conversion (see qqq_group_bias.hip):
// the negated sum of each group's 128 codes, split as 128*hi + lo.  A group is 16 consecutive
// vectors, i.e. one 16-lane row of a wave, so the sum is a row reduction of data-parallel adds.
struct RowSums {
  int8_t* lo;  // [M][Gp] or nullptr
  int8_t* hi;
  int G, Gp;
};
__device__ __forceinline__ void emit_group_sum(const RowSums& rs, int64_t m, int idx, uint2 codes) {
  int s = __builtin_amdgcn_sdot4((int)codes.x, 0x01010101, 0, false);
  s = __builtin_amdgcn_sdot4((int)codes.y, 0x01010101, s, false);
  s += __builtin_amdgcn_update_dpp(0, s, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
  s += __builtin_amdgcn_update_dpp(0, s, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
  s += __builtin_amdgcn_update_dpp(0, s, 0x141, 0xF, 0xF, false);  // row_half_mirror
  s += __builtin_amdgcn_update_dpp(0, s, 0x140, 0xF, 0xF, false);  // row_mirror
  const int g = idx >> 4;
  if ((threadIdx.x & 15) == 0 && g < rs.G) {
    const int neg = -s;
    rs.lo[m * rs.Gp + g] = (int8_t)(neg & 127);
    rs.hi[m * rs.Gp + g] = (int8_t)(neg >> 7);
  }
}

// VPT > 0: the row fits in VPT 128-bit vectors per thread and stays in registers.
// VPT == 0: any K; the row is read twice (the second read hits L2).
template <int VPT, bool SUMS>
__global__ __launch_bounds__(256) void quant_act_kernel(const uint4* __restrict__ a, int64_t lda_vec,
                                                        int nvec, uint2* __restrict__ a_q,
                                                        float* __restrict__ s_a, const RowSums rs) {
  __shared__ uint32_t smem[4];
  const int64_t m = blockIdx.x;
  const uint4* row = a + m * lda_vec;
  uint2* out = a_q + m * (int64_t)nvec;
  uint32_t amax_bits = 0;
  if constexpr (VPT > 0) {
    uint4 v[VPT];
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const int idx = threadIdx.x + 256 * j;
      v[j] = make_uint4(0, 0, 0, 0);
      if (idx < nvec) v[j] = row[idx];
      amax_bits = absmax_bits(v[j], amax_bits);
    }
    amax_bits = block_max_u32(amax_bits, smem);
    const float amax = half_bits_to_float(amax_bits);
    const float s = amax / 127.0f;
    if (threadIdx.x == 0) s_a[m] = (amax == 0.0f) ? 0.0f : s;
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const int idx = threadIdx.x + 256 * j;
      uint2 o = make_uint2(0, 0);
      if (idx < nvec && amax != 0.0f) {
        o.x = quant4(v[j].x, v[j].y, s);
        o.y = quant4(v[j].z, v[j].w, s);
      }
      if (idx < nvec) out[idx] = o;
      if constexpr (SUMS) emit_group_sum(rs, m, idx, o);  // every lane takes part in the row reduction
    }
  } else {
    for (int idx = threadIdx.x; idx < nvec; idx += 256) amax_bits = absmax_bits(row[idx], amax_bits);
    amax_bits = block_max_u32(amax_bits, smem);
    const float amax = half_bits_to_float(amax_bits);
    const float s = amax / 127.0f;
    if (threadIdx.x == 0) s_a[m] = (amax == 0.0f) ? 0.0f : s;
    for (int i0 = 0; i0 < nvec; i0 += 256) {
      const int idx = i0 + threadIdx.x;
      uint2 o = make_uint2(0, 0);
      if (idx < nvec && amax != 0.0f) {
        const uint4 v = row[idx];
        o.x = quant4(v.x, v.y, s);
        o.y = quant4(v.z, v.w, s);
      }
      if (idx < nvec) out[idx] = o;
      if constexpr (SUMS) emit_group_sum(rs, m, idx, o);
    }
  }
  if constexpr (SUMS) {  // zero padding of the group axis
    for (int g = rs.G + (int)threadIdx.x; g < rs.Gp; g += 256) {
      rs.lo[m * rs.Gp + g] = 0;
      rs.hi[m * rs.Gp + g] = 0;
    }
  }
}

template <bool SUMS>
static void launch_vpt(const uint4* ap, int64_t lda_vec, int nvec, uint2* qp, float* s_a, const RowSums& rs,
                       int64_t M, hipStream_t st) {
  const dim3 grid((unsigned)M), block(256);
  const int vpt = (nvec + 255) / 256;
  if (vpt <= 1)
    hipLaunchKernelGGL((quant_act_kernel<1, SUMS>), grid, block, 0, st, ap, lda_vec, nvec, qp, s_a, rs);
  else if (vpt <= 2)
    hipLaunchKernelGGL((quant_act_kernel<2, SUMS>), grid, block, 0, st, ap, lda_vec, nvec, qp, s_a, rs);
  else if (vpt <= 4)
    hipLaunchKernelGGL((quant_act_kernel<4, SUMS>), grid, block, 0, st, ap, lda_vec, nvec, qp, s_a, rs);
  else if (vpt <= 8)
    hipLaunchKernelGGL((quant_act_kernel<8, SUMS>), grid, block, 0, st, ap, lda_vec, nvec, qp, s_a, rs);
  else
    hipLaunchKernelGGL((quant_act_kernel<0, SUMS>), grid, block, 0, st, ap, lda_vec, nvec, qp, s_a, rs);
}

// r_lo/r_hi: optional [M][Gp] outputs of the per-group row sums (K % 128 == 0 required then)
int launch_quant_act(const void* a, int64_t M, int64_t K, int64_t lda, int8_t* a_q, float* s_a,
                     hipStream_t st, int8_t* r_lo, int8_t* r_hi) {
  const int nvec = (int)(K / 8);
  RowSums rs;
  rs.lo = r_lo;
  rs.hi = r_hi;
  rs.G = (int)(K / 128);
  rs.Gp = (rs.G + 31) & ~31;
  if (r_lo && r_hi)
    launch_vpt<true>((const uint4*)a, lda / 8, nvec, (uint2*)a_q, s_a, rs, M, st);
  else
    launch_vpt<false>((const uint4*)a, lda / 8, nvec, (uint2*)a_q, s_a, rs, M, st);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "quant_act launch: %s", hipGetErrorString(e));
  route_note(r_lo ? "quant_act (+ group row sums)" : "quant_act");
  return QQQ_OK;
}

}  // namespace qqq
