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

// VPT > 0: the row fits in VPT 128-bit vectors per thread and stays in registers.
// VPT == 0: any K; the row is read twice (the second read hits L2).
template <int VPT>
__global__ __launch_bounds__(256) void quant_act_kernel(const uint4* __restrict__ a, int64_t lda_vec,
                                                        int nvec, uint2* __restrict__ a_q,
                                                        float* __restrict__ s_a) {
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
      if (idx < nvec) {
        uint2 o = make_uint2(0, 0);
        if (amax != 0.0f) {
          o.x = quant4(v[j].x, v[j].y, s);
          o.y = quant4(v[j].z, v[j].w, s);
        }
        out[idx] = o;
      }
    }
  } else {
    for (int idx = threadIdx.x; idx < nvec; idx += 256) amax_bits = absmax_bits(row[idx], amax_bits);
    amax_bits = block_max_u32(amax_bits, smem);
    const float amax = half_bits_to_float(amax_bits);
    const float s = amax / 127.0f;
    if (threadIdx.x == 0) s_a[m] = (amax == 0.0f) ? 0.0f : s;
    for (int idx = threadIdx.x; idx < nvec; idx += 256) {
      uint2 o = make_uint2(0, 0);
      if (amax != 0.0f) {
        const uint4 v = row[idx];
        o.x = quant4(v.x, v.y, s);
        o.y = quant4(v.z, v.w, s);
      }
      out[idx] = o;
    }
  }
}

int launch_quant_act(const void* a, int64_t M, int64_t K, int64_t lda, int8_t* a_q, float* s_a,
                     hipStream_t st) {
  const int nvec = (int)(K / 8);
  const int64_t lda_vec = lda / 8;
  const dim3 grid((unsigned)M), block(256);
  const uint4* ap = (const uint4*)a;
  uint2* qp = (uint2*)a_q;
  const int vpt = (nvec + 255) / 256;
  if (vpt <= 1)
    hipLaunchKernelGGL(quant_act_kernel<1>, grid, block, 0, st, ap, lda_vec, nvec, qp, s_a);
  else if (vpt <= 2)
    hipLaunchKernelGGL(quant_act_kernel<2>, grid, block, 0, st, ap, lda_vec, nvec, qp, s_a);
  else if (vpt <= 4)
    hipLaunchKernelGGL(quant_act_kernel<4>, grid, block, 0, st, ap, lda_vec, nvec, qp, s_a);
  else if (vpt <= 8)
    hipLaunchKernelGGL(quant_act_kernel<8>, grid, block, 0, st, ap, lda_vec, nvec, qp, s_a);
  else
    hipLaunchKernelGGL(quant_act_kernel<0>, grid, block, 0, st, ap, lda_vec, nvec, qp, s_a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "quant_act launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

}  // namespace qqq
