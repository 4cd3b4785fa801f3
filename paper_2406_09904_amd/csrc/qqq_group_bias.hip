// Pre-pass of the per-group prefill GEMM's "biased" conversion route (integer group scales <= 16).
//
// That route forms the int8 weight of Sec. 3.3.2 with integer byte arithmetic instead of the fp16
// FMA: with u = code + 8 in [0,15], u*s fits a byte for s <= 16 (one 16-bit packed multiply scales
// four of them) and flipping the top bit reads it as the signed value u*s - 128 = code*s + (8s-128).
// The GEMM therefore accumulates  acc' = acc + sum_g (8*s_g[g][n] - 128) * R[m][g]  with
// R[m][g] = sum of the activation codes of row m in group g, and takes that correction out at the
// end.  The correction is itself a small int8 GEMM over the groups: -R = 128*Rh + Rl with
// Rl in [0,127], Rh in [-127,127] (|R| <= 127*128), and Bc[n][g] = 8*s_g[g][n] - 128 in [-128,0].
// This kernel writes Rl, Rh ([M][Gp]) and Bc ([N][Gp]), Gp = groups rounded up to 32, zero padded.
#include "qqq_internal.h"

namespace qqq {

// one workgroup per activation row; 8 lanes sum one group (16 bytes each)
__device__ __forceinline__ void group_rowsum(const int8_t* __restrict__ a_q, int K, int G, int Gp,
                                             int8_t* __restrict__ r_lo, int8_t* __restrict__ r_hi,
                                             int64_t m) {
  const v4i* row = reinterpret_cast<const v4i*>(a_q + m * (int64_t)K);
  const int chunks = K >> 4;  // 16-byte pieces; 8 per group
  for (int c0 = 0; c0 < chunks; c0 += 256) {
    const int c = c0 + (int)threadIdx.x;
    int sum = 0;
    if (c < chunks) {
      const v4i v = row[c];
#pragma unroll
      for (int i = 0; i < 4; ++i) sum = __builtin_amdgcn_sdot4(v[i], 0x01010101, sum, false);
    }
    // lanes 8j..8j+7 hold one group (chunks is a multiple of 8, so a group never straddles waves)
    sum += __shfl_xor(sum, 1, 64);
    sum += __shfl_xor(sum, 2, 64);
    sum += __shfl_xor(sum, 4, 64);
    if ((threadIdx.x & 7) == 0 && c < chunks) {
      const int g = c >> 3;
      const int neg = -sum;  // the GEMM adds the correction, so the negated sum is stored
      r_lo[m * Gp + g] = (int8_t)(neg & 127);
      r_hi[m * Gp + g] = (int8_t)(neg >> 7);
    }
  }
  for (int g = G + (int)threadIdx.x; g < Gp; g += 256) {
    r_lo[m * Gp + g] = 0;
    r_hi[m * Gp + g] = 0;
  }
}

// Bc[n][g] = code_offset*s_g[g][n] - 128 (code_offset 8; 7 for the route of scales up to 18, whose bytes are
// (7 - code) * s), zero for the padded groups: a transpose of [G][N] into [N][Gp]
// through a 32 x 64 LDS tile, so that reads (along n) and writes (along g) are both contiguous
__device__ __forceinline__ void group_bias_weights(const int8_t* __restrict__ s_g, int N, int G, int Gp,
                                                   int8_t* __restrict__ bc, int tile_n, int tile_g, int code_offset) {
  __shared__ int8_t tile[32][64 + 4];
  const int g0 = tile_g * 32, n0 = tile_n * 64;
  const int tid = threadIdx.x;
  // 32 rows (groups) x 64 columns (channels): 8 passes of 256 threads
#pragma unroll
  for (int pass = 0; pass < 8; ++pass) {
    const int r = pass * 4 + (tid >> 6), c = tid & 63;
    const int g = g0 + r, n = n0 + c;
    tile[r][c] = (g < G && n < N) ? (int8_t)(code_offset * (int)s_g[(int64_t)g * N + n] - 128) : (int8_t)0;
  }
  __syncthreads();
  // 64 channels x 32 groups out: thread -> channel tid/4, 8 consecutive groups
  const int c = tid >> 2, r0 = (tid & 3) * 8;
  const int n = n0 + c;
  if (n < N) {
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo |= (uint32_t)(uint8_t)tile[r0 + i][c] << (8 * i);
      hi |= (uint32_t)(uint8_t)tile[r0 + 4 + i][c] << (8 * i);
    }
    *reinterpret_cast<uint2*>(bc + (int64_t)n * Gp + g0 + r0) = make_uint2(lo, hi);
  }
}

// both parts in one launch: workgroups [0, M) sum the activation rows, the rest transpose the scales
__global__ __launch_bounds__(256) void group_bias_prepass_kernel(const int8_t* __restrict__ a_q,
                                                                 const int8_t* __restrict__ s_g, int M,
                                                                 int N, int K, int G, int Gp,
                                                                 int8_t* __restrict__ r_lo,
                                                                 int8_t* __restrict__ r_hi,
                                                                 int8_t* __restrict__ bc, int code_offset) {
  if ((int)blockIdx.x < M) {
    group_rowsum(a_q, K, G, Gp, r_lo, r_hi, (int64_t)blockIdx.x);
  } else {
    const int t = (int)blockIdx.x - M, tiles_n = (N + 63) / 64;
    group_bias_weights(s_g, N, G, Gp, bc, t % tiles_n, t / tiles_n, code_offset);
  }
}

// with_row_sums == false: the activation quantiser already wrote Rl/Rh (one-call linear path)
int launch_group_bias_prepass(const int8_t* a_q, const int8_t* s_g, int64_t M, int64_t N, int64_t K,
                              int8_t* r_lo, int8_t* r_hi, int8_t* bc, bool with_row_sums, int code_offset,
                              hipStream_t st) {
  const int G = (int)(K / 128), Gp = (G + 31) & ~31;
  if (!with_row_sums) M = 0;
  const int64_t blocks = M + (int64_t)((N + 63) / 64) * (Gp / 32);
  if (blocks > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "group bias pre-pass: grid too large");
  hipLaunchKernelGGL(group_bias_prepass_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a_q, s_g, (int)M,
                     (int)N, (int)K, G, Gp, r_lo, r_hi, bc, code_offset);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "group bias pre-pass launch: %s", hipGetErrorString(e));
  route_note(with_row_sums ? "group-bias pre-pass" : "group-bias pre-pass (scales only)");
  return QQQ_OK;
}

}  // namespace qqq
