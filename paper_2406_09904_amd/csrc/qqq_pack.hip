// qqq_pack_w4 / qqq_unpack_w4: natural int4 words <-> the device tile layout (offline, untimed).
// Sec. 3.3.1 of the QQQ paper prepares the weights offline; the layout itself is this library's.
#include "qqq_internal.h"

namespace qqq {

// packed nibble q takes natural nibble 4*(q%2) + q/2  (order 0,4,1,5,2,6,3,7)
__device__ __forceinline__ uint32_t shuffle_nibbles_fwd(uint32_t w) {
  uint32_t out = 0;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int src = 4 * (q & 1) + (q >> 1);
    out |= ((w >> (4 * src)) & 0xFu) << (4 * q);
  }
  return out;
}
__device__ __forceinline__ uint32_t shuffle_nibbles_inv(uint32_t w) {
  uint32_t out = 0;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int src = 4 * (q & 1) + (q >> 1);
    out |= ((w >> (4 * q)) & 0xFu) << (4 * src);
  }
  return out;
}

// One thread per 32-bit word.  Packed word index = (((t*(N/16) + nt)*64 + lane)*4 + i).
__global__ __launch_bounds__(256) void pack_kernel(const uint32_t* __restrict__ src,
                                                   uint32_t* __restrict__ dst, int64_t total, int ntiles,
                                                   int words_per_row, bool inverse) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int i = (int)(idx & 3);
  const int lane = (int)((idx >> 2) & 63);
  const int64_t chunk = idx >> 8;  // chunk = t * (N/16) + nt
  const int64_t nt = chunk % ntiles;
  const int t = (int)(chunk / ntiles);
  const int nl = lane & 15, kc = lane >> 4;
  const int64_t n = nt * 16 + nl;
  // k of nibble 0 of this word = 128t + 64*(i/2) + 16kc + 8*(i%2): always a multiple of 8
  const int word = 16 * t + 8 * (i >> 1) + 2 * kc + (i & 1);
  const int64_t nat = n * words_per_row + word;
  if (!inverse)
    dst[idx] = shuffle_nibbles_fwd(src[nat]);
  else
    dst[nat] = shuffle_nibbles_inv(src[idx]);
}

int launch_pack(const uint32_t* src, int64_t N, int64_t K, uint32_t* dst, bool inverse,
                hipStream_t st) {
  const int64_t total = N * (K / 8);
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "pack: too many words");
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, total,
                     (int)(N / 16), (int)(K / 8), inverse);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "pack launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

}  // namespace qqq
