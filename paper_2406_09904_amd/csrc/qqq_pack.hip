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

// One thread per packed 16-byte vector (chunk, lane): the lane's dwords i = 0..3 are natural words
// 16t + 2kc + {0, 1} and 16t + 8 + 2kc + {0, 1} of row 16nt + nl, i.e. two 8-byte pieces 32 bytes apart.
// The four lanes nl, nl+16, nl+32, nl+48 of a wave cover one row's 64-byte line in full, so a wave moves
// 16 whole lines with two 8-byte loads per lane and writes (or reads) 1 KiB of the packed stream with one
// 16-byte access per lane.
__global__ __launch_bounds__(256) void pack_kernel(const uint32_t* __restrict__ src,
                                                   uint32_t* __restrict__ dst, int64_t vectors, int ntiles,
                                                   int words_per_row, bool inverse) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= vectors) return;
  const int lane = (int)(v & 63);
  const int64_t chunk = v >> 6;  // chunk = t * (N/16) + nt
  const int64_t nt = chunk % ntiles;
  const int t = (int)(chunk / ntiles);
  const int nl = lane & 15, kc = lane >> 4;
  const int64_t nat = (nt * 16 + nl) * words_per_row + 16 * t + 2 * kc;
  if (!inverse) {
    const uint2 lo = *reinterpret_cast<const uint2*>(src + nat);
    const uint2 hi = *reinterpret_cast<const uint2*>(src + nat + 8);
    *reinterpret_cast<uint4*>(dst + v * 4) =
        make_uint4(shuffle_nibbles_fwd(lo.x), shuffle_nibbles_fwd(lo.y), shuffle_nibbles_fwd(hi.x),
                   shuffle_nibbles_fwd(hi.y));
  } else {
    const uint4 p = *reinterpret_cast<const uint4*>(src + v * 4);
    *reinterpret_cast<uint2*>(dst + nat) = make_uint2(shuffle_nibbles_inv(p.x), shuffle_nibbles_inv(p.y));
    *reinterpret_cast<uint2*>(dst + nat + 8) = make_uint2(shuffle_nibbles_inv(p.z), shuffle_nibbles_inv(p.w));
  }
}

int launch_pack(const uint32_t* src, int64_t N, int64_t K, uint32_t* dst, bool inverse,
                hipStream_t st) {
  // natural words are read / written as 8-byte pairs, packed ones as 16-byte vectors
  if ((reinterpret_cast<uintptr_t>(inverse ? (const void*)dst : (const void*)src) & 7u) ||
      (reinterpret_cast<uintptr_t>(inverse ? (const void*)src : (const void*)dst) & 15u))
    return set_error(QQQ_ERR_SHAPE, "pack: the natural words must be 8-byte and the packed buffer 16-byte aligned");
  const int64_t vectors = N * (K / 8) / 4;
  const int64_t blocks = (vectors + 255) / 256;
  if (blocks > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "pack: too many words");
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, vectors,
                     (int)(N / 16), (int)(K / 8), inverse);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "pack launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

}  // namespace qqq
