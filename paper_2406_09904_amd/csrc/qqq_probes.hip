// Ceiling probes for the benchmark (bench.py --ceilings).  Not part of the W4A8 path: two plain
// kernels that measure what this GPU gives a kernel of the path's shape, so that the roofline
// fractions of the real kernels can be read against a measured ceiling next to the nominal one.
//   stream read : 128-bit coalesced loads of a contiguous buffer, nothing else (decode shapes)
//   int8 MFMA   : the prefill kernel's register dataflow (8 waves, 4 x 2 tiles of 32x32x32 per
//                 wave, two waves per SIMD) with no memory traffic in the loop; the operand
//                 VALUES come from the caller, because the chip's clock under MFMA load depends on them
#include "qqq_prefill_common.h"

namespace qqq {

template <int UNROLL>
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const uint4* __restrict__ p, size_t nvec,
                                                                uint32_t* sink) {
  uint32_t acc = 0;
  const size_t step = (size_t)gridDim.x * 256 * UNROLL;
  for (size_t i = (size_t)blockIdx.x * 256 * UNROLL + threadIdx.x; i < nvec; i += step) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t j = i + 256 * u;
      v[u] = (j < nvec) ? p[j] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) sink[0] = acc;  // keeps the loads alive; practically never true
}

constexpr int kPoolA = 4, kPoolB = 2;  // distinct operand sets the MFMAs rotate through

__global__ __launch_bounds__(512, 1) void probe_mfma_i8_kernel(int iters, const v4i* a_pool, const v4i* b_pool,
                                                              int32_t* sink) {
  v4i a[kPoolA][4], b[kPoolB][2];
#pragma unroll
  for (int i = 0; i < kPoolA; ++i)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) a[i][mt] = a_pool[(i * 4 + mt) * 512 + threadIdx.x];
#pragma unroll
  for (int i = 0; i < kPoolB; ++i)
#pragma unroll
    for (int c = 0; c < 2; ++c) b[i][c] = b_pool[(i * 2 + c) * 512 + threadIdx.x];
  v16i acc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mt][c][v] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < kPoolA; ++s)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
          acc[mt][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[s][mt], b[s % kPoolB][c], acc[mt][c], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[mt][c][v];
  if (s == 0x7fffffff && iters < 0) sink[0] = s;  // never true: iters >= 1
}

}  // namespace qqq

using namespace qqq;

extern "C" {

int qqq_probe_stream_read(const void* buf, size_t bytes, int workgroups, uint32_t* sink, void* stream) {
  if (!buf || !sink) return set_error(QQQ_ERR_NULL, "probe_stream_read: null pointer argument");
  if (bytes < 16 || bytes % 16 != 0 || workgroups < 1 || workgroups > (1 << 20) ||
      (reinterpret_cast<uintptr_t>(buf) & 15u))
    return set_error(QQQ_ERR_SHAPE, "probe_stream_read: bytes must be a multiple of 16, the buffer 16-byte aligned, "
                     "1 <= workgroups <= 2^20");
  hipLaunchKernelGGL(probe_stream_read_kernel<4>, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)buf, bytes / 16, sink);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "probe_stream_read launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

int qqq_probe_mfma_i8(const void* a_pool, const void* b_pool, int iters, int workgroups, int32_t* sink,
                      void* stream) {
  if (!a_pool || !b_pool || !sink) return set_error(QQQ_ERR_NULL, "probe_mfma_i8: null pointer argument");
  if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > 65536 ||
      (reinterpret_cast<uintptr_t>(a_pool) & 15u) || (reinterpret_cast<uintptr_t>(b_pool) & 15u))
    return set_error(QQQ_ERR_SHAPE, "probe_mfma_i8: 1 <= iters <= 2^24, 1 <= workgroups <= 65536, pools 16-byte aligned");
  hipLaunchKernelGGL(probe_mfma_i8_kernel, dim3((unsigned)workgroups), dim3(512), 0, (hipStream_t)stream, iters,
                     (const v4i*)a_pool, (const v4i*)b_pool, sink);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "probe_mfma_i8 launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

}  // extern "C"
