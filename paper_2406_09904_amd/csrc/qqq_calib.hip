// Offline (calibration-time) stage of QQQ on one layer: adaptive smoothing (Sec. 3.1, Eq. 1-2) and
// Hessian-based quantisation compensation (Sec. 3.2, Eq. 3-4).  Entry points of include/qqq_calib.h.
//
// Everything that decides an integer code is done in a fixed precision and operation order (stated at
// each kernel) so that the result can be checked bit for bit; floating-point contraction is off in
// this file for that reason.
#include "qqq_calib.h"
#include "qqq_internal.h"

#pragma clang fp contract(off)

namespace qqq {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

static bool aligned16c(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static size_t align256c(size_t v) { return (v + 255) & ~(size_t)255; }

static int check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "%s launch: %s", what, hipGetErrorString(e));
  return QQQ_OK;
}

// ------------------------------------------------------------------ small helpers

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) p[i] = v;
}

static int fill_u32(void* p, size_t n, uint32_t v, hipStream_t st) {
  const unsigned blocks = (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, st, (uint32_t*)p, n, v);
  return check_launch("fill");
}

// ------------------------------------------------------------------ Sec. 3.1: channel maxima

// absmax[t] = max_m |X[m,t]| on the fp16 bit patterns (magnitude order = integer order with the
// sign cleared); each thread owns 8 consecutive channels (one 128-bit load per row), blocks split
// the rows and meet through atomicMax on the (non-negative) bit patterns.  absmax holds fp16 bit
// patterns as uint32 until absmax_finish_kernel widens them to fp32 and takes the overall maximum.
__global__ __launch_bounds__(256) void channel_absmax_kernel(const uint4* x, int64_t M, int64_t kvec,
                                                             int64_t rows_per_block, uint32_t* absmax_bits) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= kvec) return;
  const int64_t m0 = (int64_t)blockIdx.y * rows_per_block;
  int64_t m1 = m0 + rows_per_block;
  if (m1 > M) m1 = M;
  uint32_t mx[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int64_t m = m0; m < m1; ++m) {
    const uint4 q = x[m * kvec + v];
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mx[2 * i] = max(mx[2 * i], w[i] & 0x7FFFu);
      mx[2 * i + 1] = max(mx[2 * i + 1], (w[i] >> 16) & 0x7FFFu);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) atomicMax(&absmax_bits[v * 8 + i], mx[i]);
}

// in place: fp16 bit patterns -> fp32 values; top[0] = the largest (one workgroup)
__global__ __launch_bounds__(1024) void absmax_finish_kernel(uint32_t* absmax, int64_t K, float* top) {
  __shared__ uint32_t smax;
  if (threadIdx.x == 0) smax = 0;
  __syncthreads();
  uint32_t mx = 0;
  for (int64_t t = threadIdx.x; t < K; t += 1024) {
    const uint32_t b = absmax[t];
    mx = max(mx, b);
    reinterpret_cast<float*>(absmax)[t] = half_bits_to_float(b);
  }
  atomicMax(&smax, mx);
  __syncthreads();
  if (threadIdx.x == 0 && top) top[0] = half_bits_to_float(smax);
}

// sigma_g = fp32(max|X| * g / G) with the product and the quotient in fp64, g = 1..G
__global__ void sigma_grid_kernel(const float* top, int G, float* sigmas) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g < G) sigmas[g] = (float)((double)top[0] * (double)(g + 1) / (double)G);
}

// s_t = absmax_t / sigma (one fp32 division) where absmax_t > sigma, else 1
__global__ __launch_bounds__(256) void smoothing_vector_kernel(const float* absmax, const float* sigmas,
                                                               const int32_t* index, int64_t K, float* s) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= K) return;
  const float sigma = sigmas[index ? index[0] : 0];
  const float a = absmax[t];
  s[t] = a > sigma ? a / sigma : 1.0f;
}

// out = fp16_rne(fp32(in) / s) (DIVIDE) or fp16_rne(fp32(in) * s): one fp32 operation, one rounding
template <bool DIVIDE>
__global__ __launch_bounds__(256) void smooth_apply_kernel(const uint4* in, const float* s, int64_t rows,
                                                           int64_t kvec, uint4* out) {
  const int64_t total = rows * kvec;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
    const int64_t v = i % kvec;
    const uint4 q = in[i];
    const float4 s0 = *reinterpret_cast<const float4*>(s + v * 8);
    const float4 s1 = *reinterpret_cast<const float4*>(s + v * 8 + 4);
    const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float a = half_bits_to_float(w[j] & 0xFFFFu), b = half_bits_to_float(w[j] >> 16);
      float ra = DIVIDE ? a / sv[2 * j] : a * sv[2 * j];
      float rb = DIVIDE ? b / sv[2 * j + 1] : b * sv[2 * j + 1];
      // the fp32 result is rounded before the conversion sees it: left alone, the compiler turns
      // multiply + convert into one mixed-precision instruction that rounds the exact product once
      asm volatile("" : "+v"(ra), "+v"(rb));
      o[j] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)ra) |
             ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)rb) << 16);
    }
    out[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// ------------------------------------------------------------------ X W^T in fp32 (reference product of Eq. 2)

// One wave per 32 x 32 output tile, v_mfma_f32_32x32x16_f16: lane l holds row (A) / column (B)
// l % 32 and the 8 consecutive k of half l / 32, straight from global memory (each lane walks its
// own row 16 bytes at a time, so every fetched cache line is used in full over four k-steps).
// Register v of the result is row 8*(v/4) + 4*(l/32) + v%4, column l % 32.  A calibration-time
// kernel: correctness and simplicity over speed.
__global__ __launch_bounds__(64) void fp16_gemm_nt_kernel(const _Float16* x, const _Float16* w, int M, int N,
                                                          int K, float* y) {
  const int lane = threadIdx.x, r32 = lane & 31, h = lane >> 5;
  const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int mr = min(m0 + r32, M - 1), nr = min(n0 + r32, N - 1);
  const v8h* xa = reinterpret_cast<const v8h*>(x + (int64_t)mr * K + 8 * h);
  const v8h* wb = reinterpret_cast<const v8h*>(w + (int64_t)nr * K + 8 * h);
  v16f acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  for (int k = 0; k < K; k += 16) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[k >> 3], wb[k >> 3], acc, 0, 0, 0);
  const int n = n0 + r32;
  if (n >= N) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + 8 * (v >> 2) + 4 * h + (v & 3);
    if (m < M) y[(int64_t)m * N + n] = acc[v];
  }
}

// ------------------------------------------------------------------ loss of Eq. 2 and the grid's minimum

// loss += sum ( fp64(acc) * fp64(s_a[m]) * fp64(s_w[n]) - fp64(y_ref) )^2, fp64 throughout
__global__ __launch_bounds__(256) void smooth_loss_kernel(const int32_t* acc, const float* s_a,
                                                          const uint16_t* s_w, const float* y_ref, int64_t M,
                                                          int64_t N, double* loss) {
  __shared__ double part[256];
  const int64_t total = M * N;
  const int64_t stride = (int64_t)gridDim.x * 256;
  double sum = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
    const int64_t m = i / N, n = i - m * N;
    const double d = (double)acc[i] * (double)s_a[m] * (double)half_bits_to_float(s_w[n]) - (double)y_ref[i];
    sum += d * d;
  }
  part[threadIdx.x] = sum;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) atomicAdd(loss, part[0]);
}

__global__ void argmin_kernel(const double* losses, int G, int32_t* best) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  int b = 0;
  for (int g = 1; g < G; ++g)
    if (losses[g] < losses[b]) b = g;  // first minimum
  best[0] = b;
}

// ------------------------------------------------------------------ Sec. 3.2: Hessian

// H[i,j] = 2 * sum_m X[m,i] X[m,j] in fp64.  64 x 64 tile per workgroup of 16 x 16 threads (4 x 4 each),
// 16 tokens at a time through LDS.
__global__ __launch_bounds__(256) void hessian_kernel(const _Float16* x, int64_t M, int64_t K, double* H) {
  __shared__ double a[16][65], b[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t i0 = (int64_t)blockIdx.y * 64, j0 = (int64_t)blockIdx.x * 64;
  double acc[4][4] = {};
  for (int64_t m0 = 0; m0 < M; m0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      const int mm = e >> 6, c = e & 63;
      const int64_t m = m0 + mm;
      const bool ok = m < M;
      a[mm][c] = (ok && i0 + c < K) ? (double)(float)x[m * K + i0 + c] : 0.0;
      b[mm][c] = (ok && j0 + c < K) ? (double)(float)x[m * K + j0 + c] : 0.0;
    }
    __syncthreads();
#pragma unroll 4
    for (int mm = 0; mm < 16; ++mm) {
      double av[4], bv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) av[r] = a[mm][ty * 4 + r], bv[r] = b[mm][tx * 4 + r];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] += av[r] * bv[c];
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int64_t i = i0 + ty * 4 + r, j = j0 + tx * 4 + c;
      if (i < K && j < K) H[i * K + j] = 2.0 * acc[r][c];
    }
}

// ------------------------------------------------------------------ Sec. 3.2: compensation

// working copy: Hw = H with dead channels (H_ii == 0) set to 1 on the diagonal; W64 = fp64(W) with
// dead channels zeroed; dsum accumulates the diagonal (after the dead-channel rule) for the damping
__global__ __launch_bounds__(256) void gptq_prepare_kernel(const double* H, const _Float16* w, int64_t N, int64_t K,
                                                           double* Hw, double* W64, double* dsum) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (int64_t e = tid; e < K * K; e += stride) {
    const int64_t i = e / K, j = e - i * K;
    double v = H[e];
    if (i == j && v == 0.0) v = 1.0;
    Hw[e] = v;
  }
  for (int64_t e = tid; e < N * K; e += stride) {
    const int64_t k = e % K;
    W64[e] = (H[k * K + k] == 0.0) ? 0.0 : (double)(float)w[e];
  }
  double part = 0.0;
  for (int64_t i = tid; i < K; i += stride) {
    const double d = H[i * K + i];
    part += (d == 0.0) ? 1.0 : d;
  }
  if (part != 0.0) atomicAdd(dsum, part);
}

__global__ __launch_bounds__(256) void gptq_damp_kernel(double* Hw, int64_t K, const double* dsum, double percdamp) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < K) Hw[i * K + i] += percdamp * (dsum[0] / (double)K);
}

// In-place inverse of the damped Hessian (symmetric positive definite: no pivoting) by K
// Gauss-Jordan sweeps.  Sweep p, first kernel: row[j] = A[p,j] / d (row[p] = 1 / d), col[r] = A[r,p]
// (col[p] = 0), d = A[p,p]; second kernel: A[r,j] = (j == p ? 0 : A[r,j]) - col[r] * row[j] for r != p,
// A[p,j] = row[j].
__global__ __launch_bounds__(256) void gj_pivot_kernel(const double* A, int64_t K, int64_t p, double* row, double* col) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= K) return;
  const double d = A[p * K + p];
  row[j] = (j == p) ? 1.0 / d : A[p * K + j] / d;
  col[j] = (j == p) ? 0.0 : A[j * K + p];
}

__global__ __launch_bounds__(256) void gj_update_kernel(double* A, int64_t K, int64_t p, const double* row,
                                                        const double* col) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t r = blockIdx.y;
  if (j >= K) return;
  if (r == p) {
    A[r * K + j] = row[j];
  } else {
    const double base = (j == p) ? 0.0 : A[r * K + j];
    A[r * K + j] = base - col[r] * row[j];
  }
}

// Channel i of Eq. 4 for every output channel n: code, error, and the move of the channels still in F.
//   q = clamp(rne(fp32(w / s)), -7, 7), s == 0 gives 0;  err = (w - q * s) / Hinv[i,i];
//   W[n, j] -= err * Hinv[i, j] for j > i  (product rounded, then the difference rounded: no FMA)
// grid: x = chunks of 256 trailing channels, y = output channel n
__global__ __launch_bounds__(256) void gptq_column_kernel(double* W64, const double* Hinv, const uint16_t* s_w,
                                                          int64_t N, int64_t K, int64_t i, uint32_t* w_nat) {
  const int64_t n = blockIdx.y;
  const double w = W64[n * K + i];
  const double s = (double)half_bits_to_float(s_w[n]);
  double q = 0.0;
  if (s != 0.0) {
    q = (double)__builtin_rintf((float)(w / s));
    q = q > 7.0 ? 7.0 : (q < -7.0 ? -7.0 : q);
  }
  const double err = (w - q * s) / Hinv[i * K + i];
  const int64_t j = i + 1 + (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j < K) W64[n * K + j] = W64[n * K + j] - err * Hinv[i * K + j];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t* word = &w_nat[n * (K / 8) + i / 8];
    const int sh = 4 * (int)(i % 8);
    *word = (*word & ~(0xFu << sh)) | (((uint32_t)(int)q & 0xFu) << sh);
  }
}

// channel i leaves F: Hinv[a,b] -= Hinv[a,i] * Hinv[i,b] / Hinv[i,i] for a, b > i (row i and column i
// themselves are not written, so every workgroup reads the same old values)
__global__ __launch_bounds__(256) void gptq_eliminate_kernel(double* Hinv, int64_t K, int64_t i) {
  const int64_t b = i + 1 + (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t a = i + 1 + blockIdx.y;
  if (b >= K || a >= K) return;
  const double d = Hinv[i * K + i];
  const double t = (Hinv[a * K + i] * Hinv[i * K + b]) / d;
  Hinv[a * K + b] = Hinv[a * K + b] - t;
}

// Per-group weights (Sec. 3.3.2: groups of 128 input channels): when the sweep reaches a group's first
// channel, the group's scale comes from the weights as they stand then, s = fp16(fp32(max |w|) / 7).
// One thread per output channel.
__global__ __launch_bounds__(256) void gptq_group_scale_kernel(const double* W64, int64_t N, int64_t K, int64_t i0,
                                                               int group, uint16_t* s_row) {
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  double amax = 0.0;
  for (int k = 0; k < group; ++k) amax = fmax(amax, fabs(W64[n * K + i0 + k]));
  s_row[n] = __builtin_bit_cast(uint16_t, (_Float16)((float)amax / 7.0f));
}

// After the sweep, what the front-end derives from codes and group scales (Sec. 3.3.2, Fig. 5 offline):
// s_Wc[n] = fp16(max_k |code * s_Wg| / 127) with the product in fp32, s*_Wg = fp16(s_Wg / s_Wc) capped at
// 18.203125 (0 where s_Wc is 0), integer form clamp(rne(s*_Wg), 1, 18).  One thread per output channel.
__global__ __launch_bounds__(256) void gptq_group_finish_kernel(const uint32_t* w_nat, const uint16_t* s_wg, int64_t N,
                                                                int64_t K, int group, uint16_t* s_wc, uint16_t* s_star,
                                                                int8_t* s_int) {
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  const int64_t G = K / group;
  float dmax = 0.0f;
  for (int64_t g = 0; g < G; ++g) {
    int cmax = 0;
    for (int j = 0; j < group / 8; ++j) {
      const uint32_t word = w_nat[n * (K / 8) + g * (group / 8) + j];
      for (int q = 0; q < 8; ++q) {
        const int code = ((int)(word << (28 - 4 * q))) >> 28;  // sign-extended nibble
        cmax = max(cmax, code < 0 ? -code : code);
      }
    }
    dmax = fmaxf(dmax, (float)cmax * half_bits_to_float(s_wg[g * N + n]));
  }
  const uint16_t wcb = __builtin_bit_cast(uint16_t, (_Float16)(dmax / 127.0f));
  s_wc[n] = wcb;
  const float wc = half_bits_to_float(wcb);
  for (int64_t g = 0; g < G; ++g) {
    uint16_t star = 0;
    if (wc != 0.0f) {
      const _Float16 h = (_Float16)(half_bits_to_float(s_wg[g * N + n]) / wc);
      star = __builtin_bit_cast(uint16_t, (float)h > 18.203125f ? (_Float16)18.203125f : h);
    }
    s_star[g * N + n] = star;
    if (s_int) s_int[g * N + n] = (int8_t)fminf(fmaxf(__builtin_rintf(half_bits_to_float(star)), 1.0f), 18.0f);
  }
}

static bool calib_shape_ok(int64_t M, int64_t N, int64_t K) {
  return M >= 1 && M <= 0x7FFFFFFF && N >= 16 && N % 16 == 0 && N <= 0x7FFFFFF0 && K >= 128 && K % 128 == 0 &&
         K <= 131072;
}

// workspace layout of qqq_adaptive_smoothing
struct SmoothWs {
  size_t absmax, top, y_ref, xs, ws, s, a_q, s_a, w_nat, s_w, packed, acc, y, gemm, total;
};
static SmoothWs smooth_layout(int64_t M, int64_t N, int64_t K) {
  SmoothWs L;
  size_t at = 0;
  auto take = [&](size_t bytes) { const size_t o = at; at += align256c(bytes); return o; };
  L.absmax = take((size_t)K * 4);
  L.top = take(256);
  L.y_ref = take((size_t)M * N * 4);
  L.xs = take((size_t)M * K * 2);
  L.ws = take((size_t)N * K * 2);
  L.s = take((size_t)K * 4);
  L.a_q = take((size_t)M * K);
  L.s_a = take((size_t)M * 4);
  L.w_nat = take((size_t)N * K / 2);
  L.s_w = take((size_t)N * 2);
  L.packed = take((size_t)N * K / 2);
  L.acc = take((size_t)M * N * 4);
  L.y = take((size_t)M * N * 2);
  L.gemm = take(qqq_gemm_workspace_bytes(M, N, K));
  L.total = at;
  return L;
}

static int launch_absmax(const void* x, int64_t M, int64_t K, float* absmax, float* top, hipStream_t st) {
  int rc = fill_u32(absmax, (size_t)K, 0u, st);
  if (rc != QQQ_OK) return rc;
  const int64_t kvec = K / 8;
  int64_t row_blocks = (M + 63) / 64;
  if (row_blocks > 1024) row_blocks = 1024;
  const int64_t rows_per_block = (M + row_blocks - 1) / row_blocks;
  hipLaunchKernelGGL(channel_absmax_kernel, dim3((unsigned)((kvec + 255) / 256), (unsigned)row_blocks), dim3(256), 0,
                     st, (const uint4*)x, M, kvec, rows_per_block, (uint32_t*)absmax);
  rc = check_launch("channel_absmax");
  if (rc != QQQ_OK) return rc;
  hipLaunchKernelGGL(absmax_finish_kernel, dim3(1), dim3(1024), 0, st, (uint32_t*)absmax, K, top);
  return check_launch("channel_absmax (finish)");
}

static int launch_smooth(const void* x, const void* w, const float* absmax, const float* sigmas, const int32_t* index,
                         int64_t M, int64_t N, int64_t K, void* xs, void* ws, float* s, hipStream_t st) {
  hipLaunchKernelGGL(smoothing_vector_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, absmax, sigmas, index,
                     K, s);
  int rc = check_launch("smoothing_vector");
  if (rc != QQQ_OK) return rc;
  const int64_t kvec = K / 8;
  auto blocks = [](int64_t total) { return (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096); };
  hipLaunchKernelGGL((smooth_apply_kernel<true>), dim3(blocks(M * kvec)), dim3(256), 0, st, (const uint4*)x, s, M, kvec,
                     (uint4*)xs);
  rc = check_launch("smooth_apply (activations)");
  if (rc != QQQ_OK) return rc;
  hipLaunchKernelGGL((smooth_apply_kernel<false>), dim3(blocks(N * kvec)), dim3(256), 0, st, (const uint4*)w, s, N, kvec,
                     (uint4*)ws);
  return check_launch("smooth_apply (weights)");
}

static int launch_fp16_gemm(const void* x, const void* w, int64_t M, int64_t N, int64_t K, float* y, hipStream_t st) {
  hipLaunchKernelGGL(fp16_gemm_nt_kernel, dim3((unsigned)((N + 31) / 32), (unsigned)((M + 31) / 32)), dim3(64), 0, st,
                     (const _Float16*)x, (const _Float16*)w, (int)M, (int)N, (int)K, y);
  return check_launch("fp16_gemm_nt");
}

}  // namespace qqq

using namespace qqq;

extern "C" {

int qqq_channel_absmax(const void* x_fp16, int64_t M, int64_t K, float* absmax, void* stream) {
  if (M < 1 || M > 0x7FFFFFFF || K < 8 || K % 8 != 0 || K > (1 << 24))
    return set_error(QQQ_ERR_SHAPE, "channel_absmax: unsupported M=%lld K=%lld (need K%%8==0)", (long long)M, (long long)K);
  if (!x_fp16 || !absmax) return set_error(QQQ_ERR_NULL, "channel_absmax: null pointer argument");
  if (!aligned16c(x_fp16) || (reinterpret_cast<uintptr_t>(absmax) & 3u))
    return set_error(QQQ_ERR_SHAPE, "channel_absmax: x must be 16-byte, absmax 4-byte aligned");
  return launch_absmax(x_fp16, M, K, absmax, nullptr, (hipStream_t)stream);
}

int qqq_smooth_apply(const void* x_fp16, const void* w_fp16, const float* absmax, const float* sigma, int64_t M,
                     int64_t N, int64_t K, void* xs_fp16, void* ws_fp16, float* s, void* stream) {
  if (M < 1 || N < 1 || M > 0x7FFFFFFF || N > 0x7FFFFFFF || K < 8 || K % 8 != 0 || K > (1 << 24))
    return set_error(QQQ_ERR_SHAPE, "smooth_apply: unsupported M=%lld N=%lld K=%lld (need K%%8==0)", (long long)M,
                     (long long)N, (long long)K);
  if (!x_fp16 || !w_fp16 || !absmax || !sigma || !xs_fp16 || !ws_fp16 || !s)
    return set_error(QQQ_ERR_NULL, "smooth_apply: null pointer argument");
  if (!aligned16c(x_fp16) || !aligned16c(w_fp16) || !aligned16c(xs_fp16) || !aligned16c(ws_fp16) || !aligned16c(s) ||
      (reinterpret_cast<uintptr_t>(absmax) & 3u) || (reinterpret_cast<uintptr_t>(sigma) & 3u))
    return set_error(QQQ_ERR_SHAPE, "smooth_apply: matrices and s must be 16-byte, absmax and sigma 4-byte aligned");
  return launch_smooth(x_fp16, w_fp16, absmax, sigma, nullptr, M, N, K, xs_fp16, ws_fp16, s, (hipStream_t)stream);
}

int qqq_fp16_gemm_nt(const void* x_fp16, const void* w_fp16, int64_t M, int64_t N, int64_t K, float* y, void* stream) {
  if (M < 1 || N < 1 || M > 0x7FFFFFF0 || N > 0x7FFFFFF0 || K < 16 || K % 16 != 0 || K > (1 << 24) ||
      (M + 31) / 32 > 65535)
    return set_error(QQQ_ERR_SHAPE, "fp16_gemm_nt: unsupported M=%lld N=%lld K=%lld (need K%%16==0, M <= 2097120)",
                     (long long)M, (long long)N, (long long)K);
  if (!x_fp16 || !w_fp16 || !y) return set_error(QQQ_ERR_NULL, "fp16_gemm_nt: null pointer argument");
  if (!aligned16c(x_fp16) || !aligned16c(w_fp16) || (reinterpret_cast<uintptr_t>(y) & 3u))
    return set_error(QQQ_ERR_SHAPE, "fp16_gemm_nt: x and w must be 16-byte, y 4-byte aligned");
  return launch_fp16_gemm(x_fp16, w_fp16, M, N, K, y, (hipStream_t)stream);
}

size_t qqq_smoothing_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (!calib_shape_ok(M, N, K)) return 0;
  return smooth_layout(M, N, K).total;
}

int qqq_adaptive_smoothing(const void* x_fp16, const void* w_fp16, int64_t M, int64_t N, int64_t K, int grid_points,
                           void* xs_fp16, void* ws_fp16, float* s, float* sigmas, double* losses, int32_t* best,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (!calib_shape_ok(M, N, K) || (M + 31) / 32 > 65535)
    return set_error(QQQ_ERR_SHAPE, "adaptive_smoothing: unsupported M=%lld N=%lld K=%lld (need N%%16==0, K%%128==0, "
                     "128<=K<=131072, M <= 2097120)", (long long)M, (long long)N, (long long)K);
  if (grid_points < 1 || grid_points > 256)
    return set_error(QQQ_ERR_SHAPE, "adaptive_smoothing: grid_points must be in 1..256, got %d", grid_points);
  if (!x_fp16 || !w_fp16 || !xs_fp16 || !ws_fp16 || !s || !sigmas || !losses || !best || !workspace)
    return set_error(QQQ_ERR_NULL, "adaptive_smoothing: null pointer argument");
  if (!aligned16c(x_fp16) || !aligned16c(w_fp16) || !aligned16c(xs_fp16) || !aligned16c(ws_fp16) || !aligned16c(s) ||
      !aligned16c(workspace) || (reinterpret_cast<uintptr_t>(sigmas) & 3u) || (reinterpret_cast<uintptr_t>(losses) & 7u) ||
      (reinterpret_cast<uintptr_t>(best) & 3u))
    return set_error(QQQ_ERR_SHAPE, "adaptive_smoothing: matrices, s and workspace must be 16-byte aligned, sigmas and "
                     "best 4-byte, losses 8-byte");
  const SmoothWs L = smooth_layout(M, N, K);
  if (workspace_bytes < L.total)
    return set_error(QQQ_ERR_WORKSPACE, "adaptive_smoothing: workspace %zu bytes < %zu needed", workspace_bytes, L.total);
  char* base = (char*)workspace;
  hipStream_t st = (hipStream_t)stream;
  float* absmax = (float*)(base + L.absmax);
  float* top = (float*)(base + L.top);
  float* y_ref = (float*)(base + L.y_ref);
  int8_t* a_q = (int8_t*)(base + L.a_q);
  float* s_a = (float*)(base + L.s_a);
  uint32_t* w_nat = (uint32_t*)(base + L.w_nat);
  void* s_w = base + L.s_w;
  void* packed = base + L.packed;
  int32_t* acc = (int32_t*)(base + L.acc);
  void* y = base + L.y;
  void* gemm_ws = base + L.gemm;
  const size_t gemm_ws_bytes = qqq_gemm_workspace_bytes(M, N, K);

  int rc = launch_absmax(x_fp16, M, K, absmax, top, st);
  if (rc != QQQ_OK) return rc;
  hipLaunchKernelGGL(sigma_grid_kernel, dim3(1), dim3(256), 0, st, top, grid_points, sigmas);
  if ((rc = check_launch("sigma_grid")) != QQQ_OK) return rc;
  if ((rc = launch_fp16_gemm(x_fp16, w_fp16, M, N, K, y_ref, st)) != QQQ_OK) return rc;
  if ((rc = fill_u32(losses, (size_t)grid_points * 2, 0u, st)) != QQQ_OK) return rc;
  if (gemm_ws_bytes && (rc = fill_u32(gemm_ws, (gemm_ws_bytes + 3) / 4, 0u, st)) != QQQ_OK) return rc;
  for (int g = 0; g < grid_points; ++g) {
    // the candidate's smoothed layer, quantised as the hot path quantises it, and its loss
    if ((rc = launch_smooth(x_fp16, w_fp16, absmax, sigmas + g, nullptr, M, N, K, base + L.xs, base + L.ws,
                            (float*)(base + L.s), st)) != QQQ_OK) return rc;
    if ((rc = qqq_quant_act(base + L.xs, M, K, K, a_q, s_a, stream)) != QQQ_OK) return rc;
    if ((rc = qqq_quantize_w4_perchannel(base + L.ws, N, K, K, w_nat, s_w, stream)) != QQQ_OK) return rc;
    if ((rc = qqq_pack_w4(w_nat, N, K, packed, stream)) != QQQ_OK) return rc;
    if ((rc = qqq_gemm_w4a8_perchannel(a_q, s_a, packed, s_w, y, acc, M, N, K, gemm_ws, gemm_ws_bytes, stream)) != QQQ_OK)
      return rc;
    const int64_t total = M * N;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(smooth_loss_kernel, dim3(blocks), dim3(256), 0, st, acc, s_a, (const uint16_t*)s_w, y_ref, M, N,
                       losses + g);
    if ((rc = check_launch("smooth_loss")) != QQQ_OK) return rc;
  }
  hipLaunchKernelGGL(argmin_kernel, dim3(1), dim3(64), 0, st, losses, grid_points, best);
  if ((rc = check_launch("argmin")) != QQQ_OK) return rc;
  return launch_smooth(x_fp16, w_fp16, absmax, sigmas, best, M, N, K, xs_fp16, ws_fp16, s, st);
}

int qqq_hessian(const void* x_fp16, int64_t M, int64_t K, double* H, void* stream) {
  if (M < 1 || M > 0x7FFFFFFF || K < 1 || K > 16384)
    return set_error(QQQ_ERR_SHAPE, "hessian: unsupported M=%lld K=%lld (need 1 <= K <= 16384)", (long long)M, (long long)K);
  if (!x_fp16 || !H) return set_error(QQQ_ERR_NULL, "hessian: null pointer argument");
  if ((reinterpret_cast<uintptr_t>(x_fp16) & 1u) || (reinterpret_cast<uintptr_t>(H) & 7u))
    return set_error(QQQ_ERR_SHAPE, "hessian: x must be 2-byte, H 8-byte aligned");
  const unsigned t = (unsigned)((K + 63) / 64);
  hipLaunchKernelGGL(hessian_kernel, dim3(t, t), dim3(256), 0, (hipStream_t)stream, (const _Float16*)x_fp16, M, K, H);
  return check_launch("hessian");
}

size_t qqq_gptq_workspace_bytes(int64_t N, int64_t K) {
  if (N < 1 || N > 65535 || K < 8 || K % 8 != 0 || K > 16384) return 0;
  return align256c((size_t)K * K * 8) + align256c((size_t)N * K * 8) + 2 * align256c((size_t)K * 8) + 256;
}

// what both sweeps share: argument checks, the working copies, damping and the inverse Hessian
struct GptqWork { double *Hinv, *W64; };
static int gptq_begin(const char* who, const void* w_fp16, const double* H, int64_t N, int64_t K, double percdamp,
                      const uint32_t* w_nat, void* workspace, size_t workspace_bytes, hipStream_t st, GptqWork* out) {
  if (N < 1 || N > 65535 || K < 8 || K % 8 != 0 || K > 16384 || !(percdamp >= 0.0) || percdamp > 1e6)
    return set_error(QQQ_ERR_SHAPE, "%s: unsupported N=%lld K=%lld percdamp=%g (need N <= 65535, K%%8==0, K <= 16384, "
                     "percdamp >= 0)", who, (long long)N, (long long)K, percdamp);
  if (!w_fp16 || !H || !w_nat || !workspace) return set_error(QQQ_ERR_NULL, "%s: null pointer argument", who);
  if (!aligned16c(w_fp16) || !aligned16c(workspace) || (reinterpret_cast<uintptr_t>(H) & 7u) ||
      (reinterpret_cast<uintptr_t>(w_nat) & 3u))
    return set_error(QQQ_ERR_SHAPE, "%s: w_fp16 and workspace must be 16-byte, H 8-byte, w_nat 4-byte aligned", who);
  const size_t need = qqq_gptq_workspace_bytes(N, K);
  if (workspace_bytes < need)
    return set_error(QQQ_ERR_WORKSPACE, "%s: workspace %zu bytes < %zu needed", who, workspace_bytes, need);
  char* base = (char*)workspace;
  double* Hinv = (double*)base;
  double* W64 = (double*)(base + align256c((size_t)K * K * 8));
  double* row = (double*)((char*)W64 + align256c((size_t)N * K * 8));
  double* col = (double*)((char*)row + align256c((size_t)K * 8));
  double* dsum = (double*)((char*)col + align256c((size_t)K * 8));
  int rc;
  if ((rc = fill_u32(dsum, 2, 0u, st)) != QQQ_OK) return rc;
  hipLaunchKernelGGL(gptq_prepare_kernel, dim3(2048), dim3(256), 0, st, H, (const _Float16*)w_fp16, N, K, Hinv, W64, dsum);
  if ((rc = check_launch("gptq_prepare")) != QQQ_OK) return rc;
  const unsigned kb = (unsigned)((K + 255) / 256);
  hipLaunchKernelGGL(gptq_damp_kernel, dim3(kb), dim3(256), 0, st, Hinv, K, dsum, percdamp);
  if ((rc = check_launch("gptq_damp")) != QQQ_OK) return rc;
  for (int64_t p = 0; p < K; ++p) {  // H^-1 in place
    hipLaunchKernelGGL(gj_pivot_kernel, dim3(kb), dim3(256), 0, st, Hinv, K, p, row, col);
    hipLaunchKernelGGL(gj_update_kernel, dim3(kb, (unsigned)K), dim3(256), 0, st, Hinv, K, p, row, col);
  }
  if ((rc = check_launch("gptq inverse")) != QQQ_OK) return rc;
  out->Hinv = Hinv;
  out->W64 = W64;
  return QQQ_OK;
}

// channel i of Eq. 4 with the scales at `scales` [N], then channel i leaves F
static void gptq_step(const GptqWork& wk, const uint16_t* scales, int64_t N, int64_t K, int64_t i, uint32_t* w_nat,
                      hipStream_t st) {
  const int64_t trail = K - i - 1;
  const unsigned tb = (unsigned)(trail > 0 ? (trail + 255) / 256 : 1);
  hipLaunchKernelGGL(gptq_column_kernel, dim3(tb, (unsigned)N), dim3(256), 0, st, wk.W64, wk.Hinv, scales, N, K, i,
                     w_nat);
  if (trail > 0)
    hipLaunchKernelGGL(gptq_eliminate_kernel, dim3(tb, (unsigned)trail), dim3(256), 0, st, wk.Hinv, K, i);
}

int qqq_gptq_quantize_w4_perchannel(const void* w_fp16, const double* H, int64_t N, int64_t K, double percdamp,
                                    uint32_t* w_nat, void* s_w_fp16, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  if (!s_w_fp16) return set_error(QQQ_ERR_NULL, "gptq: null pointer argument");
  if (reinterpret_cast<uintptr_t>(s_w_fp16) & 1u) return set_error(QQQ_ERR_SHAPE, "gptq: s_w must be 2-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  GptqWork wk;
  int rc = gptq_begin("gptq", w_fp16, H, N, K, percdamp, w_nat, workspace, workspace_bytes, st, &wk);
  if (rc != QQQ_OK) return rc;
  // scales from the original weights (and round-to-nearest codes, overwritten channel by channel below)
  rc = launch_quant_weight(w_fp16, N, K, K, false, w_nat, (uint16_t*)s_w_fp16, nullptr, nullptr, nullptr, st);
  if (rc != QQQ_OK) return rc;
  for (int64_t i = 0; i < K; ++i) gptq_step(wk, (const uint16_t*)s_w_fp16, N, K, i, w_nat, st);  // Eq. 4, channel by channel
  return check_launch("gptq column");
}

int qqq_gptq_quantize_w4_pergroup(const void* w_fp16, const double* H, int64_t N, int64_t K, int group, double percdamp,
                                  uint32_t* w_nat, void* s_wg_fp16, void* s_star_fp16, int8_t* s_int, void* s_wc_fp16,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (group != QQQ_GROUP) return set_error(QQQ_ERR_SHAPE, "gptq_pergroup: group must be 128, got %d", group);
  if (K % QQQ_GROUP != 0) return set_error(QQQ_ERR_SHAPE, "gptq_pergroup: K=%lld must be a multiple of 128", (long long)K);
  if (!s_wg_fp16 || !s_star_fp16 || !s_wc_fp16) return set_error(QQQ_ERR_NULL, "gptq_pergroup: null pointer argument");
  if ((reinterpret_cast<uintptr_t>(s_wg_fp16) | reinterpret_cast<uintptr_t>(s_star_fp16) |
       reinterpret_cast<uintptr_t>(s_wc_fp16)) & 1u)
    return set_error(QQQ_ERR_SHAPE, "gptq_pergroup: scale tables must be 2-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  GptqWork wk;
  int rc = gptq_begin("gptq_pergroup", w_fp16, H, N, K, percdamp, w_nat, workspace, workspace_bytes, st, &wk);
  if (rc != QQQ_OK) return rc;
  if ((rc = fill_u32(w_nat, (size_t)N * (size_t)(K / 8), 0u, st)) != QQQ_OK) return rc;
  uint16_t* s_wg = (uint16_t*)s_wg_fp16;
  const unsigned nb = (unsigned)((N + 255) / 256);
  for (int64_t i = 0; i < K; ++i) {
    uint16_t* s_row = s_wg + (i / QQQ_GROUP) * N;
    if (i % QQQ_GROUP == 0)  // the sweep enters a group: its scale from the weights as they stand now
      hipLaunchKernelGGL(gptq_group_scale_kernel, dim3(nb), dim3(256), 0, st, wk.W64, N, K, i, QQQ_GROUP, s_row);
    gptq_step(wk, s_row, N, K, i, w_nat, st);
  }
  if ((rc = check_launch("gptq_pergroup column")) != QQQ_OK) return rc;
  hipLaunchKernelGGL(gptq_group_finish_kernel, dim3(nb), dim3(256), 0, st, w_nat, s_wg, N, K, QQQ_GROUP,
                     (uint16_t*)s_wc_fp16, (uint16_t*)s_star_fp16, s_int);
  return check_launch("gptq_pergroup finish");
}

}  // extern "C"
