/*
 * CPU oracle for the QQQ W4A8 GEMM hot path (arXiv 2406.09904).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, obviously
 * correct statement of what the path computes, written from the paper's definitions:
 * no blocking, no fusion, no reordering, int64 accumulation.  It shares no code,
 * header, table or helper with the HIP library and never includes or links it.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What the path computes (paper sections in brackets):
 *   quant_act   per-token symmetric int8 quantisation of fp16 activations
 *               [Sec. 4.1 "Algorithm"; s_A in the caption of Fig. 3]
 *   W8          per-channel: the int4 code widened to int8            [Sec. 3.3.1]
 *               per-group:   int4 code times the fused per-group scale, as int8
 *                            (FusedDequantQuant followed by the FP16->INT8 step)
 *                            [Sec. 3.3.2, Fig. 4-6]; here the fused scale is an
 *                            integer and the product saturates to [-128,127];
 *                            the "_f16" functions take the paper's real-valued fp16
 *                            fused scale s*_Wg = s_Wg / s_Wc instead and follow the
 *                            steps of Sec. 3.3.2 (FastINT4toFP16, one fp16 FMA that
 *                            multiplies by the scale and adds 128 + 1024, low byte,
 *                            XOR 0x80), with no saturation, as the paper describes
 *   acc         INT8 GEMM with an integer accumulator wide enough not to overflow
 *               [Sec. 3.3, second consideration]
 *   Y           Dequant: acc * s_A[m] * s_W[n] (per-group: s_Wc[n]) -> fp16
 *               [Sec. 3.3.1 last sentences, Sec. 3.3.2 last sentence]
 *   quantize_w4 offline front-end: symmetric round-to-nearest int4 codes from fp16 weights with
 *               the per-channel scale s_W [Sec. 3.3.1] or the per-group scales s_Wg, s_Wc and
 *               the fused s*_Wg = s_Wg / s_Wc [Sec. 3.3.2, Fig. 4-5]; its readings are listed
 *               above its functions at the end of this file
 *
 * Readings taken where the paper is silent (each is listed in the design notes of
 * the repository): divisor 127, fp32 correctly rounded division, round half to even,
 * clamp to [-127,127]; an all-zero token has scale 0 and codes 0; s_A is fp32, s_W is
 * stored as fp16; int4 codes are 4-bit two's complement, eight per 32-bit word, nibble
 * i of word j holding W[n, 8j+i]; the int32 result is the true sum (not the x16 one
 * that the FastINT4toINT8 trick produces inside a kernel).
 *
 * Pins (tests, CPU only): pure-Python brute force on tiny shapes, numpy's float16
 * conversions, closed forms for constant / one-hot / extreme inputs, the x16 identity
 * of Sec. 3.3.1, exhaustive code x scale table for the per-group W8; for the front-end: weights
 * on an exact grid, exact rational arithmetic for every code of small matrices, the round-to-
 * nearest error bound, the step^2/12 noise law, the no-wrap property through the pinned
 * code x scale conversion, an end-to-end layer against float64.
 *
 * Return codes: 0 ok, 1 null pointer, 2 bad shape, 5 accumulator does not fit int32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_NULL 1
#define ORC_SHAPE 2
#define ORC_OVERFLOW 5

/* ---------- fp16 <-> fp32, written out bit by bit (IEEE 754 binary16) ---------- */

float qqq_oracle_half_to_float(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int e = (h >> 10) & 0x1F;
  const int f = h & 0x3FF;
  double v;
  if (e == 0) {
    v = ldexp((double)f, -24); /* subnormal: f * 2^-24 */
  } else if (e == 31) {
    v = f ? (double)NAN : (double)INFINITY;
  } else {
    v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */
  }
  return (float)(sign ? -v : v);
}

/* round-to-nearest-even of a finite or infinite float to binary16 bits;
 * overflow gives infinity, small values become subnormals (never flushed). */
uint16_t qqq_oracle_float_to_half(float x) {
  const uint16_t sign = signbit(x) ? 0x8000u : 0u;
  if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
  double a = fabs((double)x);
  if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
  if (a == 0.0) return sign;
  int ex;
  (void)frexp(a, &ex); /* a = m * 2^ex, m in [0.5,1) => a in [2^(ex-1), 2^ex) */
  int e = ex - 1;      /* a in [2^e, 2^(e+1)) */
  if (e < -14) e = -14; /* subnormal range shares the spacing of the lowest binade */
  /* spacing of representable values in this binade is 2^(e-10) */
  double q = ldexp(a, 10 - e); /* exact: scaling by a power of two */
  double r = nearbyint(q);     /* default rounding mode = ties to even */
  /* r in [0, 2048]; r == 2048 means it rounded up into the next binade */
  if (r >= 2048.0) {
    r = 1024.0;
    e += 1;
  }
  if (e > 15) return (uint16_t)(sign | 0x7C00u);
  uint32_t ri = (uint32_t)r;
  uint16_t bits;
  if (ri < 1024u) {
    bits = (uint16_t)ri; /* subnormal (e == -14, no hidden bit) */
  } else {
    bits = (uint16_t)(((uint32_t)(e + 15) << 10) | (ri - 1024u));
  }
  return (uint16_t)(sign | bits);
}

void qqq_oracle_half_to_float_array(const uint16_t* h, int64_t n, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = qqq_oracle_half_to_float(h[i]);
}

void qqq_oracle_float_to_half_array(const float* x, int64_t n, uint16_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = qqq_oracle_float_to_half(x[i]);
}

/* ---------- int4 codes in the natural interchange format ---------- */

/* code of W[n,k]: nibble (k mod 8) of word k/8 in row n, 4-bit two's complement */
static int code_at(const uint32_t* w_nat, int64_t K, int64_t n, int64_t k) {
  const uint32_t word = w_nat[n * (K / 8) + k / 8];
  const int nib = (int)((word >> (4 * (k % 8))) & 0xFu);
  return nib >= 8 ? nib - 16 : nib;
}

/* ---------- Sec. 4.1: per-token symmetric int8 quantisation of activations ---------- */

int qqq_oracle_quant_act(const uint16_t* a_fp16, int64_t M, int64_t K, int64_t lda,
                         int8_t* a_q, float* s_a) {
  if (!a_fp16 || !a_q || !s_a) return ORC_NULL;
  if (M < 0 || K <= 0 || lda < K) return ORC_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    const uint16_t* row = a_fp16 + m * lda;
    float amax = 0.0f;
    for (int64_t k = 0; k < K; ++k) {
      const float v = fabsf(qqq_oracle_half_to_float(row[k]));
      if (v > amax) amax = v;
    }
    if (amax == 0.0f) {
      s_a[m] = 0.0f;
      for (int64_t k = 0; k < K; ++k) a_q[m * K + k] = 0;
      continue;
    }
    /* fp32 division, correctly rounded: the double quotient rounded once more to
     * float equals the correctly rounded float quotient (53 >= 2*24+2 bits). */
    const float s = (float)((double)amax / 127.0);
    s_a[m] = s;
    for (int64_t k = 0; k < K; ++k) {
      const float x = qqq_oracle_half_to_float(row[k]);
      const float q = (float)((double)x / (double)s);
      double r = nearbyint((double)q); /* ties to even */
      if (r > 127.0) r = 127.0;
      if (r < -127.0) r = -127.0;
      a_q[m * K + k] = (int8_t)r;
    }
  }
  return ORC_OK;
}

/* ---------- Sec. 3.3.1 / 3.3.2: the int8 weight that enters the INT8 GEMM ---------- */

/* per-channel: the int4 code itself, widened */
int qqq_oracle_w8_perchannel(const uint32_t* w_nat, int64_t N, int64_t K, int8_t* w8) {
  if (!w_nat || !w8) return ORC_NULL;
  if (N <= 0 || K <= 0 || K % 8) return ORC_SHAPE;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) w8[n * K + k] = (int8_t)code_at(w_nat, K, n, k);
  return ORC_OK;
}

/* per-group: code times the fused integer group scale s_g[k/group][n], saturated to int8 */
int qqq_oracle_w8_pergroup(const uint32_t* w_nat, const int8_t* s_g, int64_t N, int64_t K,
                           int64_t group, int8_t* w8) {
  if (!w_nat || !s_g || !w8) return ORC_NULL;
  if (N <= 0 || K <= 0 || K % 8 || group <= 0 || K % group) return ORC_SHAPE;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) {
      int p = code_at(w_nat, K, n, k) * (int)s_g[(k / group) * N + n];
      if (p > 127) p = 127;
      if (p < -128) p = -128;
      w8[n * K + k] = (int8_t)p;
    }
  return ORC_OK;
}

/* ---------- Sec. 3.3: INT8 GEMM, accumulator that cannot overflow ---------- */

int qqq_oracle_int8_gemm(const int8_t* a_q, const int8_t* w8, int64_t M, int64_t N, int64_t K,
                         int64_t* acc) {
  if (!a_q || !w8 || !acc) return ORC_NULL;
  if (M < 0 || N <= 0 || K <= 0) return ORC_SHAPE;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      int64_t s = 0;
      for (int64_t k = 0; k < K; ++k) s += (int64_t)a_q[m * K + k] * (int64_t)w8[n * K + k];
      acc[m * N + n] = s;
    }
  return ORC_OK;
}

/* ---------- Sec. 3.3.1 / 3.3.2: Dequant, INT32 -> FP16 ---------- */

static uint16_t dequant_one(int64_t acc, float s_a, uint16_t s_w_bits, float* y32_out) {
  const double y = (double)acc * (double)s_a * (double)qqq_oracle_half_to_float(s_w_bits);
  const float y32 = (float)y; /* the fp32-rounded result */
  if (y32_out) *y32_out = y32;
  return qqq_oracle_float_to_half(y32);
}

int qqq_oracle_dequant(const int64_t* acc, const float* s_a, const uint16_t* s_w_fp16, int64_t M,
                       int64_t N, float* y32, uint16_t* y_fp16) {
  if (!acc || !s_a || !s_w_fp16 || !y_fp16) return ORC_NULL;
  if (M < 0 || N <= 0) return ORC_SHAPE;
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n)
      y_fp16[m * N + n] =
          dequant_one(acc[m * N + n], s_a[m], s_w_fp16[n], y32 ? &y32[m * N + n] : NULL);
  return ORC_OK;
}

/* ---------- the two GEMM variants, composed from the steps above ---------- */

static int gemm_common(const int8_t* a_q, const float* s_a, const int8_t* w8,
                       const uint16_t* s_w_fp16, int64_t M, int64_t N, int64_t K, int32_t* acc32,
                       float* y32, uint16_t* y_fp16) {
  int64_t* acc = (int64_t*)malloc(sizeof(int64_t) * (size_t)(M > 0 ? M : 1) * (size_t)N);
  if (!acc) return ORC_SHAPE;
  int rc = qqq_oracle_int8_gemm(a_q, w8, M, N, K, acc);
  if (rc == ORC_OK) {
    for (int64_t i = 0; i < M * N; ++i) {
      if (acc[i] > INT32_MAX || acc[i] < INT32_MIN) {
        rc = ORC_OVERFLOW;
        break;
      }
      if (acc32) acc32[i] = (int32_t)acc[i];
    }
  }
  if (rc == ORC_OK && y_fp16) rc = qqq_oracle_dequant(acc, s_a, s_w_fp16, M, N, y32, y_fp16);
  free(acc);
  return rc;
}

int qqq_oracle_gemm_perchannel(const int8_t* a_q, const float* s_a, const uint32_t* w_nat,
                               const uint16_t* s_w_fp16, int64_t M, int64_t N, int64_t K,
                               int32_t* acc32, float* y32, uint16_t* y_fp16) {
  if (!a_q || !s_a || !w_nat || !s_w_fp16) return ORC_NULL;
  if (M < 0 || N <= 0 || K <= 0 || K % 8) return ORC_SHAPE;
  int8_t* w8 = (int8_t*)malloc((size_t)N * (size_t)K);
  if (!w8) return ORC_SHAPE;
  int rc = qqq_oracle_w8_perchannel(w_nat, N, K, w8);
  if (rc == ORC_OK) rc = gemm_common(a_q, s_a, w8, s_w_fp16, M, N, K, acc32, y32, y_fp16);
  free(w8);
  return rc;
}

int qqq_oracle_gemm_pergroup(const int8_t* a_q, const float* s_a, const uint32_t* w_nat,
                             const int8_t* s_g, const uint16_t* s_w_fp16, int64_t group, int64_t M,
                             int64_t N, int64_t K, int32_t* acc32, float* y32, uint16_t* y_fp16) {
  if (!a_q || !s_a || !w_nat || !s_g || !s_w_fp16) return ORC_NULL;
  if (M < 0 || N <= 0 || K <= 0 || K % 8 || group <= 0 || K % group) return ORC_SHAPE;
  int8_t* w8 = (int8_t*)malloc((size_t)N * (size_t)K);
  if (!w8) return ORC_SHAPE;
  int rc = qqq_oracle_w8_pergroup(w_nat, s_g, N, K, group, w8);
  if (rc == ORC_OK) rc = gemm_common(a_q, s_a, w8, s_w_fp16, M, N, K, acc32, y32, y_fp16);
  free(w8);
  return rc;
}

/* ---------- Sec. 3.3.2 with the paper's real-valued fused scale ---------- */

/* double -> fp16 bits, round to nearest even, overflow to infinity, subnormals kept.
 * Scaling by a power of two is exact, so one rint() (default rounding mode: nearest
 * even) is the only rounding. */
uint16_t qqq_oracle_double_to_half(double x) {
  const uint16_t sign = signbit(x) ? 0x8000u : 0u;
  double a = fabs(x);
  if (isnan(a)) return (uint16_t)(sign | 0x7E00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u); /* 65520 is the midpoint above the largest fp16 */
  if (a < 6.103515625e-05) {                            /* below 2^-14: subnormal spacing 2^-24 */
    const double q = rint(ldexp(a, 24));
    return (uint16_t)(sign | (uint16_t)q);              /* q == 1024 is the smallest normal */
  }
  int e;
  (void)frexp(a, &e); /* a = f * 2^e, f in [0.5,1): a in [2^(e-1), 2^e) */
  e -= 1;
  double q = rint(ldexp(a, 10 - e)); /* in [1024, 2048] */
  if (q >= 2048.0) {
    q = 1024.0;
    e += 1;
  }
  if (e > 15) return (uint16_t)(sign | 0x7C00u);
  return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)q - 1024));
}

/* One weight, in the paper's order: the int4 code as fp16 (FastINT4toFP16 is exact), then
 * FusedDequantQuant and the first half of FastFP16toINT8 as ONE fp16 fused multiply-add
 * x = code * s + (128 + 1024), then the low mantissa byte, then XOR 0x80.  The product and
 * the sum are exact in double (15 + 11 significant bits, exponent span < 53 bits), so the
 * single fp16 rounding of the FMA is the conversion below.  Where code*s rounds into
 * [-128,127] the result is that integer (round half to even); outside, it is whatever the
 * byte extraction gives: no saturation, as in the paper. */
int8_t qqq_oracle_w8_f16scale_one(int code, uint16_t s_bits) {
  const double s = (double)qqq_oracle_half_to_float(s_bits);
  const uint16_t x = qqq_oracle_double_to_half((double)code * s + 1152.0);
  return (int8_t)(uint8_t)((x & 0xFFu) ^ 0x80u);
}

int qqq_oracle_w8_pergroup_f16(const uint32_t* w_nat, const uint16_t* s_g_fp16, int64_t N,
                               int64_t K, int64_t group, int8_t* w8) {
  if (!w_nat || !s_g_fp16 || !w8) return ORC_NULL;
  if (N <= 0 || K <= 0 || K % 8 || group <= 0 || K % group) return ORC_SHAPE;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k)
      w8[n * K + k] = qqq_oracle_w8_f16scale_one(code_at(w_nat, K, n, k), s_g_fp16[(k / group) * N + n]);
  return ORC_OK;
}

int qqq_oracle_gemm_pergroup_f16(const int8_t* a_q, const float* s_a, const uint32_t* w_nat,
                                 const uint16_t* s_g_fp16, const uint16_t* s_w_fp16, int64_t group,
                                 int64_t M, int64_t N, int64_t K, int32_t* acc32, float* y32,
                                 uint16_t* y_fp16) {
  if (!a_q || !s_a || !w_nat || !s_g_fp16 || !s_w_fp16) return ORC_NULL;
  if (M < 0 || N <= 0 || K <= 0 || K % 8 || group <= 0 || K % group) return ORC_SHAPE;
  int8_t* w8 = (int8_t*)malloc((size_t)N * (size_t)K);
  if (!w8) return ORC_SHAPE;
  int rc = qqq_oracle_w8_pergroup_f16(w_nat, s_g_fp16, N, K, group, w8);
  if (rc == ORC_OK) rc = gemm_common(a_q, s_a, w8, s_w_fp16, M, N, K, acc32, y32, y_fp16);
  free(w8);
  return rc;
}

/* ---------- single outputs, one by one, straight from the definitions ----------
 * Used to check sampled entries of shapes whose full product would take the CPU too
 * long.  s_g == NULL selects the per-channel variant. */
int qqq_oracle_gemm_samples(const int8_t* a_q, const float* s_a, const uint32_t* w_nat,
                            const int8_t* s_g, const uint16_t* s_w_fp16, int64_t group, int64_t M,
                            int64_t N, int64_t K, const int64_t* idx_m, const int64_t* idx_n,
                            int64_t count, int64_t* acc_out, uint16_t* y_fp16) {
  if (!a_q || !s_a || !w_nat || !s_w_fp16 || !idx_m || !idx_n || !acc_out) return ORC_NULL;
  if (M <= 0 || N <= 0 || K <= 0 || K % 8) return ORC_SHAPE;
  if (s_g && (group <= 0 || K % group)) return ORC_SHAPE;
  for (int64_t i = 0; i < count; ++i)
    if (idx_m[i] < 0 || idx_m[i] >= M || idx_n[i] < 0 || idx_n[i] >= N) return ORC_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    const int64_t m = idx_m[i], n = idx_n[i];
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k) {
      int w = code_at(w_nat, K, n, k);
      if (s_g) {
        w *= (int)s_g[(k / group) * N + n];
        if (w > 127) w = 127;
        if (w < -128) w = -128;
      }
      s += (int64_t)a_q[m * K + k] * (int64_t)w;
    }
    acc_out[i] = s;
    if (y_fp16) y_fp16[i] = dequant_one(s, s_a[m], s_w_fp16[n], NULL);
  }
  return ORC_OK;
}

/* the same for the real-valued fp16 group scale of Sec. 3.3.2 */
int qqq_oracle_gemm_samples_f16(const int8_t* a_q, const float* s_a, const uint32_t* w_nat,
                                const uint16_t* s_g_fp16, const uint16_t* s_w_fp16, int64_t group,
                                int64_t M, int64_t N, int64_t K, const int64_t* idx_m,
                                const int64_t* idx_n, int64_t count, int64_t* acc_out,
                                uint16_t* y_fp16) {
  if (!a_q || !s_a || !w_nat || !s_g_fp16 || !s_w_fp16 || !idx_m || !idx_n || !acc_out) return ORC_NULL;
  if (M <= 0 || N <= 0 || K <= 0 || K % 8 || group <= 0 || K % group) return ORC_SHAPE;
  for (int64_t i = 0; i < count; ++i)
    if (idx_m[i] < 0 || idx_m[i] >= M || idx_n[i] < 0 || idx_n[i] >= N) return ORC_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    const int64_t m = idx_m[i], n = idx_n[i];
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k)
      s += (int64_t)a_q[m * K + k] *
           (int64_t)qqq_oracle_w8_f16scale_one(code_at(w_nat, K, n, k), s_g_fp16[(k / group) * N + n]);
    acc_out[i] = s;
    if (y_fp16) y_fp16[i] = dequant_one(s, s_a[m], s_w_fp16[n], NULL);
  }
  return ORC_OK;
}

/* ---------- Offline front-end: symmetric round-to-nearest int4 weights from fp16 ----------
 *
 * What the offline (blue) boxes of Fig. 5 and the "scale adjusted offline" remark of
 * Sec. 3.3.1 need as input: int4 codes and their scales.  The paper says only that the
 * quantisation is symmetric (Sec. 3.3, first paragraph); the readings taken here:
 *   scale  = max|w| / 7 over the channel (per-channel) or the group of 128 (per-group),
 *            fp32 correctly rounded division, stored as fp16 (round to nearest even);
 *   code   = clamp(rne(w / scale), -7, 7) with the STORED fp16 scale, fp32 correctly
 *            rounded division, ties to even; the symmetric range keeps |code * s*| inside
 *            int8 for every scale the per-group rule below can produce;
 *   a zero scale (all-zero channel/group, or max|w|/7 below half the smallest fp16) gives
 *   codes 0.
 * Per-group additionally (Fig. 4, Fig. 5):
 *   dequantised weight  w~ = code * s_Wg   (exact in fp32: 3 x 11 significant bits)
 *   s_Wc[n]  = max_k |w~[n,k]| / 127, fp32 division, stored as fp16   (fp16 -> int8 scale)
 *   s*_Wg    = s_Wg / s_Wc, fp32 division, stored as fp16, and never above 18.203125, the
 *              largest fp16 value whose product with a code of +-7 still rounds inside
 *              [-127,127]; the cap can only bind where s_Wc is subnormal in fp16 (a channel
 *              whose largest weight is below about 0.008).  s_Wc = 0 gives s* = 0.
 *   integer form of the fused scale (for the integer-scale GEMM): clamp(rne(s*), 1, 18).
 */

static uint16_t scale_bits(float amax, double qmax) {
  return qqq_oracle_float_to_half((float)((double)amax / qmax));
}

static int rtn_code(float w, float s) {
  if (s == 0.0f) return 0;
  const float q = (float)((double)w / (double)s);
  double r = nearbyint((double)q);
  if (r > 7.0) r = 7.0;
  if (r < -7.0) r = -7.0;
  return (int)r;
}

static void put_code(uint32_t* w_nat, int64_t K, int64_t n, int64_t k, int code) {
  uint32_t* word = &w_nat[n * (K / 8) + k / 8];
  const int sh = 4 * (int)(k % 8);
  *word = (*word & ~(0xFu << sh)) | ((uint32_t)(code & 0xF) << sh);
}

/* Sec. 3.3.1: per-channel scale s_W[n] and codes.  w_fp16 [N, ldw]; w_nat [N, K/8]; s_w [N]. */
int qqq_oracle_quantize_w4_perchannel(const uint16_t* w_fp16, int64_t N, int64_t K, int64_t ldw,
                                      uint32_t* w_nat, uint16_t* s_w_fp16) {
  if (!w_fp16 || !w_nat || !s_w_fp16) return ORC_NULL;
  if (N < 0 || K <= 0 || K % 8 != 0 || ldw < K) return ORC_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    const uint16_t* row = w_fp16 + n * ldw;
    float amax = 0.0f;
    for (int64_t k = 0; k < K; ++k) {
      const float v = fabsf(qqq_oracle_half_to_float(row[k]));
      if (v > amax) amax = v;
    }
    s_w_fp16[n] = scale_bits(amax, 7.0);
    const float s = qqq_oracle_half_to_float(s_w_fp16[n]);
    for (int64_t k = 0; k < K; ++k) put_code(w_nat, K, n, k, rtn_code(qqq_oracle_half_to_float(row[k]), s));
  }
  return ORC_OK;
}

/* Sec. 3.3.2, Fig. 5 (offline part).  Outputs: w_nat [N,K/8]; s_wg [K/group, N] (may be NULL);
 * s_star [K/group, N]; s_int [K/group, N] (may be NULL); s_wc [N]. */
int qqq_oracle_quantize_w4_pergroup(const uint16_t* w_fp16, int64_t N, int64_t K, int64_t ldw,
                                    int64_t group, uint32_t* w_nat, uint16_t* s_wg_fp16,
                                    uint16_t* s_star_fp16, int8_t* s_int, uint16_t* s_wc_fp16) {
  if (!w_fp16 || !w_nat || !s_star_fp16 || !s_wc_fp16) return ORC_NULL;
  if (N < 0 || K <= 0 || group <= 0 || group % 8 != 0 || K % group != 0 || ldw < K) return ORC_SHAPE;
  const int64_t G = K / group;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    const uint16_t* row = w_fp16 + n * ldw;
    uint16_t* sg = (uint16_t*)malloc((size_t)G * sizeof(uint16_t));
    float dmax = 0.0f; /* max_k |w~[n,k]| */
    for (int64_t g = 0; g < G; ++g) {
      float amax = 0.0f;
      for (int64_t k = g * group; k < (g + 1) * group; ++k) {
        const float v = fabsf(qqq_oracle_half_to_float(row[k]));
        if (v > amax) amax = v;
      }
      sg[g] = scale_bits(amax, 7.0);
      const float s = qqq_oracle_half_to_float(sg[g]);
      for (int64_t k = g * group; k < (g + 1) * group; ++k) {
        const int code = rtn_code(qqq_oracle_half_to_float(row[k]), s);
        put_code(w_nat, K, n, k, code);
        const float wd = fabsf((float)code * s);
        if (wd > dmax) dmax = wd;
      }
    }
    s_wc_fp16[n] = scale_bits(dmax, 127.0);
    const float s_wc = qqq_oracle_half_to_float(s_wc_fp16[n]);
    for (int64_t g = 0; g < G; ++g) {
      uint16_t star = 0;
      if (s_wc != 0.0f) {
        const float q = (float)((double)qqq_oracle_half_to_float(sg[g]) / (double)s_wc);
        star = qqq_oracle_float_to_half(q);
        if (qqq_oracle_half_to_float(star) > 18.203125f) star = qqq_oracle_float_to_half(18.203125f);
      }
      s_star_fp16[g * N + n] = star;
      if (s_wg_fp16) s_wg_fp16[g * N + n] = sg[g];
      if (s_int) {
        double r = nearbyint((double)qqq_oracle_half_to_float(star));
        if (r < 1.0) r = 1.0;
        if (r > 18.0) r = 18.0;
        s_int[g * N + n] = (int8_t)r;
      }
    }
    free(sg);
  }
  return ORC_OK;
}
