// Internal declarations shared by the translation units of libqqq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qqq.h"
#include "qqq_tuning.h"

namespace qqq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

// How the int4 codes become the int8 MFMA operand.
enum Mode : int {
  kPerChannel = 0,    // Sec. 3.3.1: code in the upper nibble (x16), undone before the scales
  kGroupLinear = 1,   // Sec. 3.3.2 with s_g <= 16: clamp is dead, so the group scale is applied to
                      // the group's partial int32 sum instead of to each weight (same integers)
  kGroupClamp = 2,    // Sec. 3.3.2, general: code*s_g saturated to int8 per weight (fp16 route)
  kGroupFused = 3,    // Sec. 3.3.2 with s_g <= 16: per-weight fp16 FMA + byte extract, no clamp
  kGroupFusedWide = 7,  // the same conversion for s_g <= 18 under the promise that no code is -8 (its
                        // constants stay exact in fp16 and code * s_g stays inside int8); not eligible
                        // for the biased integer route, whose byte products (code + 8) * s_g need s_g <= 17
  kGroupBias = 5,     // Sec. 3.3.2 with s_g <= 16, prefill: byte-wise integer multiply of code+8, sign by a
                      // top-bit flip; the constant 8*s_g - 128 per weight is taken out again through
                      // per-group row sums of the activations (see qqq_group_bias.hip)
  kGroupBiasWide = 8, // the same byte-wise route for s_g <= 18 under the promise that no code is -8: bytes of
                      // (7 - code) * s_g (<= 252), i.e. the NEGATED product plus (7*s_g - 128); the sign goes
                      // into the Dequant's channel scale
  kGroupCvt = 6,      // ablation only (Sec. 4.5.2, Fig. 9): the real-valued scale through conventional
                      // conversion instructions instead of FastFP16toINT8
  kGroupReal = 4,     // Sec. 3.3.2 as printed: real-valued fp16 fused scale s*_Wg, one fp16 FMA with
                      // 128 + 1024, low byte, XOR 0x80, no saturation; s_g then points at fp16 data
};

struct GemmParams {
  const int8_t* a_q;    // [M,K]
  const float* s_a;     // [M]
  const uint4* w;       // packed int4, 1 KiB chunks [K/128][N/16][64 lanes]
  const int8_t* s_g;    // [K/128,N] or nullptr
  const _Float16* s_w;  // [N]
  _Float16* y;          // [M,N]
  int32_t* acc_out;     // [M,N] or nullptr
  int32_t* ws_cnt;      // [N/16] arrival counters (zero between calls)
  int32_t* ws_acc;      // [ws_rows,N] split-K partial sums (zero between calls)
  int M, N, K, T;       // T = K/128
  // kGroupBias only: pre-pass outputs, [M][Gp], [M][Gp], [N][Gp] int8, Gp = K/128 rounded up to 32
  const int8_t* r_lo;
  const int8_t* r_hi;
  const int8_t* bias_w;
  // prefill, per-tile kernel only: k_splits > 1 splits K over gridDim.y workgroups per tile, each
  // storing its raw int32 tile into part[split][M][N]; a second kernel sums and dequantises
  int k_splits;
  int32_t* part;
  // fused activation quantisation (decode kernel only): fp16 rows instead of a_q/s_a
  const uint4* a_fp16;  // [M, lda] fp16 as 128-bit vectors, or nullptr
  int64_t lda_vec;      // row stride of a_fp16 in 128-bit vectors
};

// host-side helpers (qqq_api.hip)
int set_error(int code, const char* fmt, ...);
int num_cus();
void route_reset();                      // qqq_last_route(): entry points reset,
void route_note(const char* fmt, ...);   // launchers append what they enqueued

// launchers; each returns QQQ_OK or QQQ_ERR_HIP/QQQ_ERR_SHAPE
int launch_quant_act(const void* a, int64_t M, int64_t K, int64_t lda, int8_t* a_q, float* s_a,
                     hipStream_t st, int8_t* r_lo = nullptr, int8_t* r_hi = nullptr);
int launch_quant_weight(const void* w, int64_t N, int64_t K, int64_t ldw, bool grouped, uint32_t* w_nat,
                        uint16_t* s_ch, uint16_t* s_wg, uint16_t* s_star, int8_t* s_int, hipStream_t st);
int launch_pack(const uint32_t* w_nat, int64_t N, int64_t K, uint32_t* w_packed, bool inverse,
                hipStream_t st);
int launch_gemm_skinny(const GemmParams& p, int mode, hipStream_t st);
int decode_channel_tiles(int64_t N, int mt, bool light_conversion);  // 16-channel tiles per decode workgroup
int launch_group_bias_prepass(const int8_t* a_q, const int8_t* s_g, int64_t M, int64_t N, int64_t K,
                              int8_t* r_lo, int8_t* r_hi, int8_t* bc, bool with_row_sums, int code_offset,
                              hipStream_t st);
// the two byte-wise integer routes of the per-group prefill GEMM
constexpr bool is_bias_mode(int mode) { return mode == kGroupBias || mode == kGroupBiasWide; }
void set_skinny_tuning(int nt, int s, int w, int u);
void set_prefill_tuning(int tune);
int get_prefill_tuning();
int get_prefill_ring_depth();
int launch_gemm_prefill_dma(const GemmParams& p, int mode, int shape, hipStream_t st);
int launch_gemm_prefill_ring(const GemmParams& p, int mode, hipStream_t st);
int launch_splitk_reduce(const GemmParams& p, int mode, hipStream_t st);
void set_prefill_ksplit(int s);
int get_prefill_ksplit();

constexpr int kFusedMaxM = 4;          // rows the decode kernel quantises itself (fused path)
constexpr int kFusedLdsBytes = 32768;  // most activations the fused path quantises: M*K int8 in LDS
constexpr int kFusedLdsSmall = 8192;   // the smaller of its two prologue sizes
constexpr int kSkinnyMaxM = 64;  // rows the split-K kernel handles (4 MFMA row tiles)
// rows up to which the decode kernel is always the automatic choice; from there to kSkinnyMaxM a
// cost model decides between it and the prefill path's 64-row tiles (which read every activation
// row once per 128 channels instead of once per 32), and the workspace carries the prefill scratch
constexpr int kDecodeAlwaysMaxM = 16;

// ---------------------------------------------------------------------------------------------
// Packed layout.  Chunk (nt, t) = output channels [16nt,16nt+16) x k in [128t,128t+128), 1 KiB at
// (t*(N/16)+nt)*1024 (k-step major: all channels of one k-step are contiguous).
// Lane l = nl + 16*kc (nl = n%16, kc = 0..3) owns 16 bytes = dwords d0..d3.
// Nibble q of dword i holds the code of k = 128t + 64*(i/2) + 16*kc + 8*(i%2) + 4*(q%2) + q/2,
// i.e. each packed dword is natural word (k/8) with its nibbles reordered 0,4,1,5,2,6,3,7 so that
// "even nibbles" and "odd nibbles" each come out as four k-consecutive bytes.
// After conversion, dwords (lo(d0),hi(d0),lo(d1),hi(d1)) are the 16 k-consecutive int8 values
// k = 128t + 16kc + 0..15 of MFMA step 0 and (lo(d2),hi(d2),lo(d3),hi(d3)) those of step 1 (+64).
// ---------------------------------------------------------------------------------------------

// Sec. 3.3.1 FastINT4toINT8: nibble into the upper half of its byte = 16*code as int8.
__device__ __forceinline__ void unpack_x16(uint32_t x, int& lo, int& hi) {
  lo = (int)((x << 4) & 0xF0F0F0F0u);
  hi = (int)(x & 0xF0F0F0F0u);
}

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// Sec. 3.3.2, general route: int4 -> fp16 by mantissa placement (FastINT4toFP16: 0x6400|u is
// 1024+u), FusedDequantQuant as one fp16 multiply by the integer group scale, saturation to
// [-128,127], then FastFP16toINT8: adding 1536 puts code*s mod 256 into the low mantissa byte
// (1536 = 1024 + 512 keeps the sum inside [1024,2048) and makes the byte two's complement
// directly, so the XOR 0x80 of the unsigned variant is not needed).
// `s` holds the scale in both halves.  All intermediate values are integers below 2048: exact.
__device__ __forceinline__ void unpack_group_clamp(uint32_t x, h2 s, int& lo, int& hi) {
  const uint32_t y = x ^ 0x88888888u;  // two's complement nibble -> offset binary u = code + 8
  const h2 k1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
  const h2 k1536 = {(_Float16)1536.0f, (_Float16)1536.0f};
  const h2 kmin = {(_Float16)-128.0f, (_Float16)-128.0f};
  const h2 kmax = {(_Float16)127.0f, (_Float16)127.0f};
  uint32_t f[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    h2 c = as_h2(((y >> (4 * j)) & 0x000F000Fu) | 0x64006400u) - k1032;  // nibbles j and j+4
    h2 p = c * s;
    p = __builtin_elementwise_min(__builtin_elementwise_max(p, kmin), kmax);
    f[j] = as_u32(p + k1536);
  }
  // bytes: lo = nibbles (0,2,4,6) = (f0.b0, f2.b0, f0.b2, f2.b2); hi = nibbles (1,3,5,7)
  lo = (int)((f[0] & 0xFFu) | ((f[2] & 0xFFu) << 8) | (f[0] & 0x00FF0000u) |
             ((f[2] & 0x00FF0000u) << 8));
  hi = (int)((f[1] & 0xFFu) | ((f[3] & 0xFFu) << 8) | (f[1] & 0x00FF0000u) |
             ((f[3] & 0x00FF0000u) << 8));
}

// Sec. 3.3.2 with the clamp dead (s <= 16): one fp16 FMA per weight pair does the scale multiply
// and the magic add together.  Even nibble pairs sit at mantissa bit 0 (value 1024+u, multiplier
// s, addend 1536-1032s); odd nibble pairs are left at mantissa bit 4 (value 1024+16u, multiplier
// s/16, addend 1536-72s) which saves their shift.  All four constants are exact in fp16 for s<=16.
struct GroupFusedConsts {
  h2 s, c0, s16, c1;
};
__device__ __forceinline__ GroupFusedConsts make_group_fused(int s) {
  const float fs = (float)s;
  GroupFusedConsts g;
  g.s = {(_Float16)fs, (_Float16)fs};
  g.c0 = {(_Float16)(1536.0f - 1032.0f * fs), (_Float16)(1536.0f - 1032.0f * fs)};
  g.s16 = {(_Float16)(fs * 0.0625f), (_Float16)(fs * 0.0625f)};
  g.c1 = {(_Float16)(1536.0f - 72.0f * fs), (_Float16)(1536.0f - 72.0f * fs)};
  return g;
}
__device__ __forceinline__ void unpack_group_fused(uint32_t x, const GroupFusedConsts& g, int& lo,
                                                   int& hi) {
  const uint32_t y = x ^ 0x88888888u;
  const uint32_t y8 = y >> 8;
  const uint32_t magic = 0x64006400u;
  const h2 f0 = __builtin_elementwise_fma(as_h2((y & 0x000F000Fu) | magic), g.s, g.c0);     // 0,4
  const h2 f1 = __builtin_elementwise_fma(as_h2((y & 0x00F000F0u) | magic), g.s16, g.c1);   // 1,5
  const h2 f2 = __builtin_elementwise_fma(as_h2((y8 & 0x000F000Fu) | magic), g.s, g.c0);    // 2,6
  const h2 f3 = __builtin_elementwise_fma(as_h2((y8 & 0x00F000F0u) | magic), g.s16, g.c1);  // 3,7
  // v_perm_b32: selector bytes 0-3 pick from the second source, 4-7 from the first
  lo = (int)__builtin_amdgcn_perm(as_u32(f2), as_u32(f0), 0x06020400u);
  hi = (int)__builtin_amdgcn_perm(as_u32(f3), as_u32(f1), 0x06020400u);
}

// ---- per-token activation quantisation arithmetic (Sec. 4.1), shared by the stand-alone pass
// ---- and the decode kernel's fused prologue so both produce the same bits
__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}

// |max| over the 8 fp16 values of a 128-bit vector, on the bit patterns (for finite values the
// magnitude order of fp16 equals the integer order of the bits with the sign cleared)
__device__ __forceinline__ uint32_t absmax_bits(uint4 v, uint32_t cur) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = w[i] & 0x7FFFu, hi = (w[i] >> 16) & 0x7FFFu;
    cur = max(cur, max(lo, hi));
  }
  return cur;
}

// Maximum over the 64 lanes of a wave, in every lane (wave-uniform result).  Data-parallel
// primitives inside the 16-lane rows, then the four row results through scalar registers: no
// LDS-crossbar shuffles, whose latency would dominate a microsecond-scale prologue.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));  // row_mirror
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return max(max(r0, r1), max(r2, r3));
}

// rne(x / s) for |x / s| <= 127 (s = amax / 127), the quotient being the correctly rounded fp32 one,
// without dividing in the common case: q~ = x * rcp(s) is within 1.5 * 2^-23 relative of x/s, i.e.
// within 1.5 * 2^-16 absolute, and the rounded quotient within 2^-17; unless q~ lies within 2^-14 of
// a half-integer the two therefore round to the same integer.  Only near a tie the IEEE division
// (never a reciprocal multiply) decides.
__device__ __forceinline__ int quant1(float x, float s, float rs) {
  const float q = x * rs;
  float r = __builtin_rintf(q);
  if (__builtin_fabsf(q - r) > 0.5f - 0x1p-14f) r = __builtin_rintf(x / s);
  return (int)__builtin_amdgcn_fmed3f(r, -127.0f, 127.0f);  // guard clamp
}

__device__ __forceinline__ uint32_t quant4(uint32_t w0, uint32_t w1, float s) {
  // four fp16 values (two dwords) -> four int8 codes packed in one dword
  const float rs = __builtin_amdgcn_rcpf(s);
  const int q0 = quant1(half_bits_to_float(w0 & 0xFFFFu), s, rs), q1 = quant1(half_bits_to_float(w0 >> 16), s, rs);
  const int q2 = quant1(half_bits_to_float(w1 & 0xFFFFu), s, rs), q3 = quant1(half_bits_to_float(w1 >> 16), s, rs);
  return (uint32_t)(q0 & 0xFF) | ((uint32_t)(q1 & 0xFF) << 8) | ((uint32_t)(q2 & 0xFF) << 16) |
         ((uint32_t)(q3 & 0xFF) << 24);
}

// Sec. 3.3.2, integer scale s <= 16, biased route: u = code + 8 per nibble, four u per dword scaled
// by one 16-bit packed multiply (u*s <= 240 stays inside its byte), top bit flipped: each byte
// is then code*s + (8s - 128) as int8.  7 VALU ops per 8 weights.
// WIDE (s <= 18, no code is -8): the nibble XOR 7 is u = 7 - code in [0,14], u*s <= 252, and the byte is
// -code*s + (7s - 128): the same seven instructions give the negated product.
template <bool WIDE>
__device__ __forceinline__ void unpack_group_bias(uint32_t x, uint32_t s2, int& lo, int& hi) {
  const uint32_t ulo = (x ^ (WIDE ? 0x77777777u : 0x88888888u)) & 0x0F0F0F0Fu;
  const uint32_t uhi = ((x >> 4) ^ (WIDE ? 0x07070707u : 0x08080808u)) & 0x0F0F0F0Fu;
  typedef unsigned short us2 __attribute__((ext_vector_type(2)));
  const us2 sv = __builtin_bit_cast(us2, s2);
  const us2 plo = __builtin_bit_cast(us2, ulo) * sv;
  const us2 phi = __builtin_bit_cast(us2, uhi) * sv;
  lo = (int)(__builtin_bit_cast(uint32_t, plo) ^ 0x80808080u);
  hi = (int)(__builtin_bit_cast(uint32_t, phi) ^ 0x80808080u);
}

// Sec. 3.3.2 with the real-valued fused scale, step by step: FastINT4toFP16 (0x6400|u is 1024+u,
// 0x5400|(u<<4) is 64+u, each minus its offset and the +8 code bias gives the exact fp16 code),
// FusedDequantQuant fused with the first half of FastFP16toINT8 as one fp16 FMA
// code * s + (128 + 1024), whose single rounding in the [1024,2048) binade rounds code*s to an
// integer (half to even), then the low mantissa bytes (v_perm_b32, the PRMT of the paper) and
// XOR 0x80.  No saturation: the caller's scales keep |code*s| inside int8.
__device__ __forceinline__ void unpack_group_real(uint32_t x, h2 s2, int& lo, int& hi) {
  const uint32_t y = x ^ 0x88888888u;  // two's complement nibble -> code + 8
  const uint32_t y8 = y >> 8;
  const h2 off_lo = {(_Float16)1032.0f, (_Float16)1032.0f}, off_hi = {(_Float16)72.0f, (_Float16)72.0f};
  const h2 magic = {(_Float16)1152.0f, (_Float16)1152.0f};
  const h2 c0 = as_h2((y & 0x000F000Fu) | 0x64006400u) - off_lo;   // nibbles 0,4
  const h2 c1 = as_h2((y & 0x00F000F0u) | 0x54005400u) - off_hi;   // nibbles 1,5
  const h2 c2 = as_h2((y8 & 0x000F000Fu) | 0x64006400u) - off_lo;  // nibbles 2,6
  const h2 c3 = as_h2((y8 & 0x00F000F0u) | 0x54005400u) - off_hi;  // nibbles 3,7
  const h2 f0 = __builtin_elementwise_fma(c0, s2, magic);
  const h2 f1 = __builtin_elementwise_fma(c1, s2, magic);
  const h2 f2 = __builtin_elementwise_fma(c2, s2, magic);
  const h2 f3 = __builtin_elementwise_fma(c3, s2, magic);
  lo = (int)(__builtin_amdgcn_perm(as_u32(f2), as_u32(f0), 0x06020400u) ^ 0x80808080u);
  hi = (int)(__builtin_amdgcn_perm(as_u32(f3), as_u32(f1), 0x06020400u) ^ 0x80808080u);
}

// Ablation counterpart of unpack_group_real (Sec. 4.5.2, Fig. 9: what FastFP16toINT8 replaces): the
// same fp16 code and scale, but a plain fp16 multiply followed by the conventional conversion
// instructions (round to nearest even, fp16 -> int16) and byte packing.  Two roundings instead of
// one, so it equals the FMA route only where code*s is exact in fp16 (e.g. scales that are
// multiples of 1/16); it exists to be timed, not used.
__device__ __forceinline__ void unpack_group_cvt(uint32_t x, h2 s2, int& lo, int& hi) {
  const uint32_t y = x ^ 0x88888888u;
  const uint32_t y8 = y >> 8;
  const h2 off_lo = {(_Float16)1032.0f, (_Float16)1032.0f}, off_hi = {(_Float16)72.0f, (_Float16)72.0f};
  const h2 p0 = (as_h2((y & 0x000F000Fu) | 0x64006400u) - off_lo) * s2;   // nibbles 0,4
  const h2 p1 = (as_h2((y & 0x00F000F0u) | 0x54005400u) - off_hi) * s2;   // nibbles 1,5
  const h2 p2 = (as_h2((y8 & 0x000F000Fu) | 0x64006400u) - off_lo) * s2;  // nibbles 2,6
  const h2 p3 = (as_h2((y8 & 0x00F000F0u) | 0x54005400u) - off_hi) * s2;  // nibbles 3,7
  auto to_byte = [](_Float16 v) { return (uint32_t)((int)(short)__builtin_rintf16(v)) & 0xFFu; };
  lo = (int)(to_byte(p0[0]) | (to_byte(p2[0]) << 8) | (to_byte(p0[1]) << 16) | (to_byte(p2[1]) << 24));
  hi = (int)(to_byte(p1[0]) | (to_byte(p3[0]) << 8) | (to_byte(p1[1]) << 16) | (to_byte(p3[1]) << 24));
}

// Dequant (Sec. 3.3.1/3.3.2 last step): t = fp32(acc) * s_a rounded to fp32, then t * s_w rounded
// ONCE to fp16 (the mixed-precision multiply-add rounds its exact fp32-operand product straight to
// fp16).  Written as the instruction itself so that every kernel rounds alike: left to the
// compiler, a lone conversion becomes this instruction while two adjacent ones become fp32
// multiplies followed by a packed convert, which rounds twice and differs in the last bit for
// about one output in 2^13.
__device__ __forceinline__ _Float16 dequant(int acc, float sa, float sw) {
  const float t = (float)acc * sa;
  uint32_t r;  // the instruction writes the low half of its destination
  asm("v_fma_mixlo_f16 %0, %1, %2, 0" : "=v"(r) : "v"(t), "v"(sw));
  return __builtin_bit_cast(_Float16, (uint16_t)r);
}

}  // namespace qqq
