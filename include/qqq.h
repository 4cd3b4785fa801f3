/*
 * qqq.h — C ABI of the MI355X (gfx950) W4A8 GEMM hot path of QQQ (arXiv 2406.09904).
 *
 * The path:  fp16 activations --qqq_quant_act--> int8 codes + per-token scale
 *            int4 weight codes --qqq_pack_w4 (offline)--> device tile layout
 *            qqq_gemm_w4a8_{perchannel,pergroup,pergroup_f16scale}:
 *                Y[m,n] = fp16( acc[m,n] * s_a[m] * s_w[n] ),  acc[m,n] = sum_k A_q[m,k] * W8[n,k]  (int32, exact)
 *            qqq_linear_w4a8_{perchannel,pergroup}: the first and the third step in one call
 *            fp16 weights --qqq_quantize_w4_{perchannel,pergroup} (offline)--> int4 codes + scales
 *
 * Conventions common to every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller, 16-byte aligned, unless a
 *     comment says "host".  The library never allocates, frees, synchronises or throws.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call only
 *     enqueues kernels on it; ordering on that stream is the only synchronisation.
 *   - Matrices are row-major and dense unless a leading dimension is given.
 *   - Supported shapes: 1 <= M, N % 16 == 0, K % 128 == 0, 128 <= K <= 131072
 *     (the worst-case |acc| = 127*128*K must stay below 2^31).  M == 0 is a no-op.
 *   - Return value: QQQ_OK, or an error code; on any error nothing was enqueued and
 *     no output was touched.  qqq_last_error() returns a static host string describing
 *     the most recent error on the calling thread.
 *   - Symmetric quantisation only: there are no zero-points anywhere (Sec. 3.3, Sec. 4.1).
 */
#ifndef QQQ_H_
#define QQQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QQQ_OK 0
#define QQQ_ERR_NULL 1      /* a required pointer is NULL */
#define QQQ_ERR_SHAPE 2     /* unsupported M/N/K/lda/group, or a misaligned pointer */
#define QQQ_ERR_WORKSPACE 3 /* workspace smaller than qqq_gemm_workspace_bytes() */
#define QQQ_ERR_HIP 4       /* the HIP runtime refused a launch */

#define QQQ_GROUP 128 /* the only group size of the per-group variant ("-g128", Table 1) */

/* Library version (major*100 + minor) and the text of the last error (host string, never NULL). */
int qqq_version(void);
const char* qqq_last_error(void);

/*
 * Per-token dynamic symmetric int8 quantisation of activations (Sec. 4.1 "Algorithm"; s_A in Fig. 3).
 *   for every row m:  amax = max_k |A[m,k]|
 *                     s_a[m] = amax / 127                      (fp32, correctly rounded division)
 *                     a_q[m,k] = clamp(rne(A[m,k] / s_a[m]), -127, 127)   (fp32 division, ties to even)
 *   an all-zero row gives s_a[m] = 0 and a_q[m,:] = 0.  Non-finite inputs are undefined.
 *   a_fp16: [M, lda] fp16, lda >= K, lda % 8 == 0 (elements).   a_q: [M,K] int8.   s_a: [M] fp32.
 */
int qqq_quant_act(const void* a_fp16, int64_t M, int64_t K, int64_t lda, int8_t* a_q, float* s_a,
                  void* stream);

/*
 * Offline weight front-end: symmetric round-to-nearest int4 codes and scales from fp16 weights
 * (the inputs of Sec. 3.3.1's offline scale adjustment and of the offline boxes of Fig. 5).
 * The paper fixes only "symmetric"; the arithmetic below is this library's reading of it.
 *   per block b (the whole channel, or a group of 128 along K):
 *     s_b  = fp16_rne( max_k |W[n,k]| / 7 )                       (fp32 division)
 *     code = clamp( rne( W[n,k] / s_b ), -7, 7 )                  (fp32 division by the STORED s_b,
 *            ties to even); s_b == 0 gives codes 0.  Non-finite weights are undefined.
 *   per-channel: s_w[n] = s_b, the s_W of Fig. 3 (the /16 of Sec. 3.3.1 is applied inside the GEMM).
 *   per-group (Fig. 4, Fig. 5): s_Wg[g][n] = s_b;
 *     s_wc[n]      = fp16_rne( max_k |code * s_Wg| / 127 )        (fp16 -> int8 scale s_Wc)
 *     s_star[g][n] = min( fp16_rne( s_Wg / s_wc ), 18.203125 )    (s*_Wg; 0 where s_wc == 0; the cap,
 *                    the largest fp16 s with rne(7*s) <= 127, binds only where s_wc is subnormal)
 *     s_int[g][n]  = clamp( rne( s_star ), 1, 18 )                (for the integer-scale GEMM; pass
 *                    sg_max = 18 | QQQ_SG_SYMMETRIC_CODES there: codes in [-7,7], no product saturates)
 *   w_fp16 [N, ldw] fp16 device, 16-byte aligned, ldw >= K, ldw % 8 == 0; K % 8 == 0 (per-group:
 *   K % 128 == 0).  w_nat [N, K/8] uint32 device, the natural format qqq_pack_w4 takes.
 *   s_w / s_wc [N] fp16; s_star, s_wg, s_int [K/128, N] row-major; s_int and s_wg may be NULL.
 *   With |code| <= 7 every product code * s_star rounds inside [-127,127], so the outputs can be fed
 *   to qqq_gemm_w4a8_pergroup_f16scale as they are.
 */
int qqq_quantize_w4_perchannel(const void* w_fp16, int64_t N, int64_t K, int64_t ldw, uint32_t* w_nat,
                               void* s_w_fp16, void* stream);
int qqq_quantize_w4_pergroup(const void* w_fp16, int64_t N, int64_t K, int64_t ldw, int group,
                             uint32_t* w_nat, void* s_star_fp16, int8_t* s_int, void* s_wc_fp16,
                             void* s_wg_fp16, void* stream);

/*
 * Offline weight repack (Sec. 3.3.1: weights are prepared offline; the kernels load int4).
 *   w_nat: [N, K/8] uint32, natural interchange format: nibble i (bits 4i..4i+3) of word j of
 *          row n is the 4-bit two's-complement code of W[n, 8j+i].
 *   w_packed: qqq_packed_w4_bytes(N,K) = N*K/2 bytes, opaque device tile layout: 1 KiB chunks of
 *          16 output channels x 128 k, ordered so that each lane's 128-bit load is, after the
 *          in-register int4->int8 conversion, its int8 MFMA operand for two consecutive K-steps.
 *   No value changes; qqq_unpack_w4 is the exact inverse (test helper).
 */
size_t qqq_packed_w4_bytes(int64_t N, int64_t K); /* 0 for unsupported shapes */
int qqq_pack_w4(const uint32_t* w_nat, int64_t N, int64_t K, void* w_packed, void* stream);
int qqq_unpack_w4(const void* w_packed, int64_t N, int64_t K, uint32_t* w_nat, void* stream);

/*
 * Scratch of the GEMM calls.  Its first part, qqq_gemm_workspace_zero_bytes() long (arrival
 * counters and split-K partial sums of the decode kernel), must be zero on entry: the caller
 * zero-fills the workspace ONCE after allocation and every call leaves that part zero again.  For
 * M > 16 (where the prefill kernels can be the automatic choice: the decode kernel handles M <= 64,
 * is always chosen up to 16 rows and by a cost model from 17 to 64) it is followed by plain scratch, which a call overwrites and no call
 * relies on: the per-group variant's pre-pass buffers (per-group row sums of the activations, a
 * transposed copy of the group scales) and, for M <= 512, slabs for K-split partial tiles
 * (4 * 1024 * N bytes).  The decode kernel requires the workspace; the prefill kernels take it as
 * optional (without it, or with a smaller one, the per-group variant uses its costlier per-weight
 * conversion and K is never split).  One workspace must not be shared by GEMM calls that may run
 * concurrently (different streams).
 */
size_t qqq_gemm_workspace_zero_bytes(int64_t M, int64_t N, int64_t K);
size_t qqq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Per-channel W4A8 GEMM (Sec. 3.3.1, Fig. 3): int4 code widened to int8 in registers
 * (upper-nibble placement = x16, undone exactly before the scales are applied), int8 MFMA with
 * int32 accumulation, Dequant fused:  Y[m,n] = fp16_rne( fp32_rne(float(acc[m,n]) * s_a[m]) * float(s_w[n]) )
 * (the second product is rounded once, straight to fp16; identical in every kernel, within 1 fp16
 * ulp of the exactly computed value).
 *   a_q [M,K] int8; s_a [M] fp32; w_packed from qqq_pack_w4; s_w_fp16 [N] fp16;
 *   y_fp16 [M,N] fp16 (written); acc_out [M,N] int32 or NULL: if given, also receives the TRUE
 *   accumulator sum_k A_q*code (parity/debug).
 */
int qqq_gemm_w4a8_perchannel(const int8_t* a_q, const float* s_a, const void* w_packed,
                             const void* s_w_fp16, void* y_fp16, int32_t* acc_out, int64_t M,
                             int64_t N, int64_t K, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * Per-group W4A8 GEMM (Sec. 3.3.2, Fig. 4-6): the int8 weight is code x fused group scale,
 *   W8[n,k] = clamp(code[n,k] * s_g[k/128][n], -128, 127),   s_g integer in 0..127,
 * then the same int8 MFMA and Dequant with the per-channel scale s_w (s_Wc in Fig. 4).
 *   s_g [K/128, N] int8 row-major; group must be 128.
 *   sg_max: the caller's promise that every s_g <= sg_max.  With 1 <= sg_max <= 16 the product
 *   cannot leave int8, the clamp is dead and a cheaper conversion is used; 0 = no promise
 *   (general saturating conversion).  A broken promise gives wrong results, not a fault
 *   (qqq_debug_count_sg_violations in qqq_tuning.h checks one).
 *   QQQ_SG_SYMMETRIC_CODES or-ed into sg_max adds the promise that no weight code is -8, i.e. the
 *   symmetric code range [-7,7] that qqq_quantize_w4_pergroup emits: then the clamp is dead up to
 *   sg_max = 18 (7 * 18 = 126), which is the range of that call's integer scales, and the cheaper
 *   conversions apply to them too: pass sg_max = 18 | QQQ_SG_SYMMETRIC_CODES for its outputs.
 */
#define QQQ_SG_SYMMETRIC_CODES 0x100
int qqq_gemm_w4a8_pergroup(const int8_t* a_q, const float* s_a, const void* w_packed,
                           const int8_t* s_g, const void* s_w_fp16, int group, int sg_max,
                           void* y_fp16, int32_t* acc_out, int64_t M, int64_t N, int64_t K,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-group W4A8 GEMM with the paper's real-valued fused scale (Sec. 3.3.2, Fig. 4-6, as printed):
 *   s_g_fp16 [K/128, N] fp16 row-major holds s*_Wg = s_Wg / s_Wc (computed offline, Fig. 5);
 *   W8[n,k] = FastFP16toINT8( fp16_fma( fp16(code[n,k]), s*_Wg[k/128][n], 128 + 1024 ) ):
 *   the FMA's single rounding in the [1024,2048) binade rounds code*s to an integer (half to
 *   even), the low mantissa byte XOR 0x80 is that integer as int8.  NO saturation: the caller's
 *   scales must keep |code * s| within int8 (|s| <= 15.875 is always safe); outside, the byte
 *   extraction wraps, exactly as the steps above do.  Then the same int8 MFMA and Dequant with
 *   s_w (s_Wc).  Other arguments as in qqq_gemm_w4a8_pergroup; s_g_fp16 must be 4-byte aligned.
 */
int qqq_gemm_w4a8_pergroup_f16scale(const int8_t* a_q, const float* s_a, const void* w_packed,
                                    const void* s_g_fp16, const void* s_w_fp16, int group,
                                    void* y_fp16, int32_t* acc_out, int64_t M, int64_t N, int64_t K,
                                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Linear layer in one call (Sec. 4.1 per-token activation quantisation feeding Sec. 3.3's W4A8
 * GEMM): the result is exactly that of qqq_quant_act followed by qqq_gemm_w4a8_perchannel /
 * qqq_gemm_w4a8_pergroup on the same inputs (acc_out bit-identical, y_fp16 bit-identical).
 * For a few decode rows (M <= 4 and M*K <= 8192; two or three rows up to M*K <= 32768; four rows
 * up to there on layers of 150 M weights and more) a single kernel does both: every workgroup
 * quantises the rows into LDS before streaming its weights, which removes one launch from a
 * microsecond-scale step.  Otherwise the two kernels run back to back on `stream`, with the
 * int8 activations and their scales in the workspace.
 *   a_fp16 [M,lda] fp16, lda >= K, lda % 8 == 0, 16-byte aligned; the other arguments as in the
 *   GEMM calls.  workspace: qqq_linear_workspace_bytes(M,N,K) bytes, zero-filled once after
 *   allocation (its split-K part is left zero by every call), never shared by concurrent calls.
 */
size_t qqq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
int qqq_linear_w4a8_perchannel(const void* a_fp16, int64_t lda, const void* w_packed,
                               const void* s_w_fp16, void* y_fp16, int32_t* acc_out, int64_t M,
                               int64_t N, int64_t K, void* workspace, size_t workspace_bytes,
                               void* stream);
int qqq_linear_w4a8_pergroup(const void* a_fp16, int64_t lda, const void* w_packed, const int8_t* s_g,
                             const void* s_w_fp16, int group, int sg_max, void* y_fp16,
                             int32_t* acc_out, int64_t M, int64_t N, int64_t K, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * For callers that cannot allocate or bring a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): qqq_linear_w4a8_perchannel with the library's own
 * scratch, a static device array of QQQ_STATIC_SCRATCH_BYTES per GPU that lives in the code
 * object until the process ends.  The call allocates nothing and takes no workspace; inputs and
 * outputs are the caller's, as above, and the result is bit-identical to qqq_linear_w4a8_perchannel.
 * Shapes whose qqq_linear_workspace_bytes(M,N,K) exceeds QQQ_STATIC_SCRATCH_BYTES return
 * QQQ_ERR_WORKSPACE (nothing enqueued): use the workspace-taking call for those.
 * Every call on a GPU shares that GPU's array, which keeps the previous call's contents: the call
 * itself clears (with a small fill kernel on `stream`) the part its kernels need zero, so one more
 * launch than the workspace-taking call for M <= 64.  Calls that may overlap on one GPU (different
 * streams, different threads) race on the array: serialise them.
 */
#define QQQ_STATIC_SCRATCH_BYTES (16u << 20)
int qqq_linear_w4a8_perchannel_static(const void* a_fp16, int64_t lda, const void* w_packed,
                                      const void* s_w_fp16, void* y_fp16, int32_t* acc_out, int64_t M,
                                      int64_t N, int64_t K, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QQQ_H_ */
