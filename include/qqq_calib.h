/*
 * qqq_calib.h — C ABI of the offline (calibration-time) stage of QQQ (arXiv 2406.09904) on one
 * layer, MI355X (gfx950): adaptive smoothing (Sec. 3.1) and Hessian-based quantisation compensation
 * (Sec. 3.2).  Its outputs feed the weight front-end / repack and the W4A8 GEMMs of qqq.h.
 *
 * Conventions as in qqq.h: every pointer is a DEVICE pointer owned by the caller (16-byte aligned
 * unless stated), `stream` is a hipStream_t passed as void*, a call only enqueues kernels, never
 * allocates, synchronises or throws; return QQQ_OK or an error code with nothing enqueued.
 * Matrices are row-major and dense: activations X [M,K] fp16 (M calibration tokens, K input
 * channels), weights W [N,K] fp16.  Supported shapes: those of the GEMMs (N % 16 == 0,
 * K % 128 == 0, K <= 131072), M >= 1; qqq_gptq_* additionally K <= 16384.
 */
#ifndef QQQ_CALIB_H_
#define QQQ_CALIB_H_

#include "qqq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Adaptive smoothing (Sec. 3.1, Eq. 1-2).  The paper fixes the selected set (channels whose
 * largest |activation| exceeds a threshold sigma: the sentence before Eq. 1; the printed "<" of
 * Eq. 1 is read as ">"), a grid search for sigma in [0, max|X|] and the loss
 * || Q(X ./ s) Q(W .* s)^T - X W^T ||^2.  This library's reading of the rest:
 *   s_t = max_m |X[m,t]| / sigma on the selected channels, 1 elsewhere (fp32, one division);
 *   grid sigma_g = fp32(max|X| * g / G), g = 1..G (g = G selects nothing: "no smoothing" is always
 *   a candidate); X' = fp16_rne(fp32(X) / s), W' = fp16_rne(fp32(W) * s);
 *   Q(X') = qqq_quant_act, Q(W') = qqq_quantize_w4_perchannel, their product the exact int32
 *   accumulator of qqq_gemm_w4a8_perchannel times s_a[m] s_w[n] in fp64; X W^T by an fp16 MFMA
 *   GEMM with fp32 accumulation; the loss summed in fp64; the first minimum over the grid wins.
 * Outputs: xs_fp16 [M,K] and ws_fp16 [N,K], the smoothed layer for the winning threshold;
 *   s [K] fp32 its smoothing vector; sigmas [G] fp32; losses [G] fp64; best [1] int32 (0-based
 *   grid index).  1 <= grid_points <= 256.
 * workspace: qqq_smoothing_workspace_bytes(M,N,K) bytes, contents irrelevant on entry.
 */
size_t qqq_smoothing_workspace_bytes(int64_t M, int64_t N, int64_t K);
int qqq_adaptive_smoothing(const void* x_fp16, const void* w_fp16, int64_t M, int64_t N, int64_t K,
                           int grid_points, void* xs_fp16, void* ws_fp16, float* s, float* sigmas,
                           double* losses, int32_t* best, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * Pieces of the above, exposed for tests and for callers that bring their own search:
 *   qqq_channel_absmax: absmax[t] = max_m |X[m,t]| (fp32, exact).
 *   qqq_smooth_apply: s from absmax [K] and *sigma (device fp32), then X' and W' as above.
 *   qqq_fp16_gemm_nt: y [M,N] fp32 = X W^T (fp16 MFMA, fp32 accumulation), M, N, K >= 1, K % 16 == 0.
 */
int qqq_channel_absmax(const void* x_fp16, int64_t M, int64_t K, float* absmax, void* stream);
int qqq_smooth_apply(const void* x_fp16, const void* w_fp16, const float* absmax, const float* sigma,
                     int64_t M, int64_t N, int64_t K, void* xs_fp16, void* ws_fp16, float* s,
                     void* stream);
int qqq_fp16_gemm_nt(const void* x_fp16, const void* w_fp16, int64_t M, int64_t N, int64_t K, float* y,
                     void* stream);

/*
 * Hessian of the layer-wise objective (Sec. 3.2): H [K,K] fp64 = 2 X^T X over the M tokens.
 */
int qqq_hessian(const void* x_fp16, int64_t M, int64_t K, double* H, void* stream);

/*
 * Hessian-based quantisation compensation (Sec. 3.2, Eq. 3-4) with the per-channel int4 quantiser
 * of qqq_quantize_w4_perchannel.  Input channels are taken in their natural order i = 0..K-1 for
 * all output channels at once (the layer-wise method the paper adopts; Eq. 3's greedy choice is not
 * used); after channel i is quantised, Eq. 4 moves the channels still in F,
 *   W[:, F] -= (W[:, i] - Q(W[:, i])) / [H_F^-1]_ii * (H_F^-1)[i, F],
 * and H_F^-1 for the smaller F follows by eliminating row and column i.  H is damped by
 * percdamp * mean(diag H) first; a channel with H_ii == 0 gets H_ii = 1 and weight 0.  All of it
 * in fp64.  Scale: s_w[n] = fp16_rne(fp32(max_k |W[n,k]|) / 7) from the original weights;
 * code = clamp(rne(fp32(w / s_w)), -7, 7) on the running fp64 weight.
 *   H [K,K] fp64 (read only); w_nat [N,K/8] natural nibble words (for qqq_pack_w4); s_w_fp16 [N].
 *   workspace: qqq_gptq_workspace_bytes(N,K) bytes, contents irrelevant on entry.
 * Cost: 4K small launches and about 3 K^3 fp64 operations (calibration-time code, not a hot path).
 */
size_t qqq_gptq_workspace_bytes(int64_t N, int64_t K);
int qqq_gptq_quantize_w4_perchannel(const void* w_fp16, const double* H, int64_t N, int64_t K,
                                    double percdamp, uint32_t* w_nat, void* s_w_fp16, void* workspace,
                                    size_t workspace_bytes, void* stream);


/*
 * The same compensation with the per-group int4 quantiser of qqq_quantize_w4_pergroup (Sec. 3.3.2: groups of
 * 128 input channels).  Sec. 3.2 does not say when a group's scale is fixed while Eq. 4 keeps moving the
 * weights; here it is fixed when the sweep reaches the group's first channel, from the weights as they stand
 * then (compensated by every channel quantised before): s_Wg[g,n] = fp16_rne(fp32(max_{k in g} |W[n,k]|) / 7),
 * code = clamp(rne(fp32(w / s_Wg)), -7, 7).  After the sweep s_Wc, s*_Wg and its integer form follow from the
 * codes and s_Wg exactly as in qqq_quantize_w4_pergroup, so with a diagonal H all outputs equal that call's.
 *   group must be 128 and K a multiple of it; s_wg_fp16, s_star_fp16 [K/128, N] fp16, s_int [K/128, N] int8 or
 *   NULL, s_wc_fp16 [N] fp16 (all written); the other arguments, the workspace and the cost as above.
 */
int qqq_gptq_quantize_w4_pergroup(const void* w_fp16, const double* H, int64_t N, int64_t K, int group,
                                  double percdamp, uint32_t* w_nat, void* s_wg_fp16, void* s_star_fp16,
                                  int8_t* s_int, void* s_wc_fp16, void* workspace, size_t workspace_bytes,
                                  void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QQQ_CALIB_H_ */
