/*
 * qqq_tuning.h — tuning and diagnostic controls of libqqq (MI355X W4A8 GEMM hot path).
 *
 * NOT part of the product interface (that is qqq.h): these functions exist for the tests, the
 * benchmark's ablations and kernel tuning.  The setters change process-global host state and are
 * not thread-safe; leave everything at 0 / default in production use.
 */
#ifndef QQQ_TUNING_H_
#define QQQ_TUNING_H_

#include "qqq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Which kernels the most recent GEMM or linear call of the calling thread enqueued, as a short
 * host string (never NULL), e.g. "decode nt=4 mt=1 waves=8 depth=1 kslices=1 fused=1 mode=0 grid=448" or
 * "prefill persistent tile=128x512 mode=0 tiles=1792 grid=256" or "prefill per-tile tile=64x128 waves=4
 * ring=6 ksplit=4 mode=5 grid=64 + k-split reduce"; a preceding "quant_act + " or "group-bias pre-pass + "
 * names the other launches of the call.  For benchmarks and tests that must know which route they measured or compared.
 */
const char* qqq_last_route(void);

/*
 * Diagnostic check of the sg_max promise of qqq_gemm_w4a8_pergroup (Sec. 3.3.2's fused group scale
 * in its integer form): counts the entries of s_g [K/128, N] outside 0..sg_max into *violations
 * (device int32, overwritten).  A caller that cannot vouch for its scales runs this once per
 * weight, offline, before promising sg_max.  Enqueues one kernel on `stream`.
 */
int qqq_debug_count_sg_violations(const int8_t* s_g, int64_t N, int64_t K, int sg_max,
                                  int32_t* violations, void* stream);

/*
 * Ceiling probes for the benchmark (not part of the path).  Each enqueues ONE kernel on `stream`;
 * the caller times it.
 *   qqq_probe_stream_read: `workgroups` x 256 threads read `bytes` (multiple of 16) of `buf` once
 *     with coalesced 128-bit loads and nothing else: the streaming ceiling of a short launch.
 *   qqq_probe_mfma_i8: `workgroups` x 8 waves, each wave 4 x 2 tiles of v_mfma_i32_32x32x32_i8 per
 *     round (the prefill kernel's register dataflow, two waves per SIMD), operands held in
 *     registers, no memory traffic in the loop: 2 * 32^3 * 32 * 8 * iters * 4 operations per
 *     workgroup.  a_pool: 4*4*512 16-byte operand values (one per pool slot, row tile and thread),
 *     b_pool: 2*2*512; every workgroup reads the same pools.  The chip's clock under MFMA load depends
 *     on the operand values, which is why the caller supplies them.  sink: 4 bytes, never written
 *     in practice.
 *   qqq_probe_prefill_loop: `workgroups` x 8 waves run `steps` k-steps of the persistent prefill
 *     kernel's per-channel k-loop (64 v_mfma_i32_16x16x64_i8 per wave and k-step, the same LDS ring,
 *     fragment layout and DMA pieces) with the parts named by `parts` switched on; the others use operands that stay
 *     in registers.  src: workgroups x region_bytes bytes (16-byte aligned; region_bytes a multiple
 *     of the 51200-byte ring stage, at most 64 MiB): per stage 16 KiB of int8 activations (128 rows x
 *     128 k), 32 KiB of packed codes (32 tiles of 16 channels), 2 KiB ignored.  Workgroup b keeps to
 *     its own region; the ring starts as the region's first bytes and, with QQQ_PROBE_DMA, is refilled
 *     from the region cyclically, two k-steps ahead, with the kernel's wait and barrier.
 *     2 * 32^3 * 32 * 8 * steps operations per workgroup.  Supported combinations: 0, CONVERT,
 *     A_READS, A_READS|CONVERT, W_READS|CONVERT, DMA, A_READS|W_READS|CONVERT and all four;
 *     FORM_32X32X32 alone or with all four.
 *     This GPU runs MFMA-heavy kernels at its board power limit, so each part costs what its
 *     energy takes from the clock; the probe measures that on the caller's bytes.
 */
#define QQQ_PROBE_A_READS 1 /* activation fragments read from LDS every k-step (16 KiB per wave) */
#define QQQ_PROBE_W_READS 2 /* packed codes read from LDS every k-step (4 KiB per wave); implies CONVERT */
#define QQQ_PROBE_CONVERT 4 /* int4 -> int8 conversion redone every k-step (else hoisted) */
#define QQQ_PROBE_DMA 8     /* global -> LDS DMA of the next k-steps, its wait and the workgroup barrier */
#define QQQ_PROBE_FORM_32X32X32 16 /* the same wave patch as 4 x 2 tiles of v_mfma_i32_32x32x32_i8 (alone or with all parts) */
int qqq_probe_prefill_loop(const void* src, size_t region_bytes, int steps, int parts, int workgroups,
                           int32_t* sink, void* stream);
int qqq_probe_stream_read(const void* buf, size_t bytes, int workgroups, uint32_t* sink, void* stream);
int qqq_probe_mfma_i8(const void* a_pool, const void* b_pool, int iters, int workgroups, int32_t* sink,
                      void* stream);

/*
 * Tuning/diagnostic knob (host state, not thread-safe): 0 makes the qqq_linear_* calls always
 * run the two kernels, 1 (default) lets them use the fused decode kernel.  Returns the previous
 * value.
 */
int qqq_set_fused_quant(int enable);

/*
 * Tuning/diagnostic knob (host state, not thread-safe): force a kernel family.
 *   0 = automatic (decode kernel up to 16 rows, prefill kernels above 64, a cost model in between),
 *   1 = decode split-K kernel
 *   (M <= 64), 2 = LDS-tiled prefill kernels.
 * Returns the previous value.  Forcing a family outside its M range gives QQQ_ERR_SHAPE.
 */
int qqq_set_kernel_override(int family);

/*
 * Tuning/diagnostic knob (host state, not thread-safe): force how the per-group variant turns
 * code x s_g into int8.  0 = automatic (from sg_max, M and a cost model), 1 = scale applied to each group's
 * partial sum (valid for s_g <= 16), 2 = per-weight saturating conversion (any s_g),
 * 3 = per-weight fp16 FMA conversion without saturation (valid for s_g <= 16).  Values 1-3 act on
 * qqq_gemm_w4a8_pergroup / qqq_linear_w4a8_pergroup (3 also keeps the prefill kernels off their
 * default integer route).  4 acts on qqq_gemm_w4a8_pergroup_f16scale on the prefill path only and exists
 * to be timed (the ablation of Sec. 4.5.2, Fig. 9): fp16 multiply, conventional round and
 * fp16->int16 conversion instructions, byte packing; two roundings, so it equals the default route
 * only where code*s is exact in fp16.  5 = the prefill kernels' biased integer route (byte-wise multiply
 * of code + 8, or of 7 - code for scales up to 18 under the symmetric-code promise, the constant taken out
 * through a pre-pass) wherever it applies, also on the
 * short launches where the automatic choice skips its pre-pass and converts with the fp16 FMA.  Returns the
 * previous value.
 */
int qqq_set_group_mode_override(int mode);

/*
 * Tuning/diagnostic knob (host state, not thread-safe) for the skinny kernel: channel tiles per
 * workgroup (1, 2 or 4), number of K slices, waves per workgroup (4, 8 or 16), load depth (1 =
 * shallow, 2 = deep batches of in-flight loads); 0 = automatic for each.  Values that do not fit
 * the shape are ignored.  Returns 0.
 */
int qqq_set_skinny_tuning(int channel_tiles, int k_slices, int waves, int depth);

/*
 * Tuning/diagnostic knob (host state, not thread-safe) for the prefill path: 0 = automatic;
 * 10 = the DMA-ring kernel, one workgroup per tile, 128x512 tile on 8 waves; 15, 16, 17 = the same
 * kernel with the narrow tiles meant for mid-size M: 128x256 on 8 waves, 128x128 on 4 waves,
 * 64x128 on 4 waves (its ring depth by the launch's workgroup count: six stages when there is at most one
 * workgroup per CU, else three); 27 = 64x128 with the six-stage ring, 37 = with the three-stage ring; 13 = the persistent DMA-ring kernel (128x512 tiles, one workgroup per CU).
 * Other values act like 0.  Returns 0.
 */
int qqq_set_prefill_tuning(int tune);

/*
 * Tuning/diagnostic knob (host state, not thread-safe): number of K splits of the per-tile prefill
 * kernel for 16 < M <= 512 (each tile's K range is divided over that many workgroups, their raw
 * int32 tiles meet in the workspace and a second kernel sums and dequantises them); 0 = automatic,
 * 1 = never split.  Capped at 1024 / M and at K / 128; ignored without a workspace of the queried
 * size.  Negative values only query.  Returns the previous value.
 */
int qqq_set_prefill_ksplit(int k_splits);

#ifdef __cplusplus
}
#endif
#endif /* QQQ_TUNING_H_ */
