// C-ABI entry points of libqqq: argument validation and kernel-family dispatch (host code only).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "qqq_internal.h"

namespace qqq {

static thread_local char g_err[256] = "no error";
static thread_local char g_route[256] = "";
static int g_override = 0;
static int g_group_mode = 0;
static int g_fuse_quant = 1;

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// the kernels a call enqueued, for qqq_last_route(): launchers append, entry points reset
void route_reset() { g_route[0] = 0; }
void route_note(const char* fmt, ...) {
  const size_t used = strlen(g_route);
  if (used + 4 >= sizeof(g_route)) return;
  size_t at = used;
  if (used > 0) at += (size_t)snprintf(g_route + used, sizeof(g_route) - used, " + ");
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_route + at, sizeof(g_route) - at, fmt, ap);
  va_end(ap);
}

int num_cus() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

static int g_prefill_tune = 0;    // 0 = automatic, see qqq_set_prefill_tuning
static int g_prefill_ksplit = 0;  // 0 = automatic
void set_prefill_tuning(int tune) { g_prefill_tune = tune; }
int get_prefill_tuning() { return g_prefill_tune; }
// ring depth of the 4-wave per-tile shapes: 0 = by the launch's workgroup count, else forced
int get_prefill_ring_depth() {
  return g_prefill_tune == 27 ? 6 : g_prefill_tune == 37 ? 3 : 0;
}
void set_prefill_ksplit(int s) { g_prefill_ksplit = s; }
int get_prefill_ksplit() { return g_prefill_ksplit; }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static bool gemm_shape_ok(int64_t M, int64_t N, int64_t K) {
  return M >= 0 && M <= 0x7FFFFFFF && N >= 16 && N % 16 == 0 && N <= 0x7FFFFFF0 && K >= 128 &&
         K % 128 == 0 && K <= 131072;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// split-K slabs of the per-tile prefill kernel: up to kSplitRows rows of int32 partial sums in all
// (k_splits * M <= kSplitRows), for the row counts where a K split can pay
constexpr int64_t kSplitRows = 1024, kSplitMaxM = 512;
static size_t split_bytes(int64_t M, int64_t N) {
  return (M > kDecodeAlwaysMaxM && M <= kSplitMaxM) ? align256((size_t)kSplitRows * (size_t)N * 4) : 0;
}

// ---------------------------------------------------------------------------------------------
// Dispatch model: every fitted constant the automatic kernel choice uses, in one place.  All were
// measured on one MI355X with the kernels of this library on the benchmark's layer shapes
// (K x N = 4096 x 4096, 4096 x 11008, 5120 x 13824, 11008 x 4096, 8192 x 28672, 21760 x 8192),
// timing GEMM launches back to back from a HIP graph with the weights rotated through > 1 GiB:
//   tile[]        K swept at fixed M, N for each forced tile shape; the slope is the cost of one
//                 k-step (128 k) of one workgroup in microseconds, measured once with at most one
//                 workgroup per CU ("alone") and once with several times more tiles than CUs,
//                 divided by the tiles per CU ("saturated"); the intercept (~4 k-steps) is the
//                 ring fill plus the epilogue of a tile.
//   stream_tbs    what the weight stream of a launch reaches at best (plain-read probe, 35-117 MiB).
//   launch_us     one more kernel in the stream (empty-kernel spacing).
//   reduce_tbs    the K-split reduce kernel's traffic rate (splits * M * N int32 written and read).
//   margins       how much cheaper (modelled) an alternative must be before the large tile or the
//                 unsplit launch is given up: set so that on a 72-case grid no pick lost more than
//                 13 % against the best forced choice.
//   decode_*      time of the decode kernel for 17..64 rows: decode_base_us + c(M) * N*K/1e6 with
//                 c linear in M per channel-group width, the width being the launcher's own choice
//                 (fit over M = 17..64 on the six layers plus 8192 x 8192, 5120 x 5120).
//   pergroup_*    the per-group prefill GEMM relative to the per-channel one of the same shape, for
//                 its two clamp-free conversions: the biased integer route (a factor on the time
//                 plus its pre-pass launch and per-tile correction) and the fp16-FMA route (a larger
//                 factor, nothing else); fitted on ten shapes from M=64 to 1024, they cross where
//                 the per-channel GEMM takes about 33 us.
// A test times the automatic pick against every forced pick on a small grid (15 % bar).
struct TileCost { int shape, bm, bn; bool one_per_cu; double alone_us, saturated_us; };
static const struct DispatchModel {
  TileCost tile[4] = {{0, 128, 512, true, 1.15, 1.33}, {3, 128, 256, true, 0.71, 0.78},
                      {4, 128, 128, false, 0.63, 0.52}, {5, 64, 128, false, 0.39, 0.275}};
  double tile_fixed_ksteps = 4.0;
  double stream_tbs = 5.0;
  double launch_us = 2.4;
  double reduce_tbs = 3.0;
  double margin_split = 0.88, margin_leave_large_tile = 0.95;
  int min_ksteps_per_split = 4;
  double decode_base_us = 5.0;
  double decode_c64_lo[2] = {0.038, 0.0015}, decode_c64_hi[2] = {0.045, 0.0017};  // 64- and 128-channel groups: M <= 32, M > 32
  double decode_c32_lo[2] = {0.06, 0.0008}, decode_c32_hi[2] = {0.093, 0.0007};   // 32-channel groups
  double decode_c16_lo[2] = {0.04, 0.0031}, decode_c16_hi[2] = {0.12, 0.0023};    // 16-channel groups
  double prefill_wins_by = 0.92;             // the prefill path must be this much cheaper at 17..64 rows
  double pergroup_bias_factor = 1.13, pergroup_prepass_us = 7.5, pergroup_fma_factor = 1.36;
  double perchannel_extra_us = 2.5;
} kModel;

// Tile shape and K split of the per-tile prefill kernel from the model: few rows want many small
// tiles, many rows the large tile with the most reuse; when even the small tiles leave CUs idle and
// K is long, splitting K over several workgroups per tile pays for the second kernel that sums the
// raw tiles.  Shape 0 with one split means "the large tile": the caller then picks between the
// persistent kernel and the per-tile one.
struct PrefillPlan {
  int shape, k_splits;
  double us;  // modelled time of the per-channel GEMM
};
static double reduce_cost_us(int k_splits, int64_t M, int64_t N) {
  return kModel.launch_us + 8e-6 * (double)k_splits * (double)M * (double)N / kModel.reduce_tbs;
}
static PrefillPlan plan_prefill(int64_t M, int64_t N, int64_t K, bool can_split, int forced_split) {
  const int cus = num_cus();
  const int T = (int)(K / 128);
  const int splits[8] = {1, 2, 3, 4, 6, 8, 12, 16};
  PrefillPlan best = {0, 1, 0.0};
  for (int i = 0; i < 4; ++i) {
    const TileCost& c = kModel.tile[i];
    const int64_t tiles_c = ((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
    for (int j = 0; j < 8; ++j) {
      int ks = splits[j];
      if (forced_split > 0) {  // the knob: capped like the forced-shape route caps it
        ks = forced_split;
        if (ks > kSplitRows / M) ks = (int)(kSplitRows / M);
        if (ks > T) ks = T;
        if (ks < 1 || !can_split) ks = 1;
      } else if (ks > 1 && (!can_split || ks * M > kSplitRows || T / ks < kModel.min_ksteps_per_split)) {
        continue;
      }
      const int64_t wgs = tiles_c * ks;
      double per_step = c.alone_us;
      if (wgs > cus)  // whole rounds where only one workgroup fits a CU, a smooth load otherwise
        per_step = c.saturated_us * (c.one_per_cu ? (double)((wgs + cus - 1) / cus) : (double)wgs / cus);
      double cost = per_step * ((double)T / ks + kModel.tile_fixed_ksteps);
      const double stream_us = (double)N * (double)K * 0.5 / (kModel.stream_tbs * 1e6);
      if (cost < stream_us) cost = stream_us;
      if (ks > 1) cost += reduce_cost_us(ks, M, N);
      // leaving the large tile has to pay, and so has a split (its model is the coarser one)
      const bool first = (i == 0 && j == 0);
      const double margin = ks > 1 && best.k_splits == 1
                                ? kModel.margin_split
                                : (best.shape == 0 && best.k_splits == 1 ? kModel.margin_leave_large_tile : 1.0);
      if (first || cost < best.us * margin) best = {c.shape, ks, cost};
      if (forced_split > 0) break;
    }
  }
  return best;
}

// Modelled time of the clamp-free per-group prefill GEMM and which conversion gives it: the biased integer
// route pays a pre-pass launch, the fp16-FMA route more per k-step, so short launches take the latter.
static double pergroup_prefill_us(const PrefillPlan& plan, int64_t M, int64_t N, bool* bias_route) {
  const double reduce_us = plan.k_splits > 1 ? reduce_cost_us(plan.k_splits, M, N) : 0.0;
  const double core = plan.us - reduce_us;
  const double bias = core * kModel.pergroup_bias_factor + kModel.pergroup_prepass_us + reduce_us;
  const double fma = core * kModel.pergroup_fma_factor + reduce_us;
  if (bias_route) *bias_route = bias < fma;
  return bias < fma ? bias : fma;
}

// Kernel family of a call: 1 = decode (split-K) kernel, 2 = prefill kernels.  Up to 16 rows the
// decode kernel streams the weights at memory speed; beyond 64 it does not apply.  In between it
// re-reads the activations once per 32 or 64 channels and its time grows with M, while the prefill
// path's 64-row tiles do not care about M: the models decide.
static int kernel_family(int64_t M, int64_t N, int64_t K, bool pergroup) {
  if (g_override != 0) return g_override;
  if (M <= kDecodeAlwaysMaxM) return 1;
  if (M > kSkinnyMaxM) return 2;
  const double nk = (double)N * (double)K * 1e-6;
  const int nt = decode_channel_tiles(N, (int)((M + 15) / 16), true);  // the launcher's own rule
  const double* f = nt >= 4 ? (M <= 32 ? kModel.decode_c64_lo : kModel.decode_c64_hi)
                  : nt == 2 ? (M <= 32 ? kModel.decode_c32_lo : kModel.decode_c32_hi)
                            : (M <= 32 ? kModel.decode_c16_lo : kModel.decode_c16_hi);
  double c = f[0] + f[1] * (double)M;
  // 16-channel groups in more than one round of workgroups: the last round counts as a whole one
  const int64_t wgs = N / (16 * nt), cus = num_cus();
  if (nt == 1 && wgs > cus) c *= (double)((wgs + cus - 1) / cus) * (double)cus / (double)wgs;
  const double decode_us = kModel.decode_base_us + c * nk;
  const PrefillPlan plan = plan_prefill(M, N, K, true, g_prefill_ksplit);
  const double prefill_us = pergroup ? pergroup_prefill_us(plan, M, N, nullptr) : plan.us + kModel.perchannel_extra_us;
  return prefill_us < kModel.prefill_wins_by * decode_us ? 2 : 1;
}

// per-group conversion route from the caller's promises about the group scales (and the codes)
static int group_mode(int sg_arg, int64_t M, int64_t N, int64_t K) {
  const bool symmetric = (sg_arg & QQQ_SG_SYMMETRIC_CODES) != 0;  // no code is -8
  const int sg_max = sg_arg & ~QQQ_SG_SYMMETRIC_CODES;
  int mode = kGroupClamp;
  const bool decode = kernel_family(M, N, K, true) == 1;
  if (sg_max >= 1 && sg_max <= 16) mode = decode ? kGroupLinear : kGroupFused;
  else if (symmetric && sg_max >= 17 && sg_max <= 18) mode = decode ? kGroupLinear : kGroupFusedWide;
  // (knob 3 asks for the fp16-FMA conversion: with scales of 17 and 18 that is its wide form)
  if (g_group_mode >= 1 && g_group_mode <= 3) mode = (g_group_mode == 3 && mode == kGroupFusedWide) ? mode : g_group_mode;
  return mode;
}

static bool sg_arg_ok(int sg_arg) {
  const int sg_max = sg_arg & ~QQQ_SG_SYMMETRIC_CODES;
  return sg_arg >= 0 && sg_max <= 127;
}

static size_t ws_rows(int64_t M) { return (size_t)(M < kSkinnyMaxM ? M : kSkinnyMaxM); }
// pre-pass buffers of the biased per-group route (prefill only): Rl, Rh [M][Gp], Bc [N][Gp]
static size_t bias_rows_bytes(int64_t M, int64_t K) {
  return M > kDecodeAlwaysMaxM ? align256((size_t)M * (size_t)(((K / 128) + 31) & ~31)) : 0;
}
static size_t bias_cols_bytes(int64_t M, int64_t N, int64_t K) {
  return M > kDecodeAlwaysMaxM ? align256((size_t)N * (size_t)(((K / 128) + 31) & ~31)) : 0;
}
static size_t ws_counter_bytes(int64_t N) { return ((size_t)(N / 16) * 4 + 255) & ~(size_t)255; }

static void bias_buffers(void* workspace, int64_t M, int64_t N, int64_t K, int8_t*& r_lo, int8_t*& r_hi,
                         int8_t*& bc) {
  char* base = (char*)workspace + ws_counter_bytes(N) + align256(ws_rows(M) * (size_t)N * 4);
  r_lo = (int8_t*)base;
  r_hi = (int8_t*)(base + bias_rows_bytes(M, K));
  bc = (int8_t*)(base + 2 * bias_rows_bytes(M, K));
}

// does gemm_common take the biased per-group route for this call? (same conditions as in there)
static bool takes_bias_route(int mode, int64_t M, int64_t N, int64_t K);

// Everything a GEMM call checks on the host; runs before the first launch of a call, so that an
// error means nothing was enqueued.  `fused`: the decode kernel quantises fp16 rows itself and takes
// no a_q / s_a.  `ws_needed`: out, the bytes the chosen kernel family requires (0 = optional).
static int gemm_validate(const int8_t* a_q, const float* s_a, const void* w_packed, const int8_t* s_g,
                         const void* s_w, void* y, int64_t M, int64_t N, int64_t K, void* workspace,
                         size_t workspace_bytes, int mode, bool fused) {
  if (!gemm_shape_ok(M, N, K))
    return set_error(QQQ_ERR_SHAPE, "gemm: unsupported shape M=%lld N=%lld K=%lld (need N%%16==0, "
                     "K%%128==0, 128<=K<=131072)", (long long)M, (long long)N, (long long)K);
  if (M == 0) return QQQ_OK;
  if ((!fused && (!a_q || !s_a)) || !w_packed || !s_w || !y || (mode != kPerChannel && !s_g))
    return set_error(QQQ_ERR_NULL, "gemm: null pointer argument");
  if (!aligned16(a_q) || !aligned16(w_packed) || !aligned16(y) || !aligned16(workspace) ||
      (reinterpret_cast<uintptr_t>(s_a) & 3u) || (reinterpret_cast<uintptr_t>(s_w) & 3u) ||
      (reinterpret_cast<uintptr_t>(s_g) & 3u))
    return set_error(QQQ_ERR_SHAPE, "gemm: a_q, w_packed, y and workspace must be 16-byte aligned, "
                     "s_a, s_w and s_g 4-byte aligned");
  if (((M + 63) / 64) * ((N + 127) / 128) > 0x7FFFFFFF)
    return set_error(QQQ_ERR_SHAPE, "gemm: too many output tiles for one launch");
  const int family = kernel_family(M, N, K, mode != kPerChannel);
  if (family == 1 && M > kSkinnyMaxM)
    return set_error(QQQ_ERR_SHAPE, "gemm: skinny kernel forced but M=%lld > %d", (long long)M,
                     kSkinnyMaxM);
  if (fused && family != 1) return set_error(QQQ_ERR_SHAPE, "gemm: fused quantisation needs the decode kernel");
  if (family == 1) {
    const size_t need = qqq_gemm_workspace_bytes(M, N, K);
    if (!workspace) return set_error(QQQ_ERR_NULL, "gemm: workspace is NULL");
    if (workspace_bytes < need)
      return set_error(QQQ_ERR_WORKSPACE, "gemm: workspace %zu bytes < %zu needed", workspace_bytes,
                       need);
  }
  return QQQ_OK;
}

static int gemm_common(const int8_t* a_q, const float* s_a, const void* w_packed, const int8_t* s_g,
                       const void* s_w, void* y, int32_t* acc_out, int64_t M, int64_t N, int64_t K,
                       void* workspace, size_t workspace_bytes, void* stream, int mode,
                       const void* a_fp16 = nullptr, int64_t lda = 0, bool row_sums_ready = false) {
  const bool fused = a_fp16 != nullptr;  // the decode kernel quantises the rows itself
  {
    const int rc = gemm_validate(a_q, s_a, w_packed, s_g, s_w, y, M, N, K, workspace, workspace_bytes, mode, fused);
    if (rc != QQQ_OK || M == 0) return rc;
  }
  const int family = kernel_family(M, N, K, mode != kPerChannel);
  GemmParams p;
  p.a_q = a_q;
  p.s_a = s_a;
  p.w = (const uint4*)w_packed;
  p.s_g = s_g;
  p.s_w = (const _Float16*)s_w;
  p.y = (_Float16*)y;
  p.acc_out = acc_out;
  p.M = (int)M;
  p.N = (int)N;
  p.K = (int)K;
  p.T = (int)(K / 128);
  p.ws_cnt = nullptr;
  p.ws_acc = nullptr;
  p.r_lo = p.r_hi = p.bias_w = nullptr;
  p.k_splits = 1;
  p.part = nullptr;
  p.a_fp16 = (const uint4*)a_fp16;
  p.lda_vec = lda / 8;
  if (family == 1) {
    p.ws_cnt = (int32_t*)workspace;
    p.ws_acc = (int32_t*)((char*)workspace + ws_counter_bytes(N));
    return launch_gemm_skinny(p, mode, (hipStream_t)stream);
  }
  const int64_t tiles = ((M + 127) / 128) * ((N + 511) / 512);
  const int tune = get_prefill_tuning();
  if (mode == kGroupCvt) return launch_gemm_prefill_dma(p, mode, 0, (hipStream_t)stream);
  // Clamp-free per-group request with a workspace of the queried size: the biased integer
  // conversion (a pre-pass computes the per-group row sums it needs) instead of the fp16 FMA one
  if (takes_bias_route(mode, M, N, K) && workspace && workspace_bytes >= qqq_gemm_workspace_bytes(M, N, K)) {
    int8_t *r_lo, *r_hi, *bc;
    bias_buffers(workspace, M, N, K, r_lo, r_hi, bc);
    // (scales up to 18 with symmetric codes: bytes of (7 - code) * s_g instead of (code + 8) * s_g)
    const bool wide = mode == kGroupFusedWide;
    const int rc = launch_group_bias_prepass(a_q, s_g, M, N, K, r_lo, r_hi, bc, !row_sums_ready, wide ? 7 : 8,
                                             (hipStream_t)stream);
    if (rc != QQQ_OK) return rc;
    p.r_lo = r_lo;
    p.r_hi = r_hi;
    p.bias_w = bc;
    mode = wide ? kGroupBiasWide : kGroupBias;
  }
  // per-tile kernel, optionally with K split over several workgroups per tile (raw tiles into the
  // workspace's slabs, then the reduce kernel); the split needs a workspace of the queried size
  const bool can_split = split_bytes(M, N) > 0 && workspace &&
                         workspace_bytes >= qqq_gemm_workspace_bytes(M, N, K);
  auto per_tile = [&](int shape, int k_splits) {
    const int64_t cap = kSplitRows / M;
    if (k_splits > cap) k_splits = (int)cap;
    if (k_splits > p.T) k_splits = p.T;
    if (!can_split || k_splits < 2) return launch_gemm_prefill_dma(p, mode, shape, (hipStream_t)stream);
    p.k_splits = k_splits;
    p.part = (int32_t*)((char*)workspace + ws_counter_bytes(N) + align256(ws_rows(M) * (size_t)N * 4) +
                        2 * bias_rows_bytes(M, K) + bias_cols_bytes(M, N, K));
    const int rc = launch_gemm_prefill_dma(p, mode, shape, (hipStream_t)stream);
    return rc != QQQ_OK ? rc : launch_splitk_reduce(p, mode, (hipStream_t)stream);
  };
  const int forced_split = get_prefill_ksplit();
  if (tune == 10 || (tune >= 15 && tune <= 17) || tune == 27 || tune == 37)
    return per_tile(tune >= 15 ? tune % 10 - 2 : 0, forced_split > 0 ? forced_split : 1);
  if (tune == 13) return launch_gemm_prefill_ring(p, mode, (hipStream_t)stream);
  {
    const PrefillPlan plan = plan_prefill(M, N, K, can_split, forced_split);
    if (plan.shape != 0 || plan.k_splits > 1) return per_tile(plan.shape, plan.k_splits);
    if (mode == kGroupReal) return launch_gemm_prefill_dma(p, mode, 0, (hipStream_t)stream);
    // Measured on MI355X (two boxes, 14 shapes with M >= 1024, both kernels in one process): with 64 k-steps
    // or more the per-tile kernel is 2-6 % ahead for the per-channel variant and 1-3 % for the per-group one
    // (K = 8192: 636 against 660 us on the 28672-channel layer; K = 21760: 455 against 483); with shorter K the
    // persistent kernel is level or up to 2 % ahead whenever a CU walks more than one tile (the next tile's
    // first k-steps load under the epilogue).
    const bool tiles_repeat = tiles > num_cus();
    if (p.T < 64 && (mode == kPerChannel || tiles_repeat))
      return launch_gemm_prefill_ring(p, mode, (hipStream_t)stream);
    return launch_gemm_prefill_dma(p, mode, 0, (hipStream_t)stream);
  }
}

static bool takes_bias_route(int mode, int64_t M, int64_t N, int64_t K) {
  // (the workspace holds the pre-pass buffers only above the rows that always take the decode kernel)
  if (!((mode == kGroupFused || mode == kGroupFusedWide) && M > kDecodeAlwaysMaxM &&
        (g_group_mode == 0 || g_group_mode == 5) &&
        kernel_family(M, N, K, true) == 2))
    return false;
  if (g_group_mode == 5) return true;  // forced
  bool bias = true;
  pergroup_prefill_us(plan_prefill(M, N, K, true, g_prefill_ksplit), M, N, &bias);
  return bias;
}

// One launch that quantises and multiplies.  Every workgroup quantises all M rows for itself, which a
// second launch (3.3-3.7 us) costs more than: always up to 8192 activations, up to 32768 with two or three
// rows, and with four rows on the large layers only (measured on five layers: M=2 0.8-2.5 us ahead everywhere,
// M=3 0.1-1.7 us; M=4 0.8 us ahead on 8192 x 28672, 0.2 us behind on the layers of 70 M weights and less).
static bool fused_ok(int64_t M, int64_t N, int64_t K) {
  if (!(g_override == 0 && g_fuse_quant && M >= 1 && M <= kFusedMaxM && M * K <= kFusedLdsBytes)) return false;
  return M * K <= kFusedLdsSmall || M <= 3 || (double)N * (double)K >= 1.5e8;
}

// quant_act followed by the GEMM; for a few decode rows a single launch that does both
static int linear_common(const void* a_fp16, int64_t lda, const void* w_packed, const int8_t* s_g,
                         const void* s_w, void* y, int32_t* acc_out, int64_t M, int64_t N, int64_t K,
                         void* workspace, size_t workspace_bytes, void* stream, int mode) {
  if (!gemm_shape_ok(M, N, K))
    return set_error(QQQ_ERR_SHAPE, "linear: unsupported shape M=%lld N=%lld K=%lld (need N%%16==0, "
                     "K%%128==0, 128<=K<=131072)", (long long)M, (long long)N, (long long)K);
  if (lda < K || lda % 8 != 0)
    return set_error(QQQ_ERR_SHAPE, "linear: lda=%lld must be >= K and a multiple of 8", (long long)lda);
  if (M == 0) return QQQ_OK;
  if (!a_fp16 || !workspace) return set_error(QQQ_ERR_NULL, "linear: null pointer argument");
  if (!aligned16(a_fp16) || !aligned16(workspace))
    return set_error(QQQ_ERR_SHAPE, "linear: a_fp16 and workspace must be 16-byte aligned");
  const size_t need = qqq_linear_workspace_bytes(M, N, K);
  if (workspace_bytes < need)
    return set_error(QQQ_ERR_WORKSPACE, "linear: workspace %zu bytes < %zu needed", workspace_bytes, need);
  const size_t gemm_ws = align256(qqq_gemm_workspace_bytes(M, N, K));
  if (fused_ok(M, N, K))
    return gemm_common(nullptr, nullptr, w_packed, s_g, s_w, y, acc_out, M, N, K, workspace, gemm_ws,
                       stream, mode, a_fp16, lda);
  float* s_a = (float*)((char*)workspace + gemm_ws);
  int8_t* a_q = (int8_t*)((char*)workspace + gemm_ws + align256((size_t)M * 4));
  {  // the GEMM's own checks, before the quantiser is enqueued: an error leaves nothing behind
    const int rc = gemm_validate(a_q, s_a, w_packed, s_g, s_w, y, M, N, K, workspace, gemm_ws, mode, false);
    if (rc != QQQ_OK) return rc;
  }
  // the per-group prefill GEMM's biased route wants per-group row sums of the codes: the quantiser
  // has them in registers, so it writes them on the way
  int8_t *r_lo = nullptr, *r_hi = nullptr, *bc = nullptr;
  const bool sums = takes_bias_route(mode, M, N, K);
  if (sums) bias_buffers(workspace, M, N, K, r_lo, r_hi, bc);
  const int rc = launch_quant_act(a_fp16, M, K, lda, a_q, s_a, (hipStream_t)stream, r_lo, r_hi);
  if (rc != QQQ_OK) return rc;
  return gemm_common(a_q, s_a, w_packed, s_g, s_w, y, acc_out, M, N, K, workspace, gemm_ws, stream, mode,
                     nullptr, 0, sums);
}

// ---- scratch of the entry point that allocates nothing: a device array that lives in the code
// object (one copy per GPU, held until the process ends).  Host code never uses the array's name as
// an address: the per-device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[QQQ_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[64] = {nullptr};
static std::mutex g_scratch_mu;

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
    return set_error(QQQ_ERR_HIP, "static scratch: no current device");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr)
      return set_error(QQQ_ERR_HIP, "static scratch: hipGetSymbolAddress: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return QQQ_OK;
}

// entries of an int8 group-scale table outside 0..sg_max, counted by one workgroup (a diagnostic:
// speed is beside the point, a single plain store of the total is)
__global__ __launch_bounds__(1024) void sg_violation_kernel(const uint32_t* s_g, int64_t words, int sg_max,
                                                            int32_t* out) {
  __shared__ int total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  int bad = 0;
  for (int64_t i = threadIdx.x; i < words; i += 1024) {
    const uint32_t w = s_g[i];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int v = (int)(int8_t)((w >> (8 * b)) & 0xFFu);
      bad += (v < 0 || v > sg_max) ? 1 : 0;
    }
  }
  if (bad) atomicAdd(&total, bad);
  __syncthreads();
  if (threadIdx.x == 0) *out = total;
}

// zero fill by a kernel (a memset node recorded into a captured graph is avoided on purpose)
__global__ __launch_bounds__(256) void zero_fill_kernel(uint4* p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
    p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace qqq

using namespace qqq;

extern "C" {

int qqq_version(void) { return 100; }

const char* qqq_last_error(void) { return g_err; }

const char* qqq_last_route(void) { return g_route; }

int qqq_debug_count_sg_violations(const int8_t* s_g, int64_t N, int64_t K, int sg_max, int32_t* violations,
                                  void* stream) {
  if (N < 4 || N % 4 != 0 || K < 128 || K % 128 != 0 || sg_max < 0 || sg_max > 127 || (K / 128) * N > 0x7FFFFFFFLL * 4)
    return set_error(QQQ_ERR_SHAPE, "count_sg_violations: unsupported N=%lld K=%lld sg_max=%d", (long long)N,
                     (long long)K, sg_max);
  if (!s_g || !violations) return set_error(QQQ_ERR_NULL, "count_sg_violations: null pointer argument");
  if ((reinterpret_cast<uintptr_t>(s_g) & 3u) || (reinterpret_cast<uintptr_t>(violations) & 3u))
    return set_error(QQQ_ERR_SHAPE, "count_sg_violations: pointers must be 4-byte aligned");
  const int64_t words = (K / 128) * N / 4;
  hipLaunchKernelGGL(sg_violation_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, (const uint32_t*)s_g, words,
                     sg_max, violations);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "count_sg_violations launch: %s", hipGetErrorString(e));
  return QQQ_OK;
}

int qqq_set_kernel_override(int family) {
  const int old = g_override;
  if (family >= 0 && family <= 2) g_override = family;
  return old;
}

int qqq_quant_act(const void* a_fp16, int64_t M, int64_t K, int64_t lda, int8_t* a_q, float* s_a,
                  void* stream) {
  route_reset();
  if (M < 0 || M > 0x7FFFFFFF || K < 8 || K % 8 != 0 || K > (1 << 24) || lda < K || lda % 8 != 0)
    return set_error(QQQ_ERR_SHAPE, "quant_act: unsupported M=%lld K=%lld lda=%lld (need K%%8==0, "
                     "lda%%8==0, lda>=K)", (long long)M, (long long)K, (long long)lda);
  if (M == 0) return QQQ_OK;
  if (!a_fp16 || !a_q || !s_a) return set_error(QQQ_ERR_NULL, "quant_act: null pointer argument");
  if (!aligned16(a_fp16) || (reinterpret_cast<uintptr_t>(a_q) & 7u))
    return set_error(QQQ_ERR_SHAPE, "quant_act: a_fp16 must be 16-byte and a_q 8-byte aligned");
  return launch_quant_act(a_fp16, M, K, lda, a_q, s_a, (hipStream_t)stream);
}

static int quantize_w4_check(const char* who, const void* w_fp16, int64_t N, int64_t K, int64_t ldw,
                             int64_t k_mult, const void* w_nat, const void* s_ch) {
  if (N < 0 || N > 0x7FFFFFFF || K < k_mult || K % k_mult != 0 || K > (1 << 24) || ldw < K || ldw % 8 != 0)
    return set_error(QQQ_ERR_SHAPE, "%s: unsupported N=%lld K=%lld ldw=%lld (need K%%%lld==0, ldw%%8==0, "
                     "ldw>=K)", who, (long long)N, (long long)K, (long long)ldw, (long long)k_mult);
  if (N == 0) return QQQ_OK;
  if (!w_fp16 || !w_nat || !s_ch) return set_error(QQQ_ERR_NULL, "%s: null pointer argument", who);
  if (!aligned16(w_fp16) || (reinterpret_cast<uintptr_t>(w_nat) & 3u) || (reinterpret_cast<uintptr_t>(s_ch) & 1u))
    return set_error(QQQ_ERR_SHAPE, "%s: w_fp16 must be 16-byte, w_nat 4-byte and the scales 2-byte aligned", who);
  return QQQ_OK;
}

int qqq_quantize_w4_perchannel(const void* w_fp16, int64_t N, int64_t K, int64_t ldw, uint32_t* w_nat,
                               void* s_w_fp16, void* stream) {
  const int rc = quantize_w4_check("quantize_w4_perchannel", w_fp16, N, K, ldw, 8, w_nat, s_w_fp16);
  if (rc != QQQ_OK || N == 0) return rc;
  return launch_quant_weight(w_fp16, N, K, ldw, false, w_nat, (uint16_t*)s_w_fp16, nullptr, nullptr, nullptr,
                             (hipStream_t)stream);
}

int qqq_quantize_w4_pergroup(const void* w_fp16, int64_t N, int64_t K, int64_t ldw, int group,
                             uint32_t* w_nat, void* s_star_fp16, int8_t* s_int, void* s_wc_fp16,
                             void* s_wg_fp16, void* stream) {
  if (group != QQQ_GROUP) return set_error(QQQ_ERR_SHAPE, "quantize_w4_pergroup: group must be %d", QQQ_GROUP);
  const int rc = quantize_w4_check("quantize_w4_pergroup", w_fp16, N, K, ldw, QQQ_GROUP, w_nat, s_wc_fp16);
  if (rc != QQQ_OK || N == 0) return rc;
  if (!s_star_fp16) return set_error(QQQ_ERR_NULL, "quantize_w4_pergroup: null s_star_fp16");
  if ((reinterpret_cast<uintptr_t>(s_star_fp16) & 1u) || (reinterpret_cast<uintptr_t>(s_wg_fp16) & 1u))
    return set_error(QQQ_ERR_SHAPE, "quantize_w4_pergroup: fp16 scale tables must be 2-byte aligned");
  return launch_quant_weight(w_fp16, N, K, ldw, true, w_nat, (uint16_t*)s_wc_fp16, (uint16_t*)s_wg_fp16,
                             (uint16_t*)s_star_fp16, s_int, (hipStream_t)stream);
}

int qqq_set_group_mode_override(int mode) {
  const int old = g_group_mode;
  if (mode >= 0 && mode <= 5) g_group_mode = mode;
  return old;
}

int qqq_set_skinny_tuning(int channel_tiles, int k_slices, int waves, int depth) {
  set_skinny_tuning(channel_tiles, k_slices, waves, depth);
  return 0;
}

int qqq_set_prefill_ksplit(int k_splits) {
  const int old = get_prefill_ksplit();
  if (k_splits >= 0) set_prefill_ksplit(k_splits);
  return old;
}

int qqq_set_prefill_tuning(int tune) {
  set_prefill_tuning(tune);
  return 0;
}


size_t qqq_packed_w4_bytes(int64_t N, int64_t K) {
  if (N < 16 || N % 16 != 0 || K < 128 || K % 128 != 0 || K > 131072 || N > 0x7FFFFFF0) return 0;
  return (size_t)N * (size_t)K / 2;
}

static int pack_common(const void* src, int64_t N, int64_t K, void* dst, bool inverse, void* stream) {
  if (qqq_packed_w4_bytes(N, K) == 0)
    return set_error(QQQ_ERR_SHAPE, "pack: unsupported N=%lld K=%lld (need N%%16==0, K%%128==0)",
                     (long long)N, (long long)K);
  if (!src || !dst) return set_error(QQQ_ERR_NULL, "pack: null pointer argument");
  if (src == dst) return set_error(QQQ_ERR_SHAPE, "pack: in-place repack is not supported");
  return launch_pack((const uint32_t*)src, N, K, (uint32_t*)dst, inverse, (hipStream_t)stream);
}

int qqq_pack_w4(const uint32_t* w_nat, int64_t N, int64_t K, void* w_packed, void* stream) {
  return pack_common(w_nat, N, K, w_packed, false, stream);
}

int qqq_unpack_w4(const void* w_packed, int64_t N, int64_t K, uint32_t* w_nat, void* stream) {
  return pack_common(w_packed, N, K, w_nat, true, stream);
}

size_t qqq_gemm_workspace_zero_bytes(int64_t M, int64_t N, int64_t K) {
  if (!gemm_shape_ok(M, N, K)) return 0;
  return ws_counter_bytes(N) + align256(ws_rows(M) * (size_t)N * 4);
}

size_t qqq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (!gemm_shape_ok(M, N, K)) return 0;
  return ws_counter_bytes(N) + align256(ws_rows(M) * (size_t)N * 4) + 2 * bias_rows_bytes(M, K) +
         bias_cols_bytes(M, N, K) + split_bytes(M, N);
}

int qqq_gemm_w4a8_perchannel(const int8_t* a_q, const float* s_a, const void* w_packed,
                             const void* s_w_fp16, void* y_fp16, int32_t* acc_out, int64_t M,
                             int64_t N, int64_t K, void* workspace, size_t workspace_bytes,
                             void* stream) {
  route_reset();
  return gemm_common(a_q, s_a, w_packed, nullptr, s_w_fp16, y_fp16, acc_out, M, N, K, workspace,
                     workspace_bytes, stream, kPerChannel);
}

int qqq_gemm_w4a8_pergroup(const int8_t* a_q, const float* s_a, const void* w_packed,
                           const int8_t* s_g, const void* s_w_fp16, int group, int sg_max,
                           void* y_fp16, int32_t* acc_out, int64_t M, int64_t N, int64_t K,
                           void* workspace, size_t workspace_bytes, void* stream) {
  route_reset();
  if (group != QQQ_GROUP) return set_error(QQQ_ERR_SHAPE, "pergroup: group must be 128, got %d", group);
  if (!sg_arg_ok(sg_max))
    return set_error(QQQ_ERR_SHAPE, "pergroup: sg_max must be in 0..127 (optionally or-ed with "
                     "QQQ_SG_SYMMETRIC_CODES), got %d", sg_max);
  return gemm_common(a_q, s_a, w_packed, s_g, s_w_fp16, y_fp16, acc_out, M, N, K, workspace,
                     workspace_bytes, stream, group_mode(sg_max, M, N, K));
}

int qqq_gemm_w4a8_pergroup_f16scale(const int8_t* a_q, const float* s_a, const void* w_packed,
                                    const void* s_g_fp16, const void* s_w_fp16, int group,
                                    void* y_fp16, int32_t* acc_out, int64_t M, int64_t N, int64_t K,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  route_reset();
  if (group != QQQ_GROUP) return set_error(QQQ_ERR_SHAPE, "pergroup: group must be 128, got %d", group);
  // knob 4: the conventional-conversion ablation of Fig. 9 (prefill kernel only)
  const int mode = (g_group_mode == 4 && kernel_family(M, N, K, true) == 2) ? kGroupCvt : kGroupReal;
  return gemm_common(a_q, s_a, w_packed, (const int8_t*)s_g_fp16, s_w_fp16, y_fp16, acc_out, M, N, K,
                     workspace, workspace_bytes, stream, mode);
}

size_t qqq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (!gemm_shape_ok(M, N, K)) return 0;
  return align256(qqq_gemm_workspace_bytes(M, N, K)) + align256((size_t)M * 4) + (size_t)M * (size_t)K;
}

int qqq_set_fused_quant(int enable) {
  const int old = g_fuse_quant;
  g_fuse_quant = enable ? 1 : 0;
  return old;
}

int qqq_linear_w4a8_perchannel(const void* a_fp16, int64_t lda, const void* w_packed,
                               const void* s_w_fp16, void* y_fp16, int32_t* acc_out, int64_t M,
                               int64_t N, int64_t K, void* workspace, size_t workspace_bytes,
                               void* stream) {
  route_reset();
  return linear_common(a_fp16, lda, w_packed, nullptr, s_w_fp16, y_fp16, acc_out, M, N, K, workspace,
                       workspace_bytes, stream, kPerChannel);
}

int qqq_linear_w4a8_pergroup(const void* a_fp16, int64_t lda, const void* w_packed, const int8_t* s_g,
                             const void* s_w_fp16, int group, int sg_max, void* y_fp16,
                             int32_t* acc_out, int64_t M, int64_t N, int64_t K, void* workspace,
                             size_t workspace_bytes, void* stream) {
  route_reset();
  if (group != QQQ_GROUP) return set_error(QQQ_ERR_SHAPE, "pergroup: group must be 128, got %d", group);
  if (!sg_arg_ok(sg_max))
    return set_error(QQQ_ERR_SHAPE, "pergroup: sg_max must be in 0..127 (optionally or-ed with "
                     "QQQ_SG_SYMMETRIC_CODES), got %d", sg_max);
  return linear_common(a_fp16, lda, w_packed, s_g, s_w_fp16, y_fp16, acc_out, M, N, K, workspace,
                       workspace_bytes, stream, group_mode(sg_max, M, N, K));
}

int qqq_linear_w4a8_perchannel_static(const void* a_fp16, int64_t lda, const void* w_packed,
                                      const void* s_w_fp16, void* y_fp16, int32_t* acc_out, int64_t M,
                                      int64_t N, int64_t K, void* stream) {
  route_reset();
  if (!gemm_shape_ok(M, N, K))
    return set_error(QQQ_ERR_SHAPE, "linear_static: unsupported shape M=%lld N=%lld K=%lld (need N%%16==0, "
                     "K%%128==0, 128<=K<=131072)", (long long)M, (long long)N, (long long)K);
  const size_t need = qqq_linear_workspace_bytes(M, N, K);
  if (need > (size_t)QQQ_STATIC_SCRATCH_BYTES)
    return set_error(QQQ_ERR_WORKSPACE, "linear_static: M=%lld N=%lld K=%lld needs %zu bytes of scratch, the "
                     "static scratch holds %zu; use qqq_linear_w4a8_perchannel with a workspace",
                     (long long)M, (long long)N, (long long)K, need, (size_t)QQQ_STATIC_SCRATCH_BYTES);
  if (M == 0) return QQQ_OK;
  // everything linear_common checks before its first launch, checked here before the fill below
  if (lda < K || lda % 8 != 0)
    return set_error(QQQ_ERR_SHAPE, "linear_static: lda=%lld must be >= K and a multiple of 8", (long long)lda);
  if (!a_fp16 || !w_packed || !s_w_fp16 || !y_fp16)
    return set_error(QQQ_ERR_NULL, "linear_static: null pointer argument");
  if (!aligned16(a_fp16) || !aligned16(w_packed) || !aligned16(y_fp16) ||
      (reinterpret_cast<uintptr_t>(s_w_fp16) & 3u))
    return set_error(QQQ_ERR_SHAPE, "linear_static: a_fp16, w_packed and y must be 16-byte aligned, s_w 4-byte");
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != QQQ_OK) return rc;
  // The array keeps the previous call's contents.  The decode kernel (M <= 64) wants its arrival
  // counters and split-K sums zero, and a previous call of another shape may have left other
  // scratch there: clear that part.  (Every call leaves its own such part zero, so the fill is
  // what protects against the OTHER parts of an earlier layout.)
  if (M <= kSkinnyMaxM) {
    const size_t n16 = (qqq_gemm_workspace_zero_bytes(M, N, K) + 15) / 16;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 1024 ? (n16 + 255) / 256 : 1024);
    hipLaunchKernelGGL(zero_fill_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)ws, n16);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "linear_static: fill launch: %s", hipGetErrorString(e));
  }
  return linear_common(a_fp16, lda, w_packed, nullptr, s_w_fp16, y_fp16, acc_out, M, N, K, ws, need, stream,
                       kPerChannel);
}

}  // extern "C"
