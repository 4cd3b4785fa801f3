// Prefill W4A8 GEMM, main kernel family: three-stage LDS ring fed by global->LDS DMA loads
// (global_load_lds_dwordx4), int8 MFMA main loop (v_mfma_i32_16x16x64_i8 in the 8-wave shapes,
// v_mfma_i32_32x32x32_i8 in the 4-wave ones), one workgroup per output tile.
//
// Shape parameters: NW waves split N; each wave owns a (32*MT) x (32*CT) patch of Y, so the
// workgroup tile is (32*MT) x (NW*32*CT).  Instances:
//   <4,2,8>  128 x 512, 8 waves, 128 accumulator registers, two waves per SIMD
//   <4,1,8>  128 x 256, <4,1,4>  128 x 128, <2,1,4>  64 x 128: narrow tiles for mid-size M, where
//            a few large tiles would leave most CUs idle
//
// Why a DMA ring on gfx950.  The int8 MFMA pipe retires 32x32x32 (or two 16x16x64) multiply-accumulates
// in 32 clocks, so one k-step (128 k) is about a thousand clocks of MFMA per wave with the large wave
// patch; a global load that misses L2 takes
// several times that.  Registers cannot hold that much prefetch next to the accumulators, but the
// 160 KiB LDS can: every wave issues the DMA loads for k-step t+2 before it computes k-step t, the
// loads need no registers, and the only wait is "my DMA of k-step t+1 has landed" right before the
// workgroup barrier (s_waitcnt vmcnt(number of DMA loads per wave per k-step)).
//
// LDS stage (<= 50 KiB): activations (32*MT) rows x 128 B with the 16-byte slots of row r
// XOR-swizzled by (r/2)%8 (DMA writes lane-linear, so the swizzle is applied on the global side:
// lane l fetches slot l%8 ^ (row/2)%8).  The LDS of gfx950 serves a 128-bit read 16 lanes at a time
// over 64 banks: the 16 rows such a group reads must land in 16 different 16-byte bank groups, i.e.
// rows of equal parity need different slots, which (r/2)%8 gives and r%8 does not (rows r and r+8
// would collide: measured 125 instead of 240 bytes per clock and CU), then each wave's own 2*CT KiB
// of packed int4 codes exactly as they lie in memory, then (per-group variant) each wave's 32*CT
// group scales of the k-step.
// Weights never cross waves: each wave converts its codes to int8 once per k-step (Sec. 3.3.1 /
// 3.3.2 of the QQQ paper) and feeds one MFMA per row tile from every converted fragment.
#include "qqq_prefill_common.h"

// The DMA helpers below name M0 as clobbered (they rewrite it before every use).  M0 is a
// reserved register, which the compiler remarks on for any clobber list that names one.
#pragma clang diagnostic ignored "-Winline-asm"

namespace qqq {

template <int MODE, int MT, int CT, int NW, int ST>
__global__ __launch_bounds__(NW * 64, 1) void gemm_prefill_dma_kernel(const GemmParams p,
                                                                     const int tiles_m,
                                                                     const int tiles_n) {
  using S = DmaShape<MT, CT, NW, ST>;
  __shared__ __attribute__((aligned(1024))) int8_t lds[S::kLds];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int N = p.N, M = p.M;
  const int64_t K = p.K;
  const int ntiles = N >> 4;
  // split K: workgroup y of gridDim.y takes k-steps [t_first, t_first + T) of the tile
  const int split = blockIdx.y;
  const int t_first = (int)((int64_t)p.T * split / p.k_splits);
  const int T = (int)((int64_t)p.T * (split + 1) / p.k_splits) - t_first;

  // XCD-aware order: consecutive workgroup ids land on different XCDs (8 of them), so each XCD
  // gets a contiguous run of tiles; within a run tiles are walked in groups of 8 row tiles, m
  // fastest, so the workgroups resident on one XCD form a compact patch of Y and share their
  // activation and weight tiles through that XCD's L2.
  constexpr int kGroupM = 8;
  const int nblk = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8;
    if (per > 0 && pid < per * 8) pid = (pid % 8) * per + pid / 8;
  }
  const int width = kGroupM * tiles_n;
  const int first_m = (pid / width) * kGroupM;
  const int gsize = (tiles_m - first_m < kGroupM) ? tiles_m - first_m : kGroupM;
  const int tm = first_m + (pid % width) % gsize, tn = (pid % width) / gsize;
  const int m0 = tm * S::kBM;
  const int n_wave = tn * S::kBN + wave * 32 * CT;  // first channel of this wave

  // ---- DMA sources.  Activations: this wave copies rows 8*kAPieces*wave .. (1 KiB pieces of 8
  // rows); lane l lands in slot l%8 of row l/8, so it fetches chunk (l%8) ^ ((row/2)%8).  Rows past M
  // re-read row M-1 (never stored).  Weights: this wave's 1 KiB chunks, copied verbatim; chunks
  // past N/16 re-read the last valid chunk (never stored).
  // Addresses are a wave-uniform 64-bit base in scalar registers plus a 32-bit per-lane offset: the
  // per-k-step advance is then scalar arithmetic, not 64-bit vector adds on every lane.
  const uint32_t wave_u = (uint32_t)__builtin_amdgcn_readfirstlane(wave);
  uint32_t a_voff[S::kAPieces];
#pragma unroll
  for (int i = 0; i < S::kAPieces; ++i) {
    const int r = 8 * (S::kAPieces * wave + i) + (lane >> 3);
    int m = m0 + r;
    if (m > M - 1) m = M - 1;
    a_voff[i] = (uint32_t)(m - m0) * (uint32_t)K + (uint32_t)(((lane & 7) ^ ((r >> 1) & 7)) << 4);
  }
  const int8_t* a_base = p.a_q + (int64_t)m0 * K + (int64_t)t_first * S::kBK;
  const int64_t w_step = (int64_t)ntiles * 1024;  // bytes between k-steps of the packed weights
  const int8_t* w_base[S::kWChunks];
  const int nt0 = (tn * S::kBN + (int)wave_u * 32 * CT) >> 4;
#pragma unroll
  for (int j = 0; j < S::kWChunks; ++j) {
    int nt = nt0 + j;
    if (nt > ntiles - 1) nt = ntiles - 1;
    w_base[j] = (const int8_t*)p.w + (int64_t)nt * 1024 + (int64_t)t_first * w_step;
  }
  const uint32_t w_voff = (uint32_t)lane * 16u;
  // group scales of the wave's 32*CT channels: the first 8*CT lanes fetch 4 bytes each, the other
  // lanes (and channels past N) re-read a valid dword; each lane writes its own LDS dword
  // (fp16 scales of the real-valued variant: the first 16*CT lanes fetch two scales each)
  constexpr int kSgBytes = (MODE == kGroupReal || MODE == kGroupCvt) ? 2 : 1;  // bytes per group scale
  constexpr int kSgPerLane = 4 / kSgBytes, kSgLanes = 32 * CT / kSgPerLane;
  const int8_t* sg_src = nullptr;
  if constexpr (MODE != kPerChannel) {
    int c0 = n_wave + kSgPerLane * (lane < kSgLanes ? lane : kSgLanes - 1);
    if (c0 > N - kSgPerLane) c0 = N - kSgPerLane;
    sg_src = p.s_g + ((int64_t)t_first * N + c0) * kSgBytes;
  }

  // The DMA loads are issued through inline assembly so that the compiler's wait-count pass does
  // not know they write LDS (it would otherwise drain every outstanding load before the first LDS
  // read of each k-step); the waits are placed by hand below.  M0 carries the wave-uniform LDS
  // destination; lane l writes its 16 (or 4) bytes at M0 + 16*l (4*l).
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  auto dma16s = [&](const int8_t* base, uint32_t voff, uint32_t dst) {  // scalar base + lane offset
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(base)
                 : "memory", "m0");
  };
  auto dma4 = [&](const int8_t* src, uint32_t dst) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(dst), "v"(src)
                 : "memory", "m0");
  };
  // One DMA instruction of k-step t into `stage` (piece 0 .. kDmaPerStep-1): the k-loop spreads a
  // k-step's requests between its MFMAs (eight waves that issue everything at once right after a
  // barrier queue up behind one address unit, and a wave that waits there issues no MFMA either).
  auto issue_dma_piece = [&](int t, int stage, int piece) {
    const uint32_t base = lds_base + (uint32_t)stage * S::kStage;
    if (piece < S::kAPieces)
      dma16s(a_base + (int64_t)t * S::kBK, a_voff[piece], base + (S::kAPieces * wave_u + piece) * 1024);
    else if (piece < S::kAPieces + S::kWChunks)
      dma16s(w_base[piece - S::kAPieces] + (int64_t)t * w_step, w_voff,
             base + S::kAStage + wave_u * S::kWWave + (piece - S::kAPieces) * 1024);
    else if constexpr (MODE != kPerChannel)
      dma4(sg_src + (int64_t)t * N * kSgBytes, base + S::kAStage + S::kWStage + wave_u * 256);
  };
  auto issue_dma = [&](int t, int stage) {
#pragma unroll
    for (int piece = 0; piece < S::kAPieces + S::kWChunks + 1; ++piece) issue_dma_piece(t, stage, piece);
  };
  // DMA loads per wave per k-step
  constexpr int kDmaPerStep = S::kAPieces + S::kWChunks + (MODE != kPerChannel ? 1 : 0);
  // k-steps of DMA in flight behind the one the MFMAs are about to read (ring of ST stages: ST - 2)
  constexpr int kFlight = ST - 2;
  static_assert(kFlight * kDmaPerStep <= 48, "wait count must fit the vmcnt field with room to spare");
  // "everything but my newest k-steps of DMA has landed, my LDS reads are done", then the barrier
  auto wait_all_but_newest_step = [&]() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kFlight * kDmaPerStep) : "memory");
  };

  // ---- MFMA form and fragment layout.
  // 8-wave shapes: v_mfma_i32_16x16x64_i8.  Lane l holds row (or channel) l%16 and the 16 k-values
  // of k-block l/16, i.e. chunk 4*s + l/16 of the row in the k-sub s (64 k) of the k-step; register
  // i of a 16x16 result tile is row 4*(l/16) + i, column l%16.  Packed codes: lane l's 16-byte
  // vector of each of the wave's 16-channel chunks is exactly its operand data (dwords 0,1: k-sub
  // 0, dwords 2,3: k-sub 1).  This form moves half the accumulator bytes per multiply-accumulate
  // of the 32x32x32 form, which is worth 10-15 % at the board's power limit, where the large shapes
  // run; it issues twice the instructions, which two waves per SIMD absorb.
  // 4-wave shapes: v_mfma_i32_32x32x32_i8.  They serve launches that leave one wave per SIMD, where
  // the instruction issue of that one wave is the limit.  Lane l holds row (or channel) l%32 and
  // the 16 k-values of chunk 2*s + l/32 in MFMA step s (32 k); register v of a 32x32 result tile is
  // row 8*(v/4) + 4*(l/32) + v%4, column l%32.  Codes: tile c is chunks 2c and 2c+1; the lane's two
  // pieces are at (l%16 + 16*(l/32))*16 and +512 of chunk 2c + (l%32)/16.
  constexpr bool k32 = NW == 4;
  constexpr int kTile = k32 ? 32 : 16;                 // edge of a result tile
  constexpr int TM = S::kBM / kTile, TC = 32 * CT / kTile;  // result tiles per wave: TM x TC
  constexpr int kRegs = k32 ? 16 : 4;                  // accumulator registers per tile
  typedef int acc_t __attribute__((ext_vector_type(kRegs)));
  const int lcol = lane & (kTile - 1);                 // the lane's column (and fragment row) in a tile
  const int kblk = lane / kTile;                       // its k-block
  // row of accumulator register v of row tile mt, relative to the workgroup tile
  auto acc_row = [&](int mt, int v) { return mt * kTile + 8 * (v >> 2) + 4 * kblk + (v & 3); };
  constexpr int kSubs = k32 ? 4 : 2;                   // MFMA steps along k per k-step
  int a_off[kSubs];  // fragment of row lcol of row tile 0 (row tile mt adds kTile rows: same swizzle term)
#pragma unroll
  for (int s = 0; s < kSubs; ++s)
    a_off[s] = lcol * 128 + ((((k32 ? 2 : 4) * s + kblk) ^ ((lcol >> 1) & 7)) << 4);
  const int w_off = S::kAStage + wave * S::kWWave +
                    (k32 ? (lcol >> 4) * 1024 + ((lcol & 15) + 16 * kblk) * 16 : lane * 16);
  const int sg_off = S::kAStage + S::kWStage + wave * 256 + lcol * kSgBytes;

  int col[TC];
  bool nvalid[TC];
#pragma unroll
  for (int c = 0; c < TC; ++c) {
    col[c] = n_wave + c * kTile + lcol;
    nvalid[c] = col[c] < N;
  }
  acc_t acc[TM][TC];
#pragma unroll
  for (int mt = 0; mt < TM; ++mt)
#pragma unroll
    for (int c = 0; c < TC; ++c)
#pragma unroll
      for (int v = 0; v < kRegs; ++v) acc[mt][c][v] = 0;
  auto mfma = [&](const v4i a, const v4i b, acc_t& d) {
    if constexpr (k32) d = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, d, 0, 0, 0);
    else d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, d, 0, 0, 0);
  };

  // ---- prologue: k-steps 0 and 1 in flight, wait for step 0.  DMA requests past the last k-step
  // re-fetch the last one (in bounds, never read), which keeps every k-step's wait count the same.
#pragma unroll
  for (int s = 0; s < ST - 1; ++s) issue_dma(s < T ? s : T - 1, s);

  // ---- biased per-group route: the conversion adds the constant (8*s_g - 128) to every weight,
  // which sums to sum_g Bc[n][g] * R[m][g] over a row.  The pre-pass stored -R = 128*Rh + Rl, so
  // starting the accumulators at 128 x (Bc x Rh) + Bc x Rl takes it out in advance: a small int8
  // contraction over the groups with the main loop's operand roles (row operand from the
  // activations' side, column operand from the weights' side), every lane reading its 16 group
  // entries straight from memory while the first two k-steps of DMA are in flight.  Rows of the
  // tables are padded with zeros to a multiple of 32 groups; where an MFMA takes 64, k-blocks past
  // the padded row feed zeros.
  if (is_bias_mode(MODE) && split == 0) {  // the whole correction goes to the first K split
    // All operands of a pass are loaded before its MFMAs (TM + TC independent loads in flight): taken
    // one (row tile, channel tile) pair at a time, the load-then-MFMA chains of a tile ran one memory
    // latency after the other, 10-24 us per tile.
    const int Gp = (p.T + 31) & ~31;
    constexpr int kStep = k32 ? 32 : 64;
    const v4i zero = {0, 0, 0, 0};
    const int8_t* bp[TC];
    uint32_t roff[TM];
#pragma unroll
    for (int c = 0; c < TC; ++c) bp[c] = p.bias_w + (int64_t)(nvalid[c] ? col[c] : N - 1) * Gp + 16 * kblk;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      int mrow = m0 + kTile * mt + lcol;
      if (mrow > M - 1) mrow = M - 1;
      roff[mt] = (uint32_t)(mrow - m0) * (uint32_t)Gp + 16u * kblk;
    }
    const int8_t* hbase = p.r_hi + (int64_t)m0 * Gp;
    const int8_t* lbase = p.r_lo + (int64_t)m0 * Gp;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int8_t* rbase = pass ? lbase : hbase;
      for (int j = 0; j < Gp; j += kStep) {
        const bool in = j + 16 * kblk < Gp;
        v4i bw[TC], ar[TM];
#pragma unroll
        for (int c = 0; c < TC; ++c) bw[c] = in ? *(const v4i*)(bp[c] + j) : zero;
#pragma unroll
        for (int mt = 0; mt < TM; ++mt) ar[mt] = in ? *(const v4i*)(rbase + roff[mt] + j) : zero;
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
          for (int c = 0; c < TC; ++c) mfma(ar[mt], bw[c], acc[mt][c]);
      }
      if (pass == 0) {
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
          for (int c = 0; c < TC; ++c)
#pragma unroll
            for (int v = 0; v < kRegs; ++v)  // modular by design near the int32 limit: unsigned
              acc[mt][c][v] = (int)((uint32_t)acc[mt][c][v] << 7);
      }
    }
  }
  wait_all_but_newest_step();

  int stage = 0;
  if constexpr (!k32) {
    static_assert(ST == 3, "the slot schedule below is written for the three-stage ring");
    // ---- main loop, 16x16x64 form: a k-step is a fixed sequence of 2*TM slots (k-sub, row tile), TC
    // MFMAs each.  Fragments are read kAhead slots (about 200 clocks of MFMAs) before their MFMAs
    // into a rotating set of registers; the closing wait and barrier of the k-step sit before its
    // last kAhead slots, whose fragment reads already go to the next stage, so that LDS latency at
    // the k-step border hides behind MFMAs whose operands are in registers.  The DMA requests of
    // k-step t+2 go out one per slot.  The wave's own packed codes and group scales of k-step t+1
    // are read at mid-step, with no barrier (their DMA is this wave's own, issued a whole k-step
    // earlier), which spreads the conversions over the whole k-step: the second k-sub's tile c in
    // the first half, the next k-step's first k-sub's in the second half.  The compiler's scheduler
    // would pull the reads next to their uses; a scheduling barrier after every slot keeps the
    // order written here.
    constexpr int kSlots = 2 * TM, kAhead = TC >= 4 ? 3 : 6, kBufs = kAhead < 4 ? 4 : 8;
    constexpr int kCvtStride = (TM - 2) / (TC - 1);
    static_assert(kDmaPerStep <= TM && kAhead < TM && 1 + (TC - 1) * kCvtStride < TM, "k-step schedule does not fit");
    v4i wq[TC];  // this lane's packed codes of a k-step, one vector per channel tile
    int sg[TC];    // and its group scales
    auto read_w = [&](const int8_t* sb) {
#pragma unroll
      for (int c = 0; c < TC; ++c) {
        wq[c] = *(const v4i*)(sb + w_off + c * 1024);
        sg[c] = 0;
        if constexpr (MODE == kGroupReal || MODE == kGroupCvt)
          sg[c] = (int)*(const uint16_t*)(sb + sg_off + c * 32);
        else if constexpr (MODE != kPerChannel)
          sg[c] = (int)sb[sg_off + c * 16];
      }
    };
    // fragment of slot i = (k-sub i / TM, row tile i % TM)
    auto read_a = [&](const int8_t* sb, int slot) {
      return *(const v4i*)(sb + a_off[slot / TM] + (slot % TM) * 2048);
    };
    auto make_b = [&](int c, int s) {
      return s ? convert_b<MODE>((uint32_t)wq[c][2], (uint32_t)wq[c][3], sg[c])
             : convert_b<MODE>((uint32_t)wq[c][0], (uint32_t)wq[c][1], sg[c]);
    };
    v4i abuf[kBufs], b0[TC], b1[TC];
    read_w(lds);
#pragma unroll
    for (int i = 0; i < kAhead; ++i) abuf[i] = read_a(lds, i);
#pragma unroll
    for (int c = 0; c < TC; ++c) b0[c] = make_b(c, 0);
    for (int t = 0; t < T; ++t) {
      // k-step t+2 goes into the stage that was read during k-step t-1 (everyone is past the
      // barrier inside it)
      const int dt = t + 2 < T ? t + 2 : T - 1;
      const int dstage = stage == 0 ? 2 : stage - 1;
      const int nstage = stage == 2 ? 0 : stage + 1;
      const int8_t* sb = lds + stage * S::kStage;
      const int8_t* nb = lds + nstage * S::kStage;
#pragma unroll
      for (int i = 0; i < kSlots; ++i) {
        if (i == TM) {  // all of k-step t+2's requests are out: what else is in flight is older
          asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kDmaPerStep) : "memory");
          read_w(nb);
        }
        if (i == kSlots - kAhead) {
          // my DMA of k-step t+1 has landed (only the loads of k-step t+2 may still be in flight), my
          // LDS reads of this stage are done; then everyone's.  From here on the fragment reads go to
          // the next k-step's stage (stale data after the last k-step: read, never used).
          wait_all_but_newest_step();
        }
        abuf[(i + kAhead) % kBufs] = (i + kAhead < kSlots) ? read_a(sb, i + kAhead) : read_a(nb, i + kAhead - kSlots);
        if (i < kDmaPerStep) issue_dma_piece(dt, dstage, i);
#pragma unroll
        for (int c = 0; c < TC; ++c) {
          if (i == 1 + c * kCvtStride) b1[c] = make_b(c, 1);
          if (i == TM + 1 + c * kCvtStride) b0[c] = make_b(c, 0);  // of k-step t+1 (tile c's last use: slot TM-1)
        }
#pragma unroll
        for (int c = 0; c < TC; ++c) mfma(abuf[i % kBufs], i < TM ? b0[c] : b1[c], acc[i % TM][c]);
        __builtin_amdgcn_sched_barrier(0);
      }
      stage = nstage;
    }
  } else {
    // ---- main loop, 32x32x32 form, software-pipelined by hand and branch-free.  The activation
    // fragments of MFMA step s+1 are read from LDS while the MFMAs of step s run; the workgroup
    // barrier sits before the LAST MFMA step of a k-step (whose int8 operands are already
    // converted), so that the LDS reads of the next k-step (first activation fragments, the lane's
    // packed codes, its group scales) are in flight behind TM*TC MFMAs instead of stalling the pipe.
    v4i wq[TC][2];  // this lane's packed codes of the current k-step: [tile][piece]
    int sg[TC];       // and its group scales
    auto read_w = [&](const int8_t* sb) {
#pragma unroll
      for (int c = 0; c < TC; ++c) {
        wq[c][0] = *(const v4i*)(sb + w_off + c * 2048);
        wq[c][1] = *(const v4i*)(sb + w_off + c * 2048 + 512);
        sg[c] = 0;
        if constexpr (MODE == kGroupReal || MODE == kGroupCvt)
          sg[c] = (int)*(const uint16_t*)(sb + sg_off + c * 64);
        else if constexpr (MODE != kPerChannel)
          sg[c] = (int)sb[sg_off + c * 32];
      }
    };
    auto read_a = [&](v4i (&a)[TM], const int8_t* sb, int s) {
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) a[mt] = *(const v4i*)(sb + a_off[s] + mt * 4096);
    };
    // MFMA step s uses piece s%2, dword pair s/2 of the lane's packed codes
    auto make_b = [&](int c, int s) {
      const v4i pc = wq[c][s & 1];
      const uint32_t d0 = (uint32_t)((s >> 1) ? pc[2] : pc[0]), d1 = (uint32_t)((s >> 1) ? pc[3] : pc[1]);
      return convert_b<MODE>(d0, d1, sg[c]);
    };
    auto mfma_col = [&](const v4i (&a)[TM], const v4i b, int c) {
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) mfma(a[mt], b, acc[mt][c]);
    };
    auto mfma_step = [&](const v4i (&a)[TM], int s) {
#pragma unroll
      for (int c = 0; c < TC; ++c) mfma_col(a, make_b(c, s), c);
    };
    v4i a0[TM], a1[TM];
    read_w(lds);
    read_a(a0, lds, 0);
    for (int t = 0; t < T; ++t) {
      // k-step t+ST-1 goes into the stage that was read during k-step t-1 (everyone is past the
      // barrier inside it)
      issue_dma(t + ST - 1 < T ? t + ST - 1 : T - 1, stage == 0 ? ST - 1 : stage - 1);
      const int8_t* sb = lds + stage * S::kStage;
      read_a(a1, sb, 1);
      mfma_step(a0, 0);
      read_a(a0, sb, 2);
      mfma_step(a1, 1);
      read_a(a1, sb, 3);
      mfma_step(a0, 2);
      v4i b3[TC];
#pragma unroll
      for (int c = 0; c < TC; ++c) b3[c] = make_b(c, 3);
      // my DMA of k-step t+1 has landed (only the loads of the k-steps after it may still be in
      // flight), my LDS reads of this stage are done; then everyone's
      wait_all_but_newest_step();
      stage = (stage == ST - 1) ? 0 : stage + 1;
      // first LDS reads of k-step t+1 (stale data after the last k-step: read, never used) ...
      const int8_t* nb = lds + stage * S::kStage;
      read_a(a0, nb, 0);
      read_w(nb);
      // ... in flight behind the last MFMA step of k-step t
#pragma unroll
      for (int c = 0; c < TC; ++c) mfma_col(a1, b3[c], c);
    }
  }
  // the clamped DMA requests of the last two k-steps may still be landing in the ring
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- split K: the raw tile goes to this split's slab; the reduce kernel does the rest
  if (p.k_splits > 1) {
    int32_t* part = p.part + (int64_t)split * M * N;
#pragma unroll
    for (int c = 0; c < TC; ++c) {
      if (!nvalid[c]) continue;
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
#pragma unroll
        for (int v = 0; v < kRegs; ++v) {
          const int m = m0 + acc_row(mt, v);
          // (the wide biased route accumulates the negated sums)
          if (m < M) part[(int64_t)m * N + col[c]] = MODE == kGroupBiasWide ? (int)(0u - (uint32_t)acc[mt][c][v]) : acc[mt][c][v];
        }
      }
    }
    return;
  }

  // ---- fused Dequant epilogue.  Every four accumulator registers of a lane are four consecutive
  // rows of its column.  The ring is free now (nothing reads it after the last barrier and every
  // DMA has landed): each wave dequantises its patch into its own fp16 LDS region (row pitch padded
  // by 16 B) and streams it out as full rows.
  float* sa_lds = (float*)(lds + NW * S::kEpWave);
  for (int r = tid; r < S::kBM; r += NW * 64) sa_lds[r] = (m0 + r < M) ? p.s_a[m0 + r] : 0.0f;
  // Per-channel sums carry the factor 16 of the conversion.  Scaling by a power of two commutes with
  // every rounding of the Dequant (int -> fp32, fp32 product, fp16 result), so the factor goes into
  // the channel scale instead of a shift per accumulator.
  // The wide biased route's sums are negated: the sign goes the same way.
  constexpr float kAccScale = MODE == kPerChannel ? 0.0625f : (MODE == kGroupBiasWide ? -1.0f : 1.0f);
  float swv[TC];
#pragma unroll
  for (int c = 0; c < TC; ++c) swv[c] = nvalid[c] ? (float)p.s_w[col[c]] * kAccScale : 0.0f;
  __syncthreads();
  int8_t* ep = lds + wave * S::kEpWave;
#pragma unroll
  for (int mt = 0; mt < TM; ++mt) {
#pragma unroll
    for (int q = 0; q < kRegs / 4; ++q) {
      const int r0 = acc_row(mt, 4 * q);
      const float4 sa4 = *(const float4*)(sa_lds + r0);
      const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w};
#pragma unroll
      for (int c = 0; c < TC; ++c) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          *(_Float16*)(ep + (r0 + j) * S::kEpRow + (c * kTile + lcol) * 2) =
              dequant(acc[mt][c][4 * q + j], sav[j], swv[c]);
        }
      }
    }
  }
  // the patch is private to this wave and LDS serves one wave's accesses in order
  {
    constexpr int kLanesPerRow = 4 * CT;            // 16-byte pieces per patch row
    constexpr int kRowsPerIt = 64 / kLanesPerRow;
    const int cc = lane % kLanesPerRow;
    const int ncol = n_wave + cc * 8;
#pragma unroll
    for (int it = 0; it < S::kBM / kRowsPerIt; ++it) {
      const int row = it * kRowsPerIt + lane / kLanesPerRow;
      const v4i d = *(const v4i*)(ep + row * S::kEpRow + cc * 16);
      const int m = m0 + row;
      if (m < M && ncol < N) *(v4i*)(p.y + (int64_t)m * N + ncol) = d;
    }
  }
  if (p.acc_out) {  // parity/debug output of the true accumulators: plain stores
#pragma unroll
    for (int c = 0; c < TC; ++c) {
      if (!nvalid[c]) continue;
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
#pragma unroll
        for (int v = 0; v < kRegs; ++v) {
          const int m = m0 + acc_row(mt, v);
          if (m < M) {
            int x = acc[mt][c][v];
            if constexpr (MODE == kPerChannel) x >>= 4;
            if constexpr (MODE == kGroupBiasWide) x = (int)(0u - (uint32_t)x);  // modular, like the sums
            p.acc_out[(int64_t)m * N + col[c]] = x;
          }
        }
      }
    }
  }
}

template <int MODE, int MT, int CT, int NW, int ST = 3>
static int launch_dma(const GemmParams& p, hipStream_t st) {
  using S = DmaShape<MT, CT, NW, ST>;
  const int tiles_m = (p.M + S::kBM - 1) / S::kBM;
  const int tiles_n = (p.N + S::kBN - 1) / S::kBN;
  const int64_t grid = (int64_t)tiles_m * tiles_n;
  if (grid > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "prefill: grid too large");
  if (p.k_splits < 1 || p.k_splits > p.T || p.k_splits > 65535 || (p.k_splits > 1 && !p.part))
    return set_error(QQQ_ERR_SHAPE, "prefill: bad K split %d for %d k-steps", p.k_splits, p.T);
  hipLaunchKernelGGL((gemm_prefill_dma_kernel<MODE, MT, CT, NW, ST>), dim3((unsigned)grid, (unsigned)p.k_splits),
                     dim3(NW * 64), 0, st, p, tiles_m, tiles_n);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "prefill gemm launch: %s", hipGetErrorString(e));
  route_note("prefill per-tile tile=%dx%d waves=%d ring=%d ksplit=%d mode=%d grid=%lld", S::kBM, S::kBN, NW, ST,
             p.k_splits, MODE, (long long)grid);
  return QQQ_OK;
}

// Second kernel of a K-split launch: sums the splits' raw tiles and applies the Dequant epilogue
// (same arithmetic as the fused one).  Four consecutive channels per thread.
template <bool X16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmParams p) {
  const int64_t quads = (int64_t)p.M * (p.N >> 2);
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= quads) return;
  const int64_t slab = (int64_t)p.M * p.N;
  const int64_t at = q * 4;
  const int m = (int)(at / p.N), n = (int)(at % p.N);
  v4i sum = *(const v4i*)(p.part + at);
  for (int s = 1; s < p.k_splits; ++s) {
    const v4i x = *(const v4i*)(p.part + s * slab + at);
    sum += x;
  }
  if constexpr (X16) sum >>= 4;  // exact: the sum is a multiple of 16
  const float sa = p.s_a[m];
  const uint32_t* swp = (const uint32_t*)(p.s_w + n);  // s_w is 4-byte aligned, n a multiple of 4
  const uint32_t sw01 = swp[0], sw23 = swp[1];
  _Float16 o[4];
  o[0] = dequant(sum[0], sa, half_bits_to_float(sw01 & 0xFFFFu));
  o[1] = dequant(sum[1], sa, half_bits_to_float(sw01 >> 16));
  o[2] = dequant(sum[2], sa, half_bits_to_float(sw23 & 0xFFFFu));
  o[3] = dequant(sum[3], sa, half_bits_to_float(sw23 >> 16));
  *(uint2*)(p.y + at) = *(const uint2*)o;
  if (p.acc_out) *(v4i*)(p.acc_out + at) = sum;
}

int launch_splitk_reduce(const GemmParams& p, int mode, hipStream_t st) {
  const int64_t quads = (int64_t)p.M * (p.N >> 2);
  const dim3 grid((unsigned)((quads + 255) / 256)), block(256);
  if (mode == kPerChannel)
    hipLaunchKernelGGL((splitk_reduce_kernel<true>), grid, block, 0, st, p);
  else
    hipLaunchKernelGGL((splitk_reduce_kernel<false>), grid, block, 0, st, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "split-K reduce launch: %s", hipGetErrorString(e));
  route_note("k-split reduce");
  return QQQ_OK;
}

// The 64 x 128 shape comes with two ring depths.  Three stages leave room for three workgroups per
// CU, which hide each other's memory latency; when the launch has at most one workgroup per CU
// anyway, a six-stage ring (five k-steps of DMA in flight) hides it instead: 10-13 % on such launches
// (M=128, K=5120, N=13824: 19.8 -> 17.3 us), 25 % slower where three-stage workgroups would share CUs.
// (The 128 x 128 shape measured 2 % slower with six stages.)
static bool lone_workgroups(const GemmParams& p, int bm, int bn) {
  const int64_t wgs = (int64_t)((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn) * p.k_splits;
  const int deep = get_prefill_ring_depth();
  return deep == 0 ? wgs <= num_cus() : deep > 3;
}

template <int MODE>
static int launch_shape(const GemmParams& p, int shape, hipStream_t st) {
  switch (shape) {
    case 3: return launch_dma<MODE, 4, 1, 8>(p, st);
    case 4: return launch_dma<MODE, 4, 1, 4>(p, st);
    case 5: return lone_workgroups(p, 64, 128) ? launch_dma<MODE, 2, 1, 4, 6>(p, st) : launch_dma<MODE, 2, 1, 4>(p, st);
    default: return launch_dma<MODE, 4, 2, 8>(p, st);
  }
}

// shape: 0 = 128x512 tile with 8 waves; narrow tiles for shapes with few rows, where the number
// of workgroups matters more than the reuse inside one: 3 = 128x256 with 8 waves, 4 = 128x128
// with 4 waves, 5 = 64x128 with 4 waves
int launch_gemm_prefill_dma(const GemmParams& p, int mode, int shape, hipStream_t st) {
  switch (mode) {
    case kPerChannel: return launch_shape<kPerChannel>(p, shape, st);
    case kGroupClamp: return launch_shape<kGroupClamp>(p, shape, st);
    // applying the group scale to partial sums costs more VALU work than the MFMAs hide once
    // the tile has many rows, so both clamp-free requests use the per-weight fp16 FMA route here
    case kGroupLinear:
    case kGroupFusedWide:
    case kGroupFused: return launch_shape<kGroupFused>(p, shape, st);
    case kGroupReal: return launch_shape<kGroupReal>(p, shape, st);
    case kGroupCvt: return launch_dma<kGroupCvt, 4, 2, 8>(p, st);  // timing ablation: one shape
    case kGroupBias: return launch_shape<kGroupBias>(p, shape, st);
    case kGroupBiasWide: return launch_shape<kGroupBiasWide>(p, shape, st);
  }
  return set_error(QQQ_ERR_SHAPE, "unknown mode %d", mode);
}

}  // namespace qqq
