// Prefill W4A8 GEMM, persistent variant of the DMA-ring kernel: one workgroup per CU walks a
// list of 128 x 512 output tiles and the LDS ring keeps rotating across tile borders.
//
// Same k-step body as gemm_prefill_dma_kernel<.,4,2,8> (8 waves splitting N, 128 accumulator
// registers per lane, v_mfma_i32_16x16x64_i8, three 50 KiB LDS stages fed by global->LDS DMA two
// k-steps ahead).  What persistence buys: the DMA stream is a cursor over (tile, k-step) that runs
// two steps ahead of the MFMAs, so the first two k-steps of the NEXT tile are already in flight
// while the current tile finishes and is written out — the per-tile pipeline fill (an HBM
// round trip with one workgroup per CU) disappears, and the output stores of tile i drain under
// the MFMAs of tile i+1.
//
// Everything the k-loop and the epilogue need from global memory arrives by DMA (activations,
// packed codes, group scales per k-step; token scales and channel scales once per tile),
// so the loop contains no compiler-visible global load and the hand-placed s_waitcnt vmcnt(N)
// counts are exact: N = DMA loads per wave per k-step (+2 right after a tile's scale loads).
//
// Epilogue: the stage of the tile's last k-step is free until someone issues the DMA of the next
// tile's third k-step, which the closing barrier of the epilogue prevents; each wave dequantises
// 32 rows at a time into its own fp16 patch there and streams them out as 128-byte row segments.
#include "qqq_prefill_common.h"

// The DMA helpers below name M0 as clobbered (they rewrite it before every use).  M0 is a
// reserved register, which the compiler remarks on for any clobber list that names one.
#pragma clang diagnostic ignored "-Winline-asm"

namespace qqq {

template <int MODE>
__global__ __launch_bounds__(512, 1) void gemm_prefill_ring_kernel(const GemmParams p,
                                                                  const int tiles_m,
                                                                  const int tiles_n) {
  constexpr int kBM = 128, kBN = 512, kBK = 128;
  constexpr int kAStage = kBM * kBK;              // 16 KiB activations
  constexpr int kWWave = 4096, kWStage = 8 * kWWave;  // 4 KiB packed codes per wave
  constexpr int kSmall = kAStage + kWStage;       // per-wave 256 B of group scales (64 used)
  constexpr int kStage = kSmall + 8 * 256;        // 50 KiB
  constexpr int kSide = 8 * 512;                  // per tile parity, per wave: 256 B s_a, 256 B s_w
  constexpr int kEpRow = 144, kEpWave = 32 * kEpRow;  // epilogue patch: 32 rows per pass
  static_assert(8 * kEpWave <= kSmall, "epilogue patches must not reach the scale slots");
  __shared__ __attribute__((aligned(1024))) int8_t lds[3 * kStage];
  __shared__ __attribute__((aligned(256))) int8_t side[2 * kSide];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int T = p.T, N = p.N, M = p.M;
  const int64_t K = p.K;
  const int ntiles = N >> 4;
  const int nblk = tiles_m * tiles_n;
  const int my_tiles = (nblk - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;

  // XCD-aware tile order: consecutive workgroup ids sit on different XCDs (8 of them); the i-th
  // tile of workgroup b is virtual id b + i*grid, remapped so that each XCD owns one contiguous run
  // of tiles, walked in groups of 8 row tiles with m fastest: the tiles resident on one XCD at any
  // time form a compact patch of Y and share activation and weight tiles through that XCD's L2.
  auto tile_coords = [&](int iter, int& tm, int& tn) {
    int pid = (int)blockIdx.x + iter * (int)gridDim.x;
    const int per = nblk / 8;
    if (per > 0 && pid < per * 8) pid = (pid % 8) * per + pid / 8;
    constexpr int kGroupM = 8;
    const int width = kGroupM * tiles_n;
    const int first_m = (pid / width) * kGroupM;
    const int gsize = (tiles_m - first_m < kGroupM) ? tiles_m - first_m : kGroupM;
    tm = first_m + (pid % width) % gsize;
    tn = (pid % width) / gsize;
  };

  // ---- DMA side: a cursor (tile iteration d_iter, k-step d_t) that runs two k-steps ahead.
  // Per-lane source pointers of the cursor's position: two activation rows (1 KiB pieces of 8
  // rows; lane l lands in slot l%8 of row l/8 and fetches chunk (l%8)^((row/2)%8); rows past M re-read
  // row M-1), four 1 KiB weight chunks (chunks past N/16 re-read the last one) and a group-scale
  // dword (lanes past the wave's 64 channels, and channels past N, re-read a valid dword).  They
  // advance by constant strides per k-step and are rebuilt when the cursor enters a new tile,
  // which is also when the tile's token scales and channel scales are fetched, once, into a small
  // side buffer indexed by the tile's parity.
  int d_iter = 0, d_t = 0;
  // (activations and weights: a wave-uniform 64-bit base in scalar registers plus a 32-bit lane
  // offset, so the per-k-step advance is scalar arithmetic)
  const int8_t* a_base = nullptr;
  uint32_t a_voff[2] = {0, 0};
  const int8_t* w_base[4] = {nullptr, nullptr, nullptr, nullptr};
  const uint32_t w_voff = (uint32_t)lane * 16u;
  const int8_t* psg = nullptr;
  // slot swizzle: 16-byte chunk c of tile row r sits in slot c ^ ((r >> 1) & 7) of its 128-byte LDS row
  // (r = 16*wave + 8*i + lane/8 here, so (r >> 1) & 7 = (4*i + lane/16) & 7)
  const int swz[2] = {((lane & 7) ^ ((lane >> 4) & 7)) << 4, ((lane & 7) ^ ((4 + (lane >> 4)) & 7)) << 4};
  const int64_t w_step = (int64_t)ntiles * 1024;  // bytes between k-steps of the packed weights

  // DMA loads are issued through inline assembly so that the compiler's wait-count pass does not
  // know they write LDS (it would drain every outstanding load before the first LDS read of each
  // k-step); the waits are placed by hand.  M0 carries the wave-uniform LDS destination; lane l
  // writes its 16 (or 4) bytes at M0 + 16*l (4*l).
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  const uint32_t side_base = (uint32_t)(uintptr_t)(lds_ptr_t)side;
  const uint32_t wave_u = (uint32_t)__builtin_amdgcn_readfirstlane(wave);
  auto dma16s = [&](const int8_t* base, uint32_t voff, uint32_t dst) {  // scalar base + lane offset
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(base)
                 : "memory", "m0");
  };
  auto dma4 = [&](const int8_t* src, uint32_t dst) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(dst), "v"(src)
                 : "memory", "m0");
  };
  // (the tile order's integer divisions run on the vector unit; this brings a wave-uniform address
  // back to scalar registers, where the per-k-step advance then stays)
  auto to_scalar = [](const int8_t* ptr) {
    const uint64_t v = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const int8_t*)(uintptr_t)(((uint64_t)hi << 32) | lo);
  };
  // enters tile `iter`: rebuilds the pointers and fetches the tile's scales (two more DMA loads)
  auto enter_dma_tile = [&](int iter) {
    int tm, tn;
    tile_coords(iter, tm, tn);
    a_base = to_scalar(p.a_q + (int64_t)tm * kBM * K);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int m = tm * kBM + 16 * wave + 8 * i + (lane >> 3);
      if (m > M - 1) m = M - 1;
      a_voff[i] = (uint32_t)(m - tm * kBM) * (uint32_t)K + (uint32_t)swz[i];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int nt = tn * (kBN / 16) + (int)wave_u * 4 + j;
      if (nt > ntiles - 1) nt = ntiles - 1;
      w_base[j] = to_scalar((const int8_t*)p.w + (int64_t)nt * 1024);
    }
    const int c0 = tn * kBN + wave * 64;
    if constexpr (MODE != kPerChannel) {
      int c = c0 + 4 * (lane & 15);
      if (c > N - 4) c = N - 4;
      psg = p.s_g + c;
    }
    int row = tm * kBM + 16 * wave + (lane & 15);  // 16 token scales per wave (lanes repeat)
    if (row > M - 1) row = M - 1;
    int col = c0 + 2 * (lane & 31);                // 64 channel scales per wave, 2 per lane
    if (col > N - 2) col = N - 2;
    const uint32_t dst = side_base + (uint32_t)(iter & 1) * kSide + wave_u * 512;
    dma4((const int8_t*)(p.s_a + row), dst);
    dma4((const int8_t*)(p.s_w + col), dst + 256);
  };
  // The cursor's k-step goes into `stage` one DMA instruction at a time (piece 0..5, plus the group
  // scales), so that the k-loop can spread the requests between its MFMAs: eight waves that
  // issue all their requests at once right after a barrier queue up behind one address unit, and
  // a wave that waits there issues no MFMA either.
  auto issue_dma_piece = [&](int stage, int piece) {
    const uint32_t base = lds_base + (uint32_t)stage * kStage;
    if (piece < 2) dma16s(a_base, a_voff[piece], base + (2 * wave_u + piece) * 1024);
    else if (piece < 6) dma16s(w_base[piece - 2], w_voff, base + kAStage + wave_u * kWWave + (piece - 2) * 1024);
    else if constexpr (MODE != kPerChannel) dma4(psg, base + kSmall + wave_u * 256);
  };
  // advances the cursor after a k-step's pieces are out; returns true when the step was the last of
  // a tile and the next tile was entered (two more loads, the tile's scales, are then in flight).
  // Past the last tile the cursor keeps re-fetching the last k-step (in bounds, never read), so
  // wait counts never change.
  auto advance_cursor = [&]() {
    ++d_t;
    if (d_t < T) {
      a_base += kBK;
#pragma unroll
      for (int j = 0; j < 4; ++j) w_base[j] += w_step;
      if constexpr (MODE != kPerChannel) psg += N;
      return false;
    }
    if (d_iter + 1 < my_tiles) {
      d_t = 0;
      ++d_iter;
      enter_dma_tile(d_iter);
      return true;
    }
    d_t = T - 1;  // stay on the last k-step
    return false;
  };
  auto issue_next_dma = [&](int stage) {
#pragma unroll
    for (int piece = 0; piece < 7; ++piece) issue_dma_piece(stage, piece);
    return advance_cursor();
  };
  constexpr int kDmaPerStep = 6 + (MODE != kPerChannel ? 1 : 0);
  // "everything but my newest k-step of DMA has landed, my LDS reads are done", then the barrier;
  // `extra` = the newest k-step was followed by a tile's two scale loads
  auto wait_all_but_newest_step = [&](bool extra) {
    if (extra)
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kDmaPerStep + 2) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kDmaPerStep) : "memory");
  };

  // ---- per-lane LDS read offsets.  v_mfma_i32_16x16x64_i8: lane l holds row (or channel) l%16 and
  // the 16 k-values of k-block l/16, i.e. chunk 4*s + l/16 of the row in the k-sub s (64 k) of the
  // k-step; register i of a 16x16 result tile is row 4*(l/16) + i, column l%16.  A wave's 128 x 64
  // patch is 8 x 4 such tiles.  (The 16x16x64 form moves half the accumulator bytes per
  // multiply-accumulate of the 32x32x32 form; at the board's power limit, where this kernel runs,
  // that is worth 10-15 % of throughput.)
  const int r16 = lane & 15, kb = lane >> 4;
  int a_off[2];  // row r16 of row tile 0 (row tile mt adds 16 rows: the swizzle term does not change)
#pragma unroll
  for (int s = 0; s < 2; ++s) a_off[s] = r16 * 128 + (((4 * s + kb) ^ ((r16 >> 1) & 7)) << 4);
  // packed codes: lane l's 16-byte vector of each of the wave's four 16-channel chunks is exactly
  // its operand data: dwords 0,1 = the 16 k-values of k-block l/16 in k-sub 0, dwords 2,3 in k-sub 1
  const int w_off = kAStage + wave * kWWave + lane * 16;
  const int small_off = kSmall + wave * 256;

  v4i acc[8][4];
  v4i wq[4];  // this lane's packed codes of a k-step, one vector per channel tile
  int sg[4];    // and its group scales
  auto read_w = [&](const int8_t* sb) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wq[c] = *(const v4i*)(sb + w_off + c * 1024);
      sg[c] = 0;
      if constexpr (MODE != kPerChannel) sg[c] = (int)sb[small_off + c * 16 + r16];
    }
  };
  // fragment of slot i = (k-sub i/8, row tile i%8): 4 MFMAs use it
  auto read_a = [&](const int8_t* sb, int slot) {
    return *(const v4i*)(sb + a_off[slot >> 3] + (slot & 7) * 2048);
  };
  auto make_b = [&](int c, int s) {
    return s ? convert_b<MODE>((uint32_t)wq[c][2], (uint32_t)wq[c][3], sg[c])
             : convert_b<MODE>((uint32_t)wq[c][0], (uint32_t)wq[c][1], sg[c]);
  };

  // ---- prologue: k-steps 0 and 1 of the first tile in flight, wait for step 0
  enter_dma_tile(0);  // its two scale loads are older than everything below: always landed
  issue_next_dma(0);
  wait_all_but_newest_step(issue_next_dma(1));

  // The k-step is a fixed sequence of 16 slots (4 MFMAs each).  Fragments are read kAhead slots
  // before their MFMAs into a rotating set of four registers; the closing wait and barrier of the
  // k-step sit before the last kAhead slots, whose fragment reads (and the reads of the packed
  // codes) already go to the next stage, so that LDS latency at the k-step border hides behind MFMAs
  // whose operands are in registers.  The compiler's scheduler would pull these reads next to their
  // uses; a scheduling barrier after every slot keeps the order written here.
  constexpr int kAhead = 3;
  int stage = 0;
  v4i abuf[4], b0[4], b1[4];
  read_w(lds);
#pragma unroll
  for (int i = 0; i < kAhead; ++i) abuf[i] = read_a(lds, i);
  for (int it = 0; it < my_tiles; ++it) {
    int tm, tn;
    tile_coords(it, tm, tn);
    const int m0 = tm * kBM;
    const int n_wave = tn * kBN + wave * 64;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[mt][c] = (v4i){0, 0, 0, 0};
    // Biased per-group route: the conversion adds (8*s_g - 128) to every weight, which sums to
    // sum_g Bc[n][g] * R[m][g] over a row; the pre-pass stored -R = 128*Rh + Rl, so the tile starts
    // at 128 x (Bc x Rh) + Bc x Rl (see gemm_prefill_dma_kernel).  Ordinary loads: the compiler
    // waits for them before the MFMAs below, so none is outstanding at the k-loop's counted waits.
    // Rows of the tables are padded with zeros to a multiple of 32 groups; an MFMA takes 64, so
    // k-blocks past the padded row feed zeros.
    if constexpr (is_bias_mode(MODE)) {
      // The operands of a pass are loaded in batches ahead of their MFMAs (4-8 independent loads in flight): taken one
      // (row tile, channel tile) pair at a time, the 64 load-then-MFMA chains of a tile ran one memory
      // latency after the other, 10-24 us per tile.
      const int Gp = (T + 31) & ~31;
      const v4i zero = {0, 0, 0, 0};
      // offsets are recomputed where they are used: registers are scarce here (the next tile's
      // first fragments and operands are already held)
      const int nb0 = n_wave < N - 1 ? n_wave : N - 1;  // a wave past the ragged edge re-reads the last channel
      auto boff = [&](int c) {
        int col = n_wave + c * 16 + r16;
        if (col > N - 1) col = N - 1;
        return (uint32_t)(col - nb0) * (uint32_t)Gp + 16u * kb;
      };
      auto roff = [&](int mt) {
        int mrow = m0 + 16 * mt + r16;
        if (mrow > M - 1) mrow = M - 1;
        return (uint32_t)(mrow - m0) * (uint32_t)Gp + 16u * kb;
      };
      const int8_t* bbase = p.bias_w + (int64_t)nb0 * Gp;
      const int8_t* hbase = p.r_hi + (int64_t)m0 * Gp;
      const int8_t* lbase = p.r_lo + (int64_t)m0 * Gp;
#pragma unroll
      for (int pass = 0; pass < 2; ++pass) {
        const int8_t* rbase = pass ? lbase : hbase;
        for (int j = 0; j < Gp; j += 64) {
          const bool in = j + 16 * kb < Gp;
          v4i bw[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) bw[c] = in ? *(const v4i*)(bbase + boff(c) + j) : zero;
#pragma unroll
          for (int half = 0; half < 2; ++half) {  // four row tiles at a time: registers are scarce here
            v4i ar[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) ar[i] = in ? *(const v4i*)(rbase + roff(4 * half + i) + j) : zero;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int c = 0; c < 4; ++c)
                acc[4 * half + i][c] =
                    __builtin_amdgcn_mfma_i32_16x16x64_i8(ar[i], bw[c], acc[4 * half + i][c], 0, 0, 0);
          }
        }
        if (pass == 0) {
#pragma unroll
          for (int mt = 0; mt < 8; ++mt)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
              for (int v = 0; v < 4; ++v)  // modular by design near the int32 limit: unsigned
                acc[mt][c][v] = (int)((uint32_t)acc[mt][c][v] << 7);
        }
      }
    }

    for (int t = 0; t < T; ++t) {
      // the cursor's k-step (two ahead, possibly already in the next tile) goes into the stage
      // that was read during the previous k-step (everyone is past the barrier inside it)
      const int dstage = stage == 0 ? 2 : stage - 1;
      const int nstage = stage == 2 ? 0 : stage + 1;
      const int8_t* sb = lds + stage * kStage;
      const int8_t* nb = lds + nstage * kStage;
      // the first k-sub's operands, from the codes read after the previous k-step's barrier
#pragma unroll
      for (int c = 0; c < 4; ++c) b0[c] = make_b(c, 0);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (i == 16 - kAhead) {
          // my DMA of the next k-step has landed (only the loads of the one after may still be in
          // flight), my LDS reads of this stage are done; then everyone's.  From here on the reads
          // go to the next k-step's stage (after a tile's last k-step: the next tile's first;
          // after the very last: stale data, read but never used).
          wait_all_but_newest_step(advance_cursor());
          read_w(nb);
        }
        abuf[(i + kAhead) & 3] = (i + kAhead < 16) ? read_a(sb, i + kAhead) : read_a(nb, i + kAhead - 16);
        if (i < 7) issue_dma_piece(dstage, i);
        if (i >= 2 && i < 6) b1[i - 2] = make_b(i - 2, 1);  // the second k-sub's operands, one per slot
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc[i & 7][c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(abuf[i & 3], i < 8 ? b0[c] : b1[c], acc[i & 7][c], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      stage = nstage;
    }

    // ---- fused Dequant epilogue in the stage of the tile's last k-step, 32 rows (two row tiles)
    // per pass: lane holds rows 4*kb .. 4*kb+3 of column r16 of each 16-wide tile.
    {
      const int8_t* fsb = lds + (stage == 0 ? 2 : stage - 1) * kStage;
      int8_t* patch = const_cast<int8_t*>(fsb) + wave * kEpWave;
      const int8_t* sd = side + (it & 1) * kSide;  // this tile's scales: [wave][256 B s_a, 256 B s_w]
      // Per-channel sums carry the factor 16 of the conversion.  Scaling by a power of two commutes with
      // every rounding of the Dequant (int -> fp32, fp32 product, fp16 result), so the factor goes
      // into the channel scale instead of a shift per accumulator.
      // (the wide biased route's sums are negated: the sign goes the same way)
      constexpr float kAccScale = MODE == kPerChannel ? 0.0625f : (MODE == kGroupBiasWide ? -1.0f : 1.0f);
      float swv[4];
#pragma unroll
      for (int c = 0; c < 4; ++c)
        swv[c] = (float)*(const _Float16*)(sd + wave * 512 + 256 + (c * 16 + r16) * 2) * kAccScale;
      const int cc = lane & 7;
      const int ncol = n_wave + cc * 8;
#pragma unroll
      for (int pass = 0; pass < 4; ++pass) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int mt = 2 * pass + half;
          // token scales of rows 16*mt + 4*kb .. +3: wave mt's slot of the side buffer
          const float4 sa4 = *(const float4*)(sd + mt * 512 + kb * 16);
          const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              *(_Float16*)(patch + (16 * half + 4 * kb + j) * kEpRow + (c * 16 + r16) * 2) =
                  dequant(acc[mt][c][j], sav[j], swv[c]);
            }
          }
        }
        // the patch is private to this wave and LDS serves one wave's accesses in order
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const int row = i4 * 8 + (lane >> 3);
          const v4i d = *(const v4i*)(patch + row * kEpRow + cc * 16);
          const int m = m0 + pass * 32 + row;
          if (m < M && ncol < N) *(v4i*)(p.y + (int64_t)m * N + ncol) = d;
        }
      }
      if (p.acc_out) {  // parity/debug output of the true accumulators: plain stores
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int col = n_wave + c * 16 + r16;
          if (col >= N) continue;
#pragma unroll
          for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int m = m0 + mt * 16 + 4 * kb + v;
              if (m < M) {
                int x = acc[mt][c][v];
                if constexpr (MODE == kPerChannel) x >>= 4;
                if constexpr (MODE == kGroupBiasWide) x = (int)(0u - (uint32_t)x);  // modular, like the sums
                p.acc_out[(int64_t)m * N + col] = x;
              }
            }
          }
        }
      }
      // nobody may start the next tile (whose first DMA reuses this stage) before all are done
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
  }
  // the cursor's last requests may still be landing in the ring
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int MODE>
static int launch_ring(const GemmParams& p, hipStream_t st) {
  const int tiles_m = (p.M + 127) / 128;
  const int tiles_n = (p.N + 511) / 512;
  const int64_t tiles = (int64_t)tiles_m * tiles_n;
  if (tiles > 0x7FFFFFFF) return set_error(QQQ_ERR_SHAPE, "prefill: too many tiles");
  int64_t grid = num_cus();
  if (grid > tiles) grid = tiles;
  hipLaunchKernelGGL((gemm_prefill_ring_kernel<MODE>), dim3((unsigned)grid), dim3(512), 0, st, p,
                     tiles_m, tiles_n);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(QQQ_ERR_HIP, "prefill gemm launch: %s", hipGetErrorString(e));
  route_note("prefill persistent tile=128x512 mode=%d tiles=%lld grid=%lld", MODE, (long long)tiles,
             (long long)grid);
  return QQQ_OK;
}

int launch_gemm_prefill_ring(const GemmParams& p, int mode, hipStream_t st) {
  // With fewer than three k-steps per tile the DMA cursor would run more than one tile ahead and
  // overwrite the two-deep scale buffer before its tile is written out: use the per-tile kernel.
  if (p.T < 3) return launch_gemm_prefill_dma(p, mode, 0, st);
  switch (mode) {
    case kPerChannel: return launch_ring<kPerChannel>(p, st);
    case kGroupClamp: return launch_ring<kGroupClamp>(p, st);
    // applying the group scale to partial sums costs more VALU work than the MFMAs hide once
    // the tile has many rows, so both clamp-free requests use the per-weight fp16 FMA route here
    case kGroupLinear:
    case kGroupFusedWide:
    case kGroupFused: return launch_ring<kGroupFused>(p, st);
    case kGroupBias: return launch_ring<kGroupBias>(p, st);
    case kGroupBiasWide: return launch_ring<kGroupBiasWide>(p, st);
    // conversion routes this kernel does not carry
    case kGroupReal:
    case kGroupCvt: return launch_gemm_prefill_dma(p, mode, 0, st);
  }
  return set_error(QQQ_ERR_SHAPE, "unknown mode %d", mode);
}

}  // namespace qqq
