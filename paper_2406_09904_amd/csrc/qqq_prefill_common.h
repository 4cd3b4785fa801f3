// Pieces shared by the DMA-ring prefill kernels: operand conversion and tile-shape constants.
#pragma once

#include "qqq_internal.h"

namespace qqq {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int MODE>
__device__ __forceinline__ v4i convert_b(uint32_t d0, uint32_t d1, int sg) {
  int o[4];
  if constexpr (MODE == kPerChannel) {
    unpack_x16(d0, o[0], o[1]);
    unpack_x16(d1, o[2], o[3]);
  } else if constexpr (MODE == kGroupClamp) {
    const _Float16 hs = (_Float16)(float)sg;
    const h2 s2 = {hs, hs};
    unpack_group_clamp(d0, s2, o[0], o[1]);
    unpack_group_clamp(d1, s2, o[2], o[3]);
  } else if constexpr (is_bias_mode(MODE)) {
    const uint32_t s2 = (uint32_t)sg | ((uint32_t)sg << 16);
    unpack_group_bias<MODE == kGroupBiasWide>(d0, s2, o[0], o[1]);
    unpack_group_bias<MODE == kGroupBiasWide>(d1, s2, o[2], o[3]);
  } else if constexpr (MODE == kGroupReal || MODE == kGroupCvt) {
    // sg carries the fp16 bit pattern of the fused scale
    const h2 s2 = as_h2((uint32_t)sg | ((uint32_t)sg << 16));
    if constexpr (MODE == kGroupReal) {
      unpack_group_real(d0, s2, o[0], o[1]);
      unpack_group_real(d1, s2, o[2], o[3]);
    } else {
      unpack_group_cvt(d0, s2, o[0], o[1]);
      unpack_group_cvt(d1, s2, o[2], o[3]);
    }
  } else {
    const GroupFusedConsts g = make_group_fused(sg);
    unpack_group_fused(d0, g, o[0], o[1]);
    unpack_group_fused(d1, g, o[2], o[3]);
  }
  return (v4i){o[0], o[1], o[2], o[3]};
}

template <int MT, int CT, int NW, int ST = 3>
struct DmaShape {
  static constexpr int kBM = 32 * MT, kBN = NW * 32 * CT, kBK = 128, kStages = ST;
  static constexpr int kAStage = kBM * kBK;           // activations of one k-step
  static constexpr int kWWave = CT * 2048;            // packed codes of one wave and k-step
  static constexpr int kWStage = NW * kWWave;
  static constexpr int kSgStage = NW * 256;           // 256 B of group scales per wave (32*CT used)
  static constexpr int kStage = kAStage + kWStage + kSgStage;
  static constexpr int kAPieces = kBM / (8 * NW);     // 1 KiB DMA pieces (8 rows) per wave
  static constexpr int kWChunks = 2 * CT;             // 1 KiB DMA chunks (16 channels) per wave
  static constexpr int kEpRow = 64 * CT + 16;         // fp16 row of the epilogue patch + bank pad
  static constexpr int kEpWave = kBM * kEpRow;
  static constexpr int kLds = kStages * kStage;
  static_assert(kBM % (8 * NW) == 0, "activation rows must split evenly over the waves");
  static_assert(NW * kEpWave + kBM * 4 <= kLds, "epilogue staging must fit the ring");
  static_assert(kLds <= 160 * 1024, "ring must fit the 160 KiB LDS");
};

}  // namespace qqq
