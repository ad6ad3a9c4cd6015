// Pieces shared by the two scan variants (scan.hip: two passes over K; scan_fused.hip: one).
#pragma once

#include "common.h"

namespace skipkv {

constexpr float kScale2 = 0.08838834764831845f * 1.4426950408889634f;  // log2(e) / sqrt(128)
constexpr float kRescaleSlack = 16.f;  // a lane's reference is refreshed when a logit exceeds it by this much (log2 units)

template <int DT>
struct Tr;
template <>
struct Tr<SKIPKV_BF16> {
  static constexpr int ESZ = 2, ROWB = 256, LSTR = 272;  // LDS row stride: +16 B so that 16-byte reads of 8 consecutive rows hit distinct banks
};
template <>
struct Tr<SKIPKV_F32> {
  static constexpr int ESZ = 4, ROWB = 512, LSTR = 528;
};

// acc[T] += Q[16T.., :] * K[token, :]^T for the lane's token.  Both operands use the same
// (arbitrary but identical) assignment of head-dim slices to MFMA k-steps: lane group g covers
// bytes [64g, 64g+64) of a bf16 row over the 4 k-steps, so every lane reads contiguous 16-byte
// pieces.
template <int DT, int NT>
__device__ __forceinline__ void tile_logits(const char *qt, const char *krow, int c16, int g, f32x4 (&acc)[NT]) {
  constexpr int LSTR = Tr<DT>::LSTR;
  if constexpr (DT == SKIPKV_BF16) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const bf16x8 bfrag = *reinterpret_cast<const bf16x8 *>(krow + g * 64 + kk * 16);
#pragma unroll
      for (int T = 0; T < NT; ++T) {
        const bf16x8 afrag = *reinterpret_cast<const bf16x8 *>(qt + (16 * T + c16) * LSTR + g * 64 + kk * 16);
        acc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, acc[T], 0, 0, 0);
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float4 bfrag = *reinterpret_cast<const float4 *>(krow + c * 64 + g * 16);
#pragma unroll
      for (int T = 0; T < NT; ++T) {
        const float4 afrag = *reinterpret_cast<const float4 *>(qt + (16 * T + c16) * LSTR + c * 64 + g * 16);
        acc[T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.x, bfrag.x, acc[T], 0, 0, 0);
        acc[T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.y, bfrag.y, acc[T], 0, 0, 0);
        acc[T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.z, bfrag.z, acc[T], 0, 0, 0);
        acc[T] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag.w, bfrag.w, acc[T], 0, 0, 0);
      }
    }
  }
}

}  // namespace skipkv
