// Pieces shared by the two matrix-core attention kernels (decode: mfma_attention.hip, partial prefill:
// prefill_attention.hip): operand types, the e4m3 -> bf16 conversion, and the permutation of the head dimension that
// lets K go from memory straight into the MFMA A operand.
#pragma once
#include "device_common.h"

namespace psdev {

constexpr int kHeadDim = 128;     // the matrix-core kernels are built for d = 128
constexpr int kTileTokens = 32;   // tokens per tile: two 16-token blocks
// log2 units a score may run ahead of a row's softmax reference before the reference moves and the accumulators
// are rescaled (probabilities then stay below 2^kLazyRescale instead of below 1)
constexpr float kLazyRescale = 8.f;
// cache-policy operand of a buffer load: bit 1 = nt, the line is not expected to be read again
constexpr int kNonTemporal = 2;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// two e4m3 codes (bytes 2*half, 2*half+1 of w) -> two bf16 in one register (exact): one
// v_cvt_scalef32_pk_bf16_fp8 with scale 1 (the instruction applies only the scale's exponent, so the real
// per-block scales are applied to the scores and probabilities instead)
__device__ __forceinline__ uint32_t e4m3x2_to_bf16x2(uint32_t w, bool hi) {
  const bf16x2 b = hi ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true)
                      : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ u32x4 e4m3x8_to_bf16x8(uint32_t lo, uint32_t hi) {
  u32x4 r;
  r.x = e4m3x2_to_bf16x2(lo, false);
  r.y = e4m3x2_to_bf16x2(lo, true);
  r.z = e4m3x2_to_bf16x2(hi, false);
  r.w = e4m3x2_to_bf16x2(hi, true);
  return r;
}

// Largest of the four scores of a block.  The fold starts from the constant -inf, which lets the compiler emit two
// three-input maxima and nothing else (a two-input float maximum first quiets its inputs, one instruction each).
__device__ __forceinline__ float max_of4(f32x4 s) {
  const float seed = -__builtin_inff();
  return fmaxf(fmaxf(fmaxf(fmaxf(seed, s[0]), s[1]), s[2]), s[3]);
}

// element offset of the 8 query values that meet K's k-step `step` in lane group kg: K rows are fetched 16 bytes per
// lane (8 bf16, or 16 e4m3 codes = two k-steps), so the contraction index is permuted, identically in K and Q
template <int KVT>
__device__ __forceinline__ int q_chunk_elem(int step, int kg) {
  if constexpr (KVT == PS_BF16) return 32 * step + 8 * kg;
  return 64 * (step >> 1) + 16 * kg + 8 * (step & 1);
}

}  // namespace psdev
