// Device-side helpers shared by the attention and merge kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ps_internal.h"

namespace psdev {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Everything a pass needs; passed by value to the kernels.
struct AttnParams {
  const int32_t* blk;        // block ids, prefix segments then suffix segments
  const int32_t* req_list;   // sharing groups, then the identity list
  const ps_item* items;
  const int32_t* slot_base;  // [R+1]
  const int32_t* visible;    // [R]: leading tokens of its prompt's prefix a request attends to
  const void* q;             // [R][Hq][d]
  const void* kv;
  const float* scales;       // [num_blocks][Hkv][2] or null
  float* ws_o;               // [num_slots][Hq][d]
  float* ws_lse;             // [num_slots][Hq]
  int32_t num_q_heads, num_kv_heads, group, block_size;
  int64_t s_block, s_head, s_kv, s_tok;  // elements
  float scale_log2;          // log2(e) / sqrt(d)
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// exp2 that maps (-inf) - (-inf) situations to 0 instead of NaN: callers pass the finite/neg-inf
// exponent difference computed with a guard.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Sum over the 16 lanes of a DPP row; every lane of the row receives the same bits.
__device__ __forceinline__ float row16_allreduce_sum(float x) {
  int v = __float_as_int(x);
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  v = __float_as_int(x);
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  v = __float_as_int(x);
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true));  // row_half_mirror
  v = __float_as_int(x);
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true));  // row_mirror
  return x;
}

__device__ __forceinline__ float lane_xor(float x, int mask) {
  const int lane = int(threadIdx.x) & 63;
  return __int_as_float(__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, __float_as_int(x)));
}

}  // namespace psdev
