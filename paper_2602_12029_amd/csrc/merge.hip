// Log-sum-exp merge of partial attention states.
//
// For each (request, q head) the partial states (o_i, lse_i) of its prefix and suffix splits are
// combined as lse = log sum_i exp(lse_i), o = sum_i exp(lse_i - lse) o_i -- exact by softmax algebra
// over the concatenated cache [C_base ; own tokens] (Background Eq. 2).  One thread owns four
// consecutive head-dim elements of one row.
#include "device_common.h"
#include "launch.h"

namespace psdev {

template <int QT>
__global__ __launch_bounds__(256) void merge_states_kernel(const int32_t* __restrict__ slot_base,
                                                           const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_lse, void* __restrict__ out,
                                                           float* __restrict__ out_lse, int num_rows, int num_q_heads,
                                                           int head_dim) {
  const int per_row = head_dim >> 2;
  const int64_t gid = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t row = gid / per_row;
  if (row >= num_rows) return;
  const int c4 = int(gid % per_row);
  const int r = int(row / num_q_heads);
  const int h = int(row % num_q_heads);
  const int s0 = slot_base[r], s1 = slot_base[r + 1];
  const float neg_inf = -__builtin_inff();

  // Batches of up to four partial states: their lse and o loads all go out before anything is used, so a row with
  // at most four splits (the usual case: one or two prefix chunks and a suffix chunk) costs one memory round trip
  // after slot_base instead of one for the maxima and one for the values.  Across batches the running state
  // (mx, total, acc) is rescaled like an online softmax; a single batch is the plain two-pass formula.
  float mx = neg_inf, total = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int b0 = s0; b0 < s1; b0 += 4) {
    float lse[4];
    f32x4 o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lse[i] = neg_inf;                    // a slot past the end has weight zero and is not read
      o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (b0 + i < s1) {
        const int64_t s = b0 + i;
        lse[i] = ws_lse[s * num_q_heads + h];
        // the states are read once: non-temporal
        o[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(ws_o + (s * num_q_heads + h) * head_dim + 4 * c4));
      }
    }
    const float bm = fmaxf(fmaxf(fmaxf(lse[0], lse[1]), fmaxf(lse[2], lse[3])), mx);
    if (bm == neg_inf) continue;           // nothing but empty states so far
    const float keep = (mx == neg_inf) ? 0.f : fast_exp2((mx - bm) * kLog2e);
    total *= keep;
    acc *= keep;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (lse[i] != neg_inf) {             // an empty state has weight zero, whatever its o holds
        const float w = fast_exp2((lse[i] - bm) * kLog2e);
        total += w;
        acc += w * o[i];
      }
    }
    mx = bm;
  }
  if (mx != neg_inf) acc *= 1.f / total;
  if constexpr (QT == PS_F32) {
    *reinterpret_cast<f32x4*>(static_cast<float*>(out) + row * head_dim + 4 * c4) = acc;
  } else {
    bf16x2 lo, hi;
    lo.x = (__bf16)acc.x; lo.y = (__bf16)acc.y; hi.x = (__bf16)acc.z; hi.y = (__bf16)acc.w;
    uint2 packed;
    packed.x = __builtin_bit_cast(uint32_t, lo);
    packed.y = __builtin_bit_cast(uint32_t, hi);
    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(out) + row * head_dim + 4 * c4) = packed;
  }
  if (out_lse && c4 == 0) out_lse[row] = (mx != neg_inf) ? mx + __builtin_amdgcn_logf(total) * kLn2 : neg_inf;
}

int32_t launch_merge(const int32_t* slot_base, const float* ws_o, const float* ws_lse, void* out, float* out_lse,
                     int num_requests, const ps_geometry& g, hipStream_t st) {
  const int64_t rows = int64_t(num_requests) * g.num_q_heads;
  if (rows == 0) return PS_OK;
  if (g.head_dim % 4 != 0) return PS_ERR_UNSUPPORTED;
  const int64_t threads = rows * (g.head_dim / 4);
  const dim3 grid(unsigned((threads + 255) / 256)), block(256);
  if (g.q_dtype == PS_F32)
    hipLaunchKernelGGL((merge_states_kernel<PS_F32>), grid, block, 0, st, slot_base, ws_o, ws_lse, out, out_lse,
                       int(rows), g.num_q_heads, g.head_dim);
  else
    hipLaunchKernelGGL((merge_states_kernel<PS_BF16>), grid, block, 0, st, slot_base, ws_o, ws_lse, out, out_lse,
                       int(rows), g.num_q_heads, g.head_dim);
  return PS_OK;
}

}  // namespace psdev
