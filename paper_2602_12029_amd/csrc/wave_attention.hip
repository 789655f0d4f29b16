// fp32 wavefront-reduction split-K attention (no matrix cores).
//
// Used where the grouped query rows per KV head are too few or the inputs too wide for the bf16
// MFMA path: fp32 inputs, unusual head sizes, or on request.  One workgroup (4 waves) handles one
// work item: a token range of one KV segment for one KV head, applied to all query rows that read
// it.  A 16-lane row of a wave owns one token at a time: lane c of the row holds d/16 consecutive
// head-dim elements of that token's K and V, scores are completed with a DPP all-reduce over the
// row, and every 16-lane row keeps its own online-softmax state (running max, sum, weighted V).
// The 16 row states of the workgroup are merged at the end and written as one partial state.
#include "device_common.h"
#include "launch.h"

namespace psdev {


template <int KVT, int E>
__device__ __forceinline__ void load_elems(const void* base, int64_t elem_off, float (&out)[E]) {
  if constexpr (KVT == PS_F32) {
    const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + elem_off);
#pragma unroll
    for (int i = 0; i < E / 4; ++i) {
      const f32x4 v = p[i];
      out[4 * i + 0] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
    }
  } else if constexpr (KVT == PS_BF16) {
    const uint16_t* p16 = static_cast<const uint16_t*>(base) + elem_off;
    if constexpr (E % 8 == 0) {
      const uint4* p = reinterpret_cast<const uint4*>(p16);
#pragma unroll
      for (int i = 0; i < E / 8; ++i) {
        const uint4 v = p[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          out[8 * i + 2 * j] = __uint_as_float(w[j] << 16);
          out[8 * i + 2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
        }
      }
    } else {
      const uint2 v = *reinterpret_cast<const uint2*>(p16);
      out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
      out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
    }
  } else {  // e4m3fn codes
    const uint32_t* p = reinterpret_cast<const uint32_t*>(static_cast<const uint8_t*>(base) + elem_off);
#pragma unroll
    for (int i = 0; i < E / 4; ++i) {
      const uint32_t w = p[i];
      const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
      const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
      out[4 * i + 0] = lo.x; out[4 * i + 1] = lo.y; out[4 * i + 2] = hi.x; out[4 * i + 3] = hi.y;
    }
  }
}

template <int D, int KVT, int QT>
__global__ __launch_bounds__(256, D <= 64 ? 3 : 2) void wave_attention_kernel(AttnParams p, int item_begin) {
  constexpr int E = D / 16;
  constexpr int kRowTile = D <= 128 ? 8 : 4;  // query rows carried in registers per pass over the tokens
  __shared__ float sm_m[4][kRowTile];
  __shared__ float sm_l[4][kRowTile];
  __shared__ float sm_acc[4][kRowTile][D];

  const ps_item it = p.items[item_begin + blockIdx.x];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int dchunk = lane & 15;
  const int stream = wave * 4 + (lane >> 4);  // which of the 16 interleaved token streams
  const int G = p.group;
  const int rows = it.n_req * G;
  const float neg_inf = -__builtin_inff();

  for (int row0 = 0; row0 < rows; row0 += kRowTile) {
    float qreg[kRowTile][E];
    float m[kRowTile], l[kRowTile], acc[kRowTile][E];
    int lim[kRowTile];   // first token the row does not see (per-request visible prefix length, or the item's end)
#pragma unroll
    for (int rr = 0; rr < kRowTile; ++rr) {
      const int row = row0 + rr;
      m[rr] = neg_inf;
      l[rr] = 0.f;
      lim[rr] = it.tok_end;
#pragma unroll
      for (int e = 0; e < E; ++e) { acc[rr][e] = 0.f; qreg[rr][e] = 0.f; }
      if (row < rows) {
        const int req = p.req_list[it.req_off + row / G];
        if (it.kind & kPsItemMasked) lim[rr] = min(it.tok_end, p.visible[req]);
        const int h = it.kv_head * G + row % G;
        load_elems<QT, E>(p.q, (int64_t(req) * p.num_q_heads + h) * D + dchunk * E, qreg[rr]);
      }
    }

    // Token loop, two steps deep in flight: while token t is worked on, the K/V rows of token t + 16 are on their way
    // and the block id of token t + 32 is being looked up (each would otherwise be a memory round trip in front of
    // every token's arithmetic).  Tokens past the range read token tok_end - 1 again and are not used.
    auto block_of = [&](int t) { return p.blk[it.blk_off + min(t, it.tok_end - 1) / p.block_size]; };
    auto fetch = [&](int t, int blk, float (&kf)[E], float (&vf)[E], float& k_scale, float& v_scale) {
      const int tc = min(t, it.tok_end - 1);
      const int slot = tc % p.block_size;
      const int64_t off = int64_t(blk) * p.s_block + int64_t(it.kv_head) * p.s_head + int64_t(slot) * p.s_tok + dchunk * E;
      load_elems<KVT, E>(p.kv, off, kf);
      load_elems<KVT, E>(p.kv, off + p.s_kv, vf);
      k_scale = p.scale_log2;
      v_scale = 1.f;
      if constexpr (KVT == PS_FP8_E4M3) {
        const float* sc = p.scales + (int64_t(blk) * p.num_kv_heads + it.kv_head) * 2;
        k_scale *= sc[0];
        v_scale = sc[1];
      }
    };
    const int t_first = it.tok_begin + stream;
    float kf[E], vf[E], k_scale = 0.f, v_scale = 0.f;
    int blk_next = 0;
    if (t_first < it.tok_end) {
      fetch(t_first, block_of(t_first), kf, vf, k_scale, v_scale);
      blk_next = block_of(t_first + 16);
    }
    for (int t = t_first; t < it.tok_end; t += 16) {
      float kf_n[E], vf_n[E], k_scale_n, v_scale_n;
      fetch(t + 16, blk_next, kf_n, vf_n, k_scale_n, v_scale_n);
      blk_next = block_of(t + 32);
#pragma unroll
      for (int rr = 0; rr < kRowTile; ++rr) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) dot = fmaf(qreg[rr][e], kf[e], dot);
        float s = row16_allreduce_sum(dot) * k_scale;         // score in log2 units
        if (t >= lim[rr]) s = neg_inf;
        const float m_new = fmaxf(m[rr], s);
        const float m_ref = (m_new == neg_inf) ? 0.f : m_new; // a row that has seen nothing yet: exponents stay -inf
        const float alpha = fast_exp2(m[rr] - m_ref);         // m = -inf gives 0
        const float w = fast_exp2(s - m_ref);
        l[rr] = fmaf(l[rr], alpha, w);
        const float wv = w * v_scale;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[rr][e] = fmaf(acc[rr][e], alpha, wv * vf[e]);
        m[rr] = m_new;
      }
#pragma unroll
      for (int e = 0; e < E; ++e) { kf[e] = kf_n[e]; vf[e] = vf_n[e]; }
      k_scale = k_scale_n;
      v_scale = v_scale_n;
    }

    // merge the four 16-lane rows of this wave
#pragma unroll
    for (int mask = 16; mask <= 32; mask <<= 1) {
#pragma unroll
      for (int rr = 0; rr < kRowTile; ++rr) {
        const float mo = lane_xor(m[rr], mask);
        const float lo = lane_xor(l[rr], mask);
        const float mn = fmaxf(m[rr], mo);
        const float a = (m[rr] == neg_inf) ? 0.f : fast_exp2(m[rr] - mn);
        const float b = (mo == neg_inf) ? 0.f : fast_exp2(mo - mn);
        l[rr] = l[rr] * a + lo * b;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[rr][e] = acc[rr][e] * a + lane_xor(acc[rr][e], mask) * b;
        m[rr] = mn;
      }
    }
    if (lane < 16) {
#pragma unroll
      for (int rr = 0; rr < kRowTile; ++rr) {
        if (dchunk == 0) { sm_m[wave][rr] = m[rr]; sm_l[wave][rr] = l[rr]; }
#pragma unroll
        for (int e = 0; e < E; ++e) sm_acc[wave][rr][dchunk * E + e] = acc[rr][e];
      }
    }
    __syncthreads();

    // merge the four waves and write the partial state: 32 threads per row
    {
      const int rr = threadIdx.x >> 5;
      const int row = row0 + rr;
      if (rr < kRowTile && row < rows) {
        float mw[4], mn = neg_inf;
#pragma unroll
        for (int w = 0; w < 4; ++w) { mw[w] = sm_m[w][rr]; mn = fmaxf(mn, mw[w]); }
        float coef[4], lsum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          coef[w] = (mw[w] == neg_inf) ? 0.f : fast_exp2(mw[w] - mn);
          lsum += coef[w] * sm_l[w][rr];
        }
        const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
        const int req = p.req_list[it.req_off + row / G];
        const int h = it.kv_head * G + row % G;
        const int64_t slot = int64_t(p.slot_base[req]) + it.split_local;
        float* o = p.ws_o + (slot * p.num_q_heads + h) * D;
        for (int c = threadIdx.x & 31; c < D; c += 32) {
          float v = 0.f;
#pragma unroll
          for (int w = 0; w < 4; ++w) v += coef[w] * sm_acc[w][rr][c];
          o[c] = v * inv;
        }
        if ((threadIdx.x & 31) == 0)
          p.ws_lse[slot * p.num_q_heads + h] = lsum > 0.f ? (mn + __builtin_amdgcn_logf(lsum)) * kLn2 : neg_inf;
      }
    }
    __syncthreads();
  }
}

template <int D>
static bool dispatch_dtype(const AttnParams& p, const ps_geometry& g, int item_begin, int n_items, hipStream_t st) {
  const dim3 grid(n_items), block(256);
#define PS_CASE(KVT, QT)                                                                        \
  if (g.kv_dtype == KVT && g.q_dtype == QT) {                                                   \
    hipLaunchKernelGGL((wave_attention_kernel<D, KVT, QT>), grid, block, 0, st, p, item_begin); \
    return true;                                                                                \
  }
  PS_CASE(PS_F32, PS_F32)
  PS_CASE(PS_BF16, PS_BF16)
  PS_CASE(PS_FP8_E4M3, PS_BF16)
  PS_CASE(PS_BF16, PS_F32)
  PS_CASE(PS_F32, PS_BF16)
  PS_CASE(PS_FP8_E4M3, PS_F32)
#undef PS_CASE
  return false;
}

bool wave_supported(const ps_geometry& g) { return g.head_dim == 64 || g.head_dim == 128 || g.head_dim == 256; }

int32_t launch_wave_attention(const AttnParams& p, const ps_geometry& g, int item_begin, int n_items, hipStream_t st) {
  if (n_items <= 0) return PS_OK;
  bool ok = false;
  switch (g.head_dim) {
    case 64: ok = dispatch_dtype<64>(p, g, item_begin, n_items, st); break;
    case 128: ok = dispatch_dtype<128>(p, g, item_begin, n_items, st); break;
    case 256: ok = dispatch_dtype<256>(p, g, item_begin, n_items, st); break;
    default: break;
  }
  return ok ? PS_OK : PS_ERR_UNSUPPORTED;
}

}  // namespace psdev
