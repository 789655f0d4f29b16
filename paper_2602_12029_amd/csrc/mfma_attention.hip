// Grouped-query attention over a KV token range on the gfx950 matrix cores (bf16 Q, bf16 or e4m3 KV).
//
// One workgroup (4 waves) handles one work item: a token range of one KV segment and one KV head,
// applied to every query row that reads it (all requests sharing the prefix x the G q heads of the
// KV head's group; a private suffix has just the G rows of its request).  Each K/V byte of the
// range is loaded from HBM exactly once, straight into the MFMA operand registers of one wave.
//
// Per wave, per tile of 32 tokens (two 16-token blocks a, b), with rows padded to 16-row tiles:
//   S^T[token, row] = K[token, :] . Q[row, :]        v_mfma_f32_16x16x32_bf16, A = K, B = Q^T
//   online softmax per row (a row lives in lanes n, n+16, n+32, n+48; n = lane % 16)
//   O^T[dcol, row] += V^T[dcol, token] . P^T[token, row]          A = V^T, B = P^T
// The C layout of S^T (lane (n, kg) holds tokens 4kg..4kg+3 of a block for row n) is exactly the B
// layout PV needs, so probabilities never leave their lane.  K rows are fetched 16 bytes per lane in
// the A layout (the contraction index is permuted consistently in K and Q); V is fetched row-wise
// (one 16-lane group covers a full token row) and transposed inside each lane with 16-bit picks.
// Waves take tiles round-robin, keep private (max, sum, O) state and are merged through LDS at the
// end into one normalised partial state per (request, q head).
#include <cstdlib>
#include <type_traits>

#include "device_common.h"
#include "launch.h"

namespace psdev {

namespace {

constexpr int kD = 128;
constexpr int kWaves = 4;
constexpr int kTile = 32;        // tokens per wave iteration
constexpr int kLdsRow = kD + 4;  // padded row of the merge buffer

template <int KVT>
struct TileRegs;                 // raw K/V of one 32-token tile as loaded
template <>
struct TileRegs<PS_BF16> {
  uint4 k[2][4];                 // [block][k-step]: 8 bf16 of token (lane%16), d-chunk 4*step + lane/16
  uint4 v[8];                    // token i of this lane's 8 tokens, d columns 8*(lane%16)..+7
};
template <>
struct TileRegs<PS_FP8_E4M3> {
  uint4 k[2][2];                 // [block][half]: 16 codes of token (lane%16), d 64*half + 16*(lane/16)..+15
  uint2 v[8];                    // 8 codes: token i, d columns 8*(lane%16)..+7
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// two e4m3 codes (bytes 2*half, 2*half+1 of w) -> two bf16 in one register (exact)
__device__ __forceinline__ uint32_t e4m3x2_to_bf16x2(uint32_t w, bool hi) {
  const f32x2 f = hi ? __builtin_amdgcn_cvt_pk_f32_fp8(w, true) : __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
  bf16x2 b;
  b.x = (__bf16)f.x;
  b.y = (__bf16)f.y;
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(uint32_t lo, uint32_t hi) {
  uint4 r;
  r.x = e4m3x2_to_bf16x2(lo, false);
  r.y = e4m3x2_to_bf16x2(lo, true);
  r.z = e4m3x2_to_bf16x2(hi, false);
  r.w = e4m3x2_to_bf16x2(hi, true);
  return r;
}

// element offset of the 8 query values that meet K's k-step `step` in lane group kg
template <int KVT>
__device__ __forceinline__ int q_chunk_elem(int step, int kg) {
  if constexpr (KVT == PS_BF16) return 32 * step + 8 * kg;
  return 64 * (step >> 1) + 16 * kg + 8 * (step & 1);
}

}  // namespace

// NT: 16-row tiles carried; NB: tile buffers in registers (NB - 1 tiles of loads in flight ahead of the
// math); OCC: waves per SIMD the register budget is sized for.
template <int NT, int KVT, int NB, int OCC>
__global__ __launch_bounds__(256, OCC) void mfma_attention_kernel(AttnParams p, int item_begin) {
  __shared__ float sm_o[kWaves][16][kLdsRow];
  __shared__ float sm_m[kWaves][16];
  __shared__ float sm_l[kWaves][16];
  __shared__ __attribute__((aligned(16))) uint16_t sm_q[NT][16][kD + 8];  // rows padded by 16 B against bank conflicts

  const ps_item it = p.items[item_begin + blockIdx.x];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int n = lane & 15;   // query row within a row tile / token within a block / d-chunk, by role
  const int kg = lane >> 4;
  const int G = p.group;
  const int rows = it.n_req * G;
  const int nt_used = (rows + 15) >> 4;
  const float neg_inf = -__builtin_inff();
  const int sub_per_blk = p.block_size >> 4;  // 16-token sub-blocks per physical block

  // ---- query rows, staged in LDS and re-read as B operands for every tile ------------------------------
  // (keeping them in registers would cost 16 VGPRs per row tile for the whole kernel)
  {
    const int r = threadIdx.x >> 4, c = threadIdx.x & 15;  // one 16-byte piece per thread and row tile
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int row = 16 * t + r;
      uint4 piece = uint4{0, 0, 0, 0};
      if (row < rows) {
        const int req = p.req_list[it.req_off + row / G];
        const int h = it.kv_head * G + row % G;
        piece = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p.q) +
                                                (int64_t(req) * p.num_q_heads + h) * kD + 8 * c);
      }
      *reinterpret_cast<uint4*>(&sm_q[t][r][8 * c]) = piece;
    }
  }
  __syncthreads();

  // ---- per-wave tile schedule ----------------------------------------------------------------------
  const int span = it.tok_end - it.tok_begin;
  const int tiles_total = (span + kTile - 1) / kTile;
  const int my_tiles = tiles_total > wave ? (tiles_total - wave + kWaves - 1) / kWaves : 0;
  const int sub0 = it.tok_begin >> 4;  // first 16-token sub-block of the item within its segment
  const int sub_end = (it.tok_end + 15) >> 4;

  // block ids (and fp8 scales) of the next 32 tiles of this wave: lane 2j+h <- sub-block h of tile j
  int ids = 0;
  float ksc = 1.f, vsc = 1.f;
  auto fetch_ids = [&](int tile_first) {
    const int k = tile_first + (lane >> 1);
    const int sub = sub0 + 2 * (wave + kWaves * k) + (lane & 1);
    ids = 0;
    ksc = 1.f;
    vsc = 1.f;
    if (k < my_tiles && sub < sub_end) {
      ids = p.blk[it.blk_off + sub / sub_per_blk];
      if constexpr (KVT == PS_FP8_E4M3) {
        const float* sc = p.scales + (int64_t(ids) * p.num_kv_heads + it.kv_head) * 2;
        ksc = sc[0];
        vsc = sc[1];
      }
    }
  };

  const int64_t head_off = int64_t(it.kv_head) * p.s_head;
  using Elem = typename std::conditional<KVT == PS_BF16, uint16_t, uint8_t>::type;
  const Elem* kv = static_cast<const Elem*>(p.kv);

  auto load_tile = [&](TileRegs<KVT>& tr, int k) {
    const int kl = k & 31;
    const int sub_a = sub0 + 2 * (wave + kWaves * k);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int sub = sub_a + b;
      if (sub < sub_end) {
        const int id = __builtin_amdgcn_readlane(ids, 2 * kl + b);
        const Elem* base = kv + int64_t(id) * p.s_block + head_off + int64_t((sub % sub_per_blk) << 4) * p.s_tok;
        const Elem* krow = base + int64_t(n) * p.s_tok;
        const Elem* vbase = base + p.s_kv + int64_t(4 * kg) * p.s_tok + 8 * n;
        if constexpr (KVT == PS_BF16) {
#pragma unroll
          for (int s = 0; s < 4; ++s) tr.k[b][s] = *reinterpret_cast<const uint4*>(krow + 32 * s + 8 * kg);
#pragma unroll
          for (int i = 0; i < 4; ++i) tr.v[4 * b + i] = *reinterpret_cast<const uint4*>(vbase + int64_t(i) * p.s_tok);
        } else {
#pragma unroll
          for (int s = 0; s < 2; ++s) tr.k[b][s] = *reinterpret_cast<const uint4*>(krow + 64 * s + 16 * kg);
#pragma unroll
          for (int i = 0; i < 4; ++i) tr.v[4 * b + i] = *reinterpret_cast<const uint2*>(vbase + int64_t(i) * p.s_tok);
        }
      } else {
        if constexpr (KVT == PS_BF16) {
#pragma unroll
          for (int s = 0; s < 4; ++s) tr.k[b][s] = uint4{0, 0, 0, 0};
#pragma unroll
          for (int i = 0; i < 4; ++i) tr.v[4 * b + i] = uint4{0, 0, 0, 0};
        } else {
#pragma unroll
          for (int s = 0; s < 2; ++s) tr.k[b][s] = uint4{0, 0, 0, 0};
#pragma unroll
          for (int i = 0; i < 4; ++i) tr.v[4 * b + i] = uint2{0, 0};
        }
      }
    }
  };

  // ---- running state ---------------------------------------------------------------------------------
  float m_run[NT], l_run[NT];
  f32x4 acc[NT][8];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    m_run[t] = neg_inf;
    l_run[t] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  auto compute_tile = [&](TileRegs<KVT>& tr, int k) {
    const int kl = k & 31;
    const int tok0 = it.tok_begin + kTile * (wave + kWaves * k);  // first token of the tile
    const bool full = tok0 + kTile <= it.tok_end;
    float sc_k[2] = {p.scale_log2, p.scale_log2}, sc_v[2] = {1.f, 1.f};
    if constexpr (KVT == PS_FP8_E4M3) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        sc_k[b] *= __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ksc), 2 * kl + b));
        sc_v[b] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(vsc), 2 * kl + b));
      }
    }

    // K operands
    bf16x8 ka[2][4];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if constexpr (KVT == PS_BF16) {
#pragma unroll
        for (int s = 0; s < 4; ++s) ka[b][s] = as_bf16x8(tr.k[b][s]);
      } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          ka[b][2 * h] = as_bf16x8(e4m3x8_to_bf16x8(tr.k[b][h].x, tr.k[b][h].y));
          ka[b][2 * h + 1] = as_bf16x8(e4m3x8_to_bf16x8(tr.k[b][h].z, tr.k[b][h].w));
        }
      }
    }
    // V rows of this lane's 8 tokens as bf16, invalid tokens zeroed (their slots may hold anything)
    uint4 vr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if constexpr (KVT == PS_BF16) vr[i] = tr.v[i];
      else vr[i] = e4m3x8_to_bf16x8(tr.v[i].x, tr.v[i].y);
    }
    if (!full) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tok = tok0 + 16 * (i >> 2) + 4 * kg + (i & 3);
        if (tok >= it.tok_end) vr[i] = uint4{0, 0, 0, 0};
      }
    }
    // scores and probabilities of every row tile first ...
    bf16x8 pb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      pb[t] = bf16x8{};
      if (t < nt_used) {
        bf16x8 qb[4];
#pragma unroll
        for (int st = 0; st < 4; ++st)
          qb[st] = as_bf16x8(*reinterpret_cast<const uint4*>(&sm_q[t][n][q_chunk_elem<KVT>(st, kg)]));
        f32x4 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          s[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int st = 0; st < 4; ++st) s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[b][st], qb[st], s[b], 0, 0, 0);
          s[b] *= sc_k[b];  // scores in log2 units
        }
        if (!full) {
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (tok0 + 16 * b + 4 * kg + j >= it.tok_end) s[b][j] = neg_inf;
        }
        float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                         fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
        mx = fmaxf(mx, lane_xor(mx, 16));
        mx = fmaxf(mx, lane_xor(mx, 32));
        const float m_new = fmaxf(m_run[t], mx);  // finite: every tile holds at least one valid token
        if (__builtin_amdgcn_ballot_w64(m_new != m_run[t]) != 0) {
          const float alpha = fast_exp2(m_run[t] - m_new);
          l_run[t] *= alpha;
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[t][c] *= alpha;
          m_run[t] = m_new;
        }
        float lsum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float pw = fast_exp2(s[b][j] - m_new);
            lsum += pw;
            pb[t][4 * b + j] = (__bf16)(pw * sc_v[b]);
          }
        l_run[t] += lsum;
      }
    }
    // ... then O^T += V^T P^T, one 16-column group of V at a time, transposed inside the lane:
    // vt = column c of this lane's 8 token rows
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      uint32_t w[4];
#pragma unroll
      for (int i2 = 0; i2 < 4; ++i2) {
        const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&vr[2 * i2]);
        const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&vr[2 * i2 + 1]);
        const uint32_t a = r0[c >> 1], b = r1[c >> 1];
        w[i2] = (c & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
      }
      const bf16x8 vt = as_bf16x8(uint4{w[0], w[1], w[2], w[3]});
#pragma unroll
      for (int t = 0; t < NT; ++t)
        if (t < nt_used) acc[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb[t], acc[t][c], 0, 0, 0);
    }
  };

  // ---- stream the tiles, NB - 1 tiles of loads in flight ahead of the math ---------------------------
  TileRegs<KVT> buf[NB];
  for (int k0 = 0; k0 < my_tiles; k0 += 32) {
    fetch_ids(k0);
    const int k1 = min(my_tiles, k0 + 32);
#pragma unroll
    for (int u = 0; u < NB - 1; ++u)
      if (k0 + u < k1) load_tile(buf[u], k0 + u);
    for (int k = k0; k < k1; k += NB) {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int kk = k + u;
        if (kk < k1) {
          if (kk + NB - 1 < k1) load_tile(buf[(u + NB - 1) % NB], kk + NB - 1);
          compute_tile(buf[u], kk);
        }
      }
    }
  }

  // ---- merge the four waves and write one partial state per row ----------------------------------------
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t < nt_used) {
      float l = l_run[t];
      l += lane_xor(l, 16);
      l += lane_xor(l, 32);
      if (kg == 0) {
        sm_m[wave][n] = m_run[t];
        sm_l[wave][n] = l;
      }
      // lane (n, kg), acc[c][j] = O[row n][32 kg + 8 j + c]
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        *reinterpret_cast<f32x4*>(&sm_o[wave][n][32 * kg + 8 * j]) =
            f32x4{acc[t][0][j], acc[t][1][j], acc[t][2][j], acc[t][3][j]};
        *reinterpret_cast<f32x4*>(&sm_o[wave][n][32 * kg + 8 * j + 4]) =
            f32x4{acc[t][4][j], acc[t][5][j], acc[t][6][j], acc[t][7][j]};
      }
    }
    __syncthreads();
    if (t < nt_used) {
      const int r = threadIdx.x >> 4;  // row of the tile
      const int c0 = (threadIdx.x & 15) * 8;
      const int row = 16 * t + r;
      if (row < rows) {
        float mw[kWaves], mn = neg_inf;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          mw[w] = sm_m[w][r];
          mn = fmaxf(mn, mw[w]);
        }
        float coef[kWaves], lsum = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          coef[w] = (mw[w] == neg_inf) ? 0.f : fast_exp2(mw[w] - mn);
          lsum += coef[w] * sm_l[w][r];
        }
        const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
        f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          if (coef[w] != 0.f) {
            o0 += coef[w] * *reinterpret_cast<const f32x4*>(&sm_o[w][r][c0]);
            o1 += coef[w] * *reinterpret_cast<const f32x4*>(&sm_o[w][r][c0 + 4]);
          }
        }
        const int req = p.req_list[it.req_off + row / G];
        const int h = it.kv_head * G + row % G;
        const int64_t slot = int64_t(p.slot_base[req]) + it.split_local;
        float* o = p.ws_o + (slot * p.num_q_heads + h) * kD + c0;
        *reinterpret_cast<f32x4*>(o) = o0 * inv;
        *reinterpret_cast<f32x4*>(o + 4) = o1 * inv;
        if ((threadIdx.x & 15) == 0)
          p.ws_lse[slot * p.num_q_heads + h] = lsum > 0.f ? (mn + __builtin_amdgcn_logf(lsum)) * kLn2 : neg_inf;
      }
    }
    __syncthreads();
  }
}

int32_t launch_mfma_attention(const AttnParams& p, const ps_geometry& g, int max_rows, int item_begin, int n_items,
                              hipStream_t st) {
  if (n_items <= 0) return PS_OK;
  if (g.head_dim != kD || g.q_dtype != PS_BF16 || g.block_size % 16 != 0 || max_rows > 64) return PS_ERR_UNSUPPORTED;
  if (g.kv_dtype != PS_BF16 && g.kv_dtype != PS_FP8_E4M3) return PS_ERR_UNSUPPORTED;
  const dim3 grid(n_items), block(256);
  const int nt = max_rows <= 16 ? 1 : (max_rows <= 32 ? 2 : 4);
  int cfg = 0;
  if (const char* e = getenv("PS_MFMA_CFG")) cfg = atoi(e);
#define PS_LAUNCH(NT, KVT, NB, OCC) \
  hipLaunchKernelGGL((mfma_attention_kernel<NT, KVT, NB, OCC>), grid, block, 0, st, p, item_begin)
#define PS_BY_CFG(NT, KVT)                     \
  do {                                         \
    if (cfg == 1) PS_LAUNCH(NT, KVT, 3, 1);    \
    else if (cfg == 2) PS_LAUNCH(NT, KVT, 4, 1); \
    else if (cfg == 4) PS_LAUNCH(NT, KVT, 2, 1); \
    else PS_LAUNCH(NT, KVT, 2, 2);             \
  } while (0)
  if (g.kv_dtype == PS_BF16) {
    if (nt == 1) PS_BY_CFG(1, PS_BF16);
    else if (nt == 2) { if (cfg == 0) PS_LAUNCH(2, PS_BF16, 3, 1); else PS_BY_CFG(2, PS_BF16); }
    else PS_LAUNCH(4, PS_BF16, 2, 1);
  } else {
    if (nt == 1) PS_BY_CFG(1, PS_FP8_E4M3);
    else if (nt == 2) PS_BY_CFG(2, PS_FP8_E4M3);
    else PS_LAUNCH(4, PS_FP8_E4M3, 2, 1);
  }
#undef PS_BY_CFG
#undef PS_LAUNCH
  return PS_OK;
}

}  // namespace psdev
