// Partial-prefill attention on the gfx950 matrix cores: many query rows per KV head against the cached context.
//
// When a context grows by a segment, only the new tokens are prefilled (System Design, execution pipeline step 1):
// every new token is a query row on its context's shared KV, the token at position t seeing the first t + 1
// tokens.  With G q heads per KV head a chunk of c new tokens is c * G rows per KV head -- hundreds, where a decode
// step has a few dozen -- so the work is a dense contraction and the matrix cores, not HBM, are the bound.
//
// One workgroup (4 waves) takes one work item: a token range of one context and KV head, and up to 256 query rows
// that see into it.  The rows are split over the waves, 64 each, and every wave walks the whole token range, so a
// wave never shares anything with its neighbours: no barrier, no cross-wave merge.  The four waves read the same
// K/V tiles at nearly the same time, so HBM (and mostly L2) sees each tile once per 256 rows.  A wave's query rows
// are kept as ready-made MFMA B operands, 16 bytes per lane and piece, in a lane-private corner of LDS (every lane
// reads back exactly what it wrote, so no synchronisation is involved; registers hold the accumulators, the tile
// buffers and the scores of two tiles).
//
// Per wave and 32-token tile the math is that of the decode kernel (S^T = K Q^T, online softmax with a lazily
// moving reference, O^T += V^T P^T; K straight into the A layout, V transposed in the lane), over four 16-row
// tiles.  Tiles past what every row of the wave sees are skipped; the per-row limit is applied only to tiles that
// reach past the shortest row.
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "mfma_common.h"

namespace psdev {

namespace {

constexpr int kD = kHeadDim;
constexpr int kNT = 4;            // 16-row tiles per wave
constexpr int kTile = kTileTokens;
constexpr float kLazy = kLazyRescale;

__device__ __forceinline__ int wave_max(int x) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) x = max(x, __builtin_amdgcn_ds_bpermute(((int(threadIdx.x) & 63) ^ m) << 2, x));
  return __builtin_amdgcn_readfirstlane(x);
}

}  // namespace

template <int KVT>
__global__ __launch_bounds__(256, 1) void prefill_attention_kernel(AttnParams p, const ps_item* __restrict__ items) {
  __shared__ u32x4 sm_qb[4][kNT * 4][64];   // [wave][row tile * 4 + k-step][lane]: that lane's B operand
  const ps_item* it = items + blockIdx.x;
  const int blk_off = __builtin_amdgcn_readfirstlane(it->blk_off);
  const int tok_begin = __builtin_amdgcn_readfirstlane(it->tok_begin);
  const int tok_end = __builtin_amdgcn_readfirstlane(it->tok_end);
  const int req_off = __builtin_amdgcn_readfirstlane(it->req_off);
  const int n_req = __builtin_amdgcn_readfirstlane(it->n_req);
  const int kv_head = __builtin_amdgcn_readfirstlane(it->kv_head);
  const int split_local = __builtin_amdgcn_readfirstlane(it->split_local);
  // visible lengths apply to a prompt's own prefix, and only where the plan found a row that sees less
  const bool limited = (__builtin_amdgcn_readfirstlane(it->kind) & kPsItemMasked) != 0;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int n = lane & 15;   // query row within a row tile / token within a block / d-chunk, by role
  const int kg = lane >> 4;
  const int G = p.group;
  const int rows = n_req * G;
  const int row_base = 64 * wave;
  if (row_base >= rows) return;   // nothing shared between waves: a wave without rows simply leaves
  const int nt_used = min(kNT, (rows - row_base + 15) >> 4);
  const float neg_inf = -__builtin_inff();

  // ---- this lane's query rows (row 16 t + n of the wave): request, visible length, and the row itself as the
  // four B operands of S^T = K Q^T
  int req_of[kNT], lim[kNT];
  int lim_hi = 0, lim_lo = 0x7fffffff;
#pragma unroll
  for (int t = 0; t < kNT; ++t) {
    const int row = row_base + 16 * t + n;
    req_of[t] = -1;
    lim[t] = 0;   // a padding row sees nothing
    u32x4 piece[4] = {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};
    if (row < rows) {
      const int req = p.req_list[req_off + row / G];
      req_of[t] = req;
      lim[t] = limited ? min(tok_end, p.visible[req]) : tok_end;
      const uint16_t* qrow = static_cast<const uint16_t*>(p.q) + (int64_t(req) * p.num_q_heads + kv_head * G + row % G) * kD;
#pragma unroll
      for (int st = 0; st < 4; ++st) piece[st] = *reinterpret_cast<const u32x4*>(qrow + q_chunk_elem<KVT>(st, kg));
      lim_hi = max(lim_hi, lim[t]);
      lim_lo = min(lim_lo, lim[t]);
    }
#pragma unroll
    for (int st = 0; st < 4; ++st) sm_qb[wave][4 * t + st][lane] = piece[st];
  }
  const int see_end = wave_max(lim_hi);      // no row of this wave sees a token at or past this one
  const int see_all = -wave_max(-lim_lo);    // every row of this wave sees every token before this one
  if (see_end <= tok_begin) return;          // cannot happen for planned items; keeps the loop bounds honest
  const int n_tiles = (see_end - tok_begin + kTile - 1) / kTile;

  // ---- addressing (as in the decode kernel): block base in SGPRs, two loop-invariant VGPR offsets
  const int sub_shift = __builtin_ctz(unsigned(p.block_size >> 4));
  const int sub_mask = (p.block_size >> 4) - 1;
  constexpr int kEsz = KVT == PS_BF16 ? 2 : 1;
  const int tok_bytes = int(p.s_tok) * kEsz;
  const int kv_bytes = int(p.s_kv) * kEsz;
  const int k_lane_off = n * tok_bytes + kg * 16;
  const int v_lane_off = 4 * kg * tok_bytes + n * (8 * kEsz);
  const int64_t head_base = reinterpret_cast<int64_t>(p.kv) + int64_t(kv_head) * p.s_head * kEsz;
  const int64_t blk_bytes = p.s_block * kEsz;
  const int sub_bytes = 16 * tok_bytes;
  const int sub0 = tok_begin >> 4;
  const int sub_end = (see_end + 15) >> 4;

  struct TileIds { int id[2]; float ksc[2], lvs[2]; };
  auto fetch_ids = [&](int k) __attribute__((always_inline)) {    // block ids (and e4m3 scales) of the two 16-token blocks of tile k; wave-uniform
    TileIds r;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      // no branch around these loads (the index is clamped into the range instead), so that the counting of
      // outstanding loads in the streaming loop stays exact; a block past the range is never fetched from
      const int sub = min(sub0 + 2 * k + b, sub_end - 1);
      r.id[b] = __builtin_amdgcn_readfirstlane(p.blk[blk_off + (sub >> sub_shift)]);
      r.ksc[b] = 1.f;
      r.lvs[b] = 0.f;
      if constexpr (KVT == PS_FP8_E4M3) {
        const float* sc = p.scales + (int64_t(r.id[b]) * p.num_kv_heads + kv_head) * 2;
        r.ksc[b] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(sc[0])));
        r.lvs[b] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(__builtin_amdgcn_logf(sc[1]))));
      }
    }
    return r;
  };
  // K and V of a tile live in separate buffers, because they are needed at different times (see the loop below).
  // Every call issues the same loads; a block past the range gets a zero-sized descriptor (zeros, no traffic).
  struct KTile { u32x4 k[2][KVT == PS_BF16 ? 4 : 2]; };
  struct VTile { std::conditional_t<KVT == PS_BF16, u32x4, u32x2> v[8]; };
  auto tile_rsrc = [&](const TileIds& ids, int k, int b) __attribute__((always_inline)) {
    const int sub = sub0 + 2 * k + b;
    const bool valid = sub < sub_end;
    const int64_t addr = head_base + int64_t(ids.id[b]) * blk_bytes + (sub & sub_mask) * sub_bytes;
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(addr), 0, valid ? 0x7fffffff : 0, 0x00020000);
  };
  auto load_k = [&](KTile& kt, const TileIds& ids, int k) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const __amdgpu_buffer_rsrc_t rs = tile_rsrc(ids, k, b);
#pragma unroll
      for (int s = 0; s < (KVT == PS_BF16 ? 4 : 2); ++s)
        kt.k[b][s] = __builtin_amdgcn_raw_buffer_load_b128(rs, k_lane_off + 64 * s, 0, 0);
    }
  };
  auto load_v = [&](VTile& vt, const TileIds& ids, int k) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const __amdgpu_buffer_rsrc_t rs = tile_rsrc(ids, k, b);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (KVT == PS_BF16)
          vt.v[4 * b + i] = __builtin_amdgcn_raw_buffer_load_b128(rs, v_lane_off, kv_bytes + i * tok_bytes, 0);
        else
          vt.v[4 * b + i] = __builtin_amdgcn_raw_buffer_load_b64(rs, v_lane_off, kv_bytes + i * tok_bytes, 0);
      }
    }
  };

  float m_run[kNT], l_run[kNT];
  f32x4 acc[kNT][8];
#pragma unroll
  for (int t = 0; t < kNT; ++t) {
    m_run[t] = neg_inf;
    l_run[t] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  struct Scores { f32x4 s[kNT][2]; };
  struct KOperands { bf16x8 a[2][4]; };
  auto k_operands = [&](const KTile& kt) __attribute__((always_inline)) {
    KOperands ka;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if constexpr (KVT == PS_BF16) {
#pragma unroll
        for (int s = 0; s < 4; ++s) ka.a[b][s] = as_bf16x8(kt.k[b][s]);
      } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          ka.a[b][2 * h] = as_bf16x8(e4m3x8_to_bf16x8(kt.k[b][h].x, kt.k[b][h].y));
          ka.a[b][2 * h + 1] = as_bf16x8(e4m3x8_to_bf16x8(kt.k[b][h].z, kt.k[b][h].w));
        }
      }
    }
    return ka;
  };
  // The query operands of row tile t, read back from LDS.  (The lane index goes through an empty asm so that they
  // are read tile by tile: hoisted out of the streaming loop they would occupy 64 registers that the accumulators
  // and tile buffers need.)
  struct QOperands { bf16x8 b[4]; };
  auto q_operands = [&](int t) __attribute__((always_inline)) {
    int q_lane = lane;
    asm volatile("" : "+v"(q_lane));
    QOperands q;
#pragma unroll
    for (int st = 0; st < 4; ++st) q.b[st] = as_bf16x8(sm_qb[wave][4 * t + st][q_lane]);
    return q;
  };
  // Raw scores S^T = K Q^T of one tile for row tile t: two accumulation chains (one per 16-token block), issued
  // alternately.
  auto qk_row_tile = [&](const KOperands& ka, const QOperands& q, Scores& sc, int t) __attribute__((always_inline)) {
    sc.s[t][0] = f32x4{0.f, 0.f, 0.f, 0.f};
    sc.s[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
      for (int b = 0; b < 2; ++b) sc.s[t][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka.a[b][st], q.b[st], sc.s[t][b], 0, 0, 0);
  };
  auto qk_scores = [&](const KTile& kt, Scores& sc) __attribute__((always_inline)) {
    const KOperands ka = k_operands(kt);
#pragma unroll
    for (int t = 0; t < kNT; ++t) qk_row_tile(ka, q_operands(t), sc, t);
  };

  // Online softmax of a tile's scores and O^T += V^T P^T, with the scores of the next tile (K in kt_next, result
  // in sc_next) issued row tile by row tile in between: each batch of eight matrix instructions is followed by the
  // exponentials of one row tile of this tile, which the vector units work off while the matrix cores are busy.
  // limited_tag: std::true_type applies the per-row limits (and guards rows that have seen nothing yet);
  // std::false_type promises that every row of the wave sees the whole tile.
  // bf16 KV: the scores of the next tile are issued row tile by row tile between the exponentials (measured 11 %
  // faster than issuing them first); e4m3 KV: all of them first, then the softmax (the interleaved order measured
  // 25 % slower there, next to the conversions of the K codes).
  constexpr bool kInterleave = KVT == PS_BF16;
  auto softmax_pv = [&](Scores& sc, const VTile& vtile, const TileIds& ids, int k, const KTile& kt_next, Scores& sc_next,
                        auto limited_tag) __attribute__((always_inline)) {
    constexpr bool kLimited = decltype(limited_tag)::value;
    if constexpr (!kInterleave) qk_scores(kt_next, sc_next);
    const int tok0 = tok_begin + kTile * k;
    float sc_k[2], lvs[2], inv_v[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      sc_k[b] = p.scale_log2 * ids.ksc[b];
      lvs[b] = ids.lvs[b];
      inv_v[b] = KVT == PS_FP8_E4M3 ? fast_exp2(-lvs[b]) : 1.f;
    }
    if constexpr (kLimited) {
#pragma unroll
      for (int t = 0; t < kNT; ++t)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (tok0 + 16 * b + 4 * kg + j >= lim[t]) sc.s[t][b][j] = neg_inf;
    }
    // The softmax reference m_run follows the row maximum lazily: it moves (and the accumulators are rescaled)
    // only when some score gets more than kLazy ahead of it, so probabilities stay below 2^kLazy instead of below 1
    // -- the same result by shift invariance of softmax.  The test is local to the lane (its own scores, in log2
    // units; the scales are positive, so a block's maximum scales like its scores) and one vote covers the four
    // row tiles; only when it fires somewhere in the wave is the maximum of each row put together across the
    // row's four lanes, which must agree on m_run.  A row that has seen nothing yet has m_run = -inf and stays
    // there until a score arrives.
    float mx[kNT];
    bool ahead = false;
#pragma unroll
    for (int t = 0; t < kNT; ++t) {
      if constexpr (KVT == PS_BF16)   // (the shorter max_of4 form makes this variant spill and run 25 % slower)
        mx[t] = fmaxf(fmaxf(fmaxf(sc.s[t][0][0], sc.s[t][0][1]), fmaxf(sc.s[t][0][2], sc.s[t][0][3])) * sc_k[0],
                      fmaxf(fmaxf(sc.s[t][1][0], sc.s[t][1][1]), fmaxf(sc.s[t][1][2], sc.s[t][1][3])) * sc_k[1]);
      else
        mx[t] = fmaxf(max_of4(sc.s[t][0]) * sc_k[0], max_of4(sc.s[t][1]) * sc_k[1]);
      ahead |= mx[t] > m_run[t] + kLazy;
    }
    if (__builtin_amdgcn_ballot_w64(ahead) != 0) {
#pragma unroll
      for (int t = 0; t < kNT; ++t) {
        float row_mx = fmaxf(mx[t], lane_xor(mx[t], 16));
        row_mx = fmaxf(row_mx, lane_xor(row_mx, 32));
        const float m_new = (row_mx > m_run[t] + kLazy) ? row_mx : m_run[t];
        const float alpha = (m_new == m_run[t]) ? 1.f : fast_exp2(m_run[t] - m_new);   // -inf -> finite gives 0
        l_run[t] *= alpha;
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) acc[t][cc] *= alpha;
        m_run[t] = m_new;
      }
    }
    KOperands ka_next;
    QOperands q_cur;
    if constexpr (kInterleave) {
      ka_next = k_operands(kt_next);
      q_cur = q_operands(0);
    }
    bf16x8 pb[kNT];
#pragma unroll
    for (int t = 0; t < kNT; ++t) {
      if constexpr (kInterleave) {
        // the query operands of the next row tile are requested before this row tile's work (hides the LDS latency)
        const QOperands q_nxt = q_operands((t + 1) % kNT);
        qk_row_tile(ka_next, q_cur, sc_next, t);
        q_cur = q_nxt;
      }
      const float m_ref = (kLimited && m_run[t] == neg_inf) ? 0.f : m_run[t];
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const float shift = lvs[b] - m_ref;
        float lsum = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float pw = fast_exp2(__builtin_fmaf(sc.s[t][b][j], sc_k[b], shift));
          lsum += pw;
          pb[t][4 * b + j] = (__bf16)pw;
        }
        l_run[t] += (KVT == PS_FP8_E4M3) ? lsum * inv_v[b] : lsum;
      }
    }
    u32x4 vr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if constexpr (KVT == PS_BF16) vr[i] = vtile.v[i];
      else vr[i] = e4m3x8_to_bf16x8(vtile.v[i].x, vtile.v[i].y);
    }
    if constexpr (kLimited) {      // slots past the item's range may hold anything: zero them
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tok = tok0 + 16 * (i >> 2) + 4 * kg + (i & 3);
        if (tok >= tok_end) vr[i] = u32x4{0, 0, 0, 0};
      }
    }
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) {
      uint32_t w[4];
#pragma unroll
      for (int i2 = 0; i2 < 4; ++i2) {
        const uint32_t a = vr[2 * i2][cc >> 1], b = vr[2 * i2 + 1][cc >> 1];
        w[i2] = __builtin_amdgcn_perm(b, a, (cc & 1) ? 0x07060302u : 0x05040100u);
      }
      const bf16x8 vt = as_bf16x8(u32x4{w[0], w[1], w[2], w[3]});
#pragma unroll
      for (int t = 0; t < kNT; ++t) acc[t][cc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb[t], acc[t][cc], 0, 0, 0);
    }
  };

  // ---- stream the token range, software-pipelined across tiles: the scores of tile k + 1 go to the matrix cores
  // before the softmax of tile k starts, so that the vector work of one tile overlaps with the matrix work of the
  // next.  K of tile k + 1 is consumed one step before V of tile k + 1, hence the separate buffers: a K buffer is
  // refilled (tile k + 3) as soon as its scores are issued, a V buffer (tile k + 2) after its P V.  First the tiles
  // that every row of the wave sees whole (an even number, so the buffers keep their roles), then the rest with the
  // per-row limits.  No branch surrounds a load, so the counting of outstanding loads stays exact.
  const int n_whole = max(0, (see_all - tok_begin) / kTile) & ~1;
  KTile kb[2];
  VTile vb[2];
  Scores sc_a, sc_b;
  TileIds ids_a = fetch_ids(0), ids_b = fetch_ids(1);
  load_k(kb[0], ids_a, 0);
  load_v(vb[0], ids_a, 0);
  load_k(kb[1], ids_b, 1);
  load_v(vb[1], ids_b, 1);
  TileIds ids_c = fetch_ids(2), ids_d = fetch_ids(3);
  qk_scores(kb[0], sc_a);
  load_k(kb[0], ids_c, 2);
  auto two_tiles = [&](int k, auto limited_tag) __attribute__((always_inline)) {
    // tile k: scores in sc_a, V in vb[0]; tile k + 1: K in kb[1], V in vb[1]; tile k + 2: K arriving in kb[0]
    softmax_pv(sc_a, vb[0], ids_a, k, kb[1], sc_b, limited_tag);
    load_k(kb[1], ids_d, k + 3);
    load_v(vb[0], ids_c, k + 2);
    const TileIds ids_e = fetch_ids(k + 4), ids_f = fetch_ids(k + 5);
    // tile k + 1, with the scores of tile k + 2 (zeros past the range, never used then)
    softmax_pv(sc_b, vb[1], ids_b, k + 1, kb[0], sc_a, limited_tag);
    load_k(kb[0], ids_e, k + 4);
    load_v(vb[1], ids_d, k + 3);
    ids_a = ids_c;
    ids_b = ids_d;
    ids_c = ids_e;
    ids_d = ids_f;
  };
  int k = 0;
  for (; k < n_whole; k += 2) two_tiles(k, std::false_type{});
  for (; k < n_tiles; k += 2) two_tiles(k, std::true_type{});

  // ---- one partial state per row, straight from the accumulators: lane (n, kg) holds O[row n][32 kg + 8 j + cc]
#pragma unroll
  for (int t = 0; t < kNT; ++t) {
    if (t < nt_used) {
      float l = l_run[t];
      l += lane_xor(l, 16);
      l += lane_xor(l, 32);
      if (req_of[t] >= 0) {
        const float inv = l > 0.f ? 1.f / l : 0.f;
        const int row = row_base + 16 * t + n;
        const int h = kv_head * G + row % G;
        const int64_t slot = int64_t(p.slot_base[req_of[t]]) + split_local;
        float* o = p.ws_o + (slot * p.num_q_heads + h) * kD + 32 * kg;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          *reinterpret_cast<f32x4*>(o + 8 * j) =
              f32x4{acc[t][0][j], acc[t][1][j], acc[t][2][j], acc[t][3][j]} * inv;
          *reinterpret_cast<f32x4*>(o + 8 * j + 4) =
              f32x4{acc[t][4][j], acc[t][5][j], acc[t][6][j], acc[t][7][j]} * inv;
        }
        if (kg == 0)
          p.ws_lse[slot * p.num_q_heads + h] = l > 0.f ? (m_run[t] + __builtin_amdgcn_logf(l)) * kLn2 : neg_inf;
      }
    }
  }
}

int32_t launch_prefill_attention(const AttnParams& p, const ps_geometry& g, const ps_item* items, int num_items,
                                 hipStream_t st) {
  if (num_items <= 0) return PS_OK;
  const int spb = g.block_size / 16;
  if (g.head_dim != kD || g.q_dtype != PS_BF16 || g.block_size % 16 != 0 || (spb & (spb - 1)) != 0)
    return PS_ERR_UNSUPPORTED;
  const dim3 grid(num_items), block(256);
  if (g.kv_dtype == PS_BF16)
    hipLaunchKernelGGL((prefill_attention_kernel<PS_BF16>), grid, block, 0, st, p, items);
  else if (g.kv_dtype == PS_FP8_E4M3)
    hipLaunchKernelGGL((prefill_attention_kernel<PS_FP8_E4M3>), grid, block, 0, st, p, items);
  else
    return PS_ERR_UNSUPPORTED;
  return PS_OK;
}

}  // namespace psdev
