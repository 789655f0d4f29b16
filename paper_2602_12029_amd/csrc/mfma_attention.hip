// Grouped-query attention over KV token ranges on the gfx950 matrix cores (bf16 Q, bf16 or e4m3 KV).
//
// Persistent kernel: every workgroup (4 waves) walks its own list of work items, fixed by the host
// plan.  A work item is a token range of one KV segment and one KV head, applied to every query row
// that reads it (all requests sharing the prefix x the G q heads of the KV head's group; a private
// suffix has just the G rows of its request).  Each K/V byte of the range is loaded from HBM exactly
// once, straight into the MFMA operand registers of one wave.
//
// Per wave, per tile of 32 tokens (two 16-token blocks a, b), with rows padded to 16-row tiles:
//   S^T[token, row] = K[token, :] . Q[row, :]        v_mfma_f32_16x16x32_bf16, A = K, B = Q^T
//   online softmax per row (a row lives in lanes n, n+16, n+32, n+48; n = lane % 16)
//   O^T[dcol, row] += V^T[dcol, token] . P^T[token, row]          A = V^T, B = P^T
// The C layout of S^T (lane (n, kg) holds tokens 4kg..4kg+3 of a block for row n) is exactly the B
// layout PV needs, so probabilities never leave their lane.  K rows are fetched 16 bytes per lane, eight
// lanes to a 128-byte line, and reach the A layout with one rotation inside each row of 16 lanes (the
// contraction index is permuted consistently in K and Q); V is fetched row-wise (one 16-lane group covers
// a full token row) and transposed inside each lane with 16-bit picks.
//
// Streaming: a wave owns a ring of NB tile buffers in VGPRs; the loads of the tile NB - 1 slots ahead
// are issued before the math of the current one.  Every slot issues the same 16 buffer loads -- a slot
// without a tile uses a zero-sized buffer descriptor, which returns zeros without touching memory -- so
// the inner loop has no branch around a memory instruction and the outstanding-load counter the
// compiler waits on is exact (a conditional load anywhere in the loop makes it wait for *all* loads,
// including the prefetch).  The ring runs across item boundaries: the last NB - 1 slots of an item
// fetch the first tiles of the workgroup's next item, whose block ids and query rows were fetched
// one item earlier, so the cross-wave merge and partial-state store at the end of an item overlap
// with loads in flight.
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "mfma_common.h"

namespace psdev {

namespace {

constexpr int kD = kHeadDim;
constexpr int kWaves = 4;
constexpr int kTile = kTileTokens;
constexpr int kLdsRow = kD + 4;   // padded row of the merge buffer (floats)
constexpr int kQRow = kD + 8;     // padded query row (bf16), 16 bytes of padding against bank conflicts
constexpr int kHdrRing = 128;     // item headers staged in LDS (circular, refilled in halves)
constexpr float kLazy = kLazyRescale;

template <int KVT>
struct TileRegs;                  // raw K/V of one 32-token tile as loaded
template <>
struct TileRegs<PS_BF16> {
  u32x4 k[2][4];                  // [block][2 T + h]: 16 bytes of token 8 T + lane % 8, see load_item_tile
  u32x4 v[8];                     // token i of this lane's 8 tokens, d columns 8*(lane%16)..+7
};
template <>
struct TileRegs<PS_FP8_E4M3> {
  u32x4 k[2][2];                  // [block][T]: 16 codes of token 8 T + lane % 8, see load_item_tile
  u32x2 v[8];                     // 8 codes: token i, d columns 8*(lane%16)..+7
};

// Wave-uniform view of one work item for one wave.
struct ItemCtx {
  int blk_off, tok_begin, tok_end, req_off, n_req, kv_head, split_local;
  int rows, nt_used, my_tiles, sub0, sub_end;
  int kind;            // the item's flag bits
  int masked;          // non-zero: some row of the item sees fewer tokens than tok_end (MASKED kernels only)
  // (fourteen ints, then the 64-bit address: no padding anywhere, so the struct still splits into registers)
  int64_t head_base;   // address of the item's KV head slice in block 0
};

// Per-lane metadata of an item: block ids (and e4m3 scales) of this wave's tiles.  Lane 2 k + h of word r describes
// 16-token block h of the wave's tile 32 r + k, so an item holds up to 64 tiles per wave (kPsMfmaMaxChunk tokens).
struct ItemMeta {
  int ids[2];
  float ksc[2], lvs[2];   // e4m3: K scale and log2 of the V scale of the block (1 and 0 otherwise)
};
constexpr ItemMeta kNoMeta = {{0, 0}, {1.f, 1.f}, {0.f, 0.f}};
// entry (k, b) of a metadata word pair: the wave's tile k, block b (k is wave-uniform)
__device__ __forceinline__ int meta_pick(const int (&word)[2], int k, int b) {
  const int lo = __builtin_amdgcn_readlane(word[0], ((2 * k) & 63) + b), hi = __builtin_amdgcn_readlane(word[1], ((2 * k) & 63) + b);
  return (k & 32) ? hi : lo;
}
__device__ __forceinline__ float meta_pick(const float (&word)[2], int k, int b) {
  const int lo = __builtin_amdgcn_readlane(__float_as_int(word[0]), ((2 * k) & 63) + b);
  const int hi = __builtin_amdgcn_readlane(__float_as_int(word[1]), ((2 * k) & 63) + b);
  return __int_as_float((k & 32) ? hi : lo);
}

// K rows reach the lanes in whole 128-byte lines: one load instruction covers 8 tokens, 8 lanes each -- lane (n, kg)
// takes 16 bytes at chunk (n >> 3) + 2 kg of the line, for token 8 T + (n & 7).  (Fetching 16 bytes per lane for token n
// directly would ask for half a line per token and instruction; a read kernel with that footprint tops out at 6.2 TB/s
// on this chip against 7.0 TB/s with whole lines.)  Lanes n < 8 then hold their own token in the T = 0 load and lane
// (n + 8)'s token in the T = 1 load, lanes n >= 8 the other way round; one rotation by 8 inside each row of 16 lanes
// hands the foreign half over.  Afterwards every lane (n, kg) holds chunks 2 kg (even) and 2 kg + 1 (odd) of token n.
constexpr int kRowRor8 = 0x128;   // DPP control: rotate by 8 lanes within each row of 16
__device__ __forceinline__ u32x4 k_even(u32x4 t0, u32x4 t1) {   // lanes n < 8 keep t0, lanes n >= 8 get lane (n - 8)'s t1
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_update_dpp(t0[i], t1[i], kRowRor8, 0xF, 0xC, false);
  return r;
}
__device__ __forceinline__ u32x4 k_odd(u32x4 t0, u32x4 t1) {    // lanes n >= 8 keep t1, lanes n < 8 get lane (n + 8)'s t0
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_update_dpp(t1[i], t0[i], kRowRor8, 0xF, 0x3, false);
  return r;
}
// element offset of the 8 query values that meet K's k-step `step` in lane group kg (the contraction index is
// permuted, identically in K and Q): bf16 rows have two lines, steps (2 h, 2 h + 1) = even and odd chunk of line h;
// an e4m3 row is one line, steps (0, 1) = the two halves of the even chunk, (2, 3) of the odd one
template <int KVT>
__device__ __forceinline__ int k_step_elem(int step, int kg) {
  if constexpr (KVT == PS_BF16) return 64 * (step >> 1) + 16 * kg + 8 * (step & 1);
  return 32 * kg + 8 * step;
}

template <int NT>
struct QIndex { int idx[NT]; };   // global q row (request * Hq + head) this thread fetches per row tile, -1 = padding
template <int NT>
struct QRegs { u32x4 piece[NT]; };
template <int NT>
struct RowLimit { int lim[NT]; };  // per row tile: first token that row (lane % 16) of the tile does not see

}  // namespace

// NT: 16-row tiles carried; NB: tile buffers in the register ring; OCC: waves per SIMD the register
// budget is sized for; MASKED: rows may see only a leading part of an item's token range (per-request visible
// prefix length), which costs a compare per score and guards against rows that have seen nothing yet.
template <int NT, int KVT, int NB, int OCC, bool MASKED, bool STREAM>
__global__ __launch_bounds__(256, OCC) void mfma_attention_kernel(AttnParams p, const ps_item* __restrict__ wg_items,
                                                                  const int32_t* __restrict__ wg_indptr) {
  __shared__ float sm_o[kWaves][16][kLdsRow];
  __shared__ float sm_m[kWaves][16];
  __shared__ float sm_l[kWaves][16];
  __shared__ __attribute__((aligned(16))) uint16_t sm_q[NT][16][kQRow];
  __shared__ __attribute__((aligned(16))) int32_t sm_hdr[kHdrRing][8];

  const int j_first = wg_indptr[blockIdx.x], j_last = wg_indptr[blockIdx.x + 1];
  if (j_first >= j_last) return;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int n = lane & 15;   // query row within a row tile / token within a block / d-chunk, by role
  const int kg = lane >> 4;
  const int G = p.group;
  const float neg_inf = -__builtin_inff();
  // 16-token sub-blocks per physical block: a power of two (the launcher checks), so index math is shifts
  const int sub_shift = __builtin_ctz(unsigned(p.block_size >> 4));
  const int sub_mask = (p.block_size >> 4) - 1;
  constexpr int kEsz = KVT == PS_BF16 ? 2 : 1;
  const int tok_bytes = int(p.s_tok) * kEsz;
  const int kv_bytes = int(p.s_kv) * kEsz;    // K -> V distance inside a (block, head)
  // per-lane byte offsets inside a 16-token sub-block
  const int k_lane_off = (n & 7) * tok_bytes + ((n >> 3) + 2 * kg) * 16;
  const int v_lane_off = 4 * kg * tok_bytes + n * (8 * kEsz);

  const int64_t kv_base = reinterpret_cast<int64_t>(p.kv);
  const int64_t blk_bytes = p.s_block * kEsz;
  const int sub_bytes = 16 * tok_bytes;

  // ---- item headers: staged in LDS (circular) so that looking two items ahead costs no memory round trip ----
  auto stage_headers = [&](int first, int count) {   // items [first, first + count) -> their ring slots
    const int32_t* src = reinterpret_cast<const int32_t*>(wg_items + first);
    for (int i = threadIdx.x; i < count * 8; i += 256)
      sm_hdr[((first - j_first) + (i >> 3)) % kHdrRing][i & 7] = src[i];
  };
  auto item_ctx = [&](int j) {
    const int32_t* h = sm_hdr[(j - j_first) % kHdrRing];
    ItemCtx c;
    c.blk_off = __builtin_amdgcn_readfirstlane(h[0]);
    c.tok_begin = __builtin_amdgcn_readfirstlane(h[1]);
    c.tok_end = __builtin_amdgcn_readfirstlane(h[2]);
    c.req_off = __builtin_amdgcn_readfirstlane(h[3]);
    c.n_req = __builtin_amdgcn_readfirstlane(h[4]);
    c.kv_head = __builtin_amdgcn_readfirstlane(h[5]);
    c.split_local = __builtin_amdgcn_readfirstlane(h[6]);
    c.kind = __builtin_amdgcn_readfirstlane(h[7]);
    c.masked = MASKED ? (c.kind & kPsItemMasked) : 0;
    c.rows = c.n_req * G;
    c.nt_used = (c.rows + 15) >> 4;
    const int tiles_total = (c.tok_end - c.tok_begin + kTile - 1) / kTile;
    c.my_tiles = tiles_total > wave ? (tiles_total - wave + kWaves - 1) / kWaves : 0;
    c.sub0 = c.tok_begin >> 4;
    c.sub_end = (c.tok_end + 15) >> 4;
    c.head_base = kv_base + int64_t(c.kv_head) * p.s_head * kEsz;
    return c;
  };

  // block ids (and scales) of this wave's tiles of an item: lane 2k+h of word r <- 16-token block h of tile 32 r + k
  auto fetch_meta = [&](const ItemCtx& c) {
    ItemMeta m = kNoMeta;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int k = 32 * r + (lane >> 1);
      const int sub = c.sub0 + 2 * (wave + kWaves * k) + (lane & 1);
      if (k < c.my_tiles && sub < c.sub_end) {
        m.ids[r] = p.blk[c.blk_off + (sub >> sub_shift)];
        if constexpr (KVT == PS_FP8_E4M3) {
          // K and V scale of the (block, head) as one 8-byte load: the addresses differ from lane to lane, so every
          // load instruction here costs a cache lookup per lane
          const u32x2 sc = *reinterpret_cast<const u32x2*>(p.scales + (int64_t(m.ids[r]) * p.num_kv_heads + c.kv_head) * 2);
          m.ksc[r] = __uint_as_float(sc.x);
          m.lvs[r] = __builtin_amdgcn_logf(__uint_as_float(sc.y));   // log2
        }
      }
    }
    return m;
  };

  // visible length of this lane's row in every row tile, clamped to the item's token range
  auto fetch_limits = [&](const ItemCtx& c) {
    RowLimit<NT> r;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      r.lim[t] = c.tok_end;
      if constexpr (MASKED) {
        const int row = 16 * t + n;
        if (c.masked && row < c.rows) r.lim[t] = min(c.tok_end, p.visible[p.req_list[c.req_off + row / G]]);
      }
    }
    return r;
  };

  // query rows: one 16-byte piece per thread and row tile (row = thread / 16, piece = thread % 16)
  auto q_row_index = [&](const ItemCtx& c) {
    QIndex<NT> r;
    const int rr = threadIdx.x >> 4;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int row = 16 * t + rr;
      r.idx[t] = -1;
      if (row < c.rows) r.idx[t] = p.req_list[c.req_off + row / G] * p.num_q_heads + c.kv_head * G + row % G;
    }
    return r;
  };
  auto load_q = [&](const QIndex<NT>& rows_idx) {
    QRegs<NT> q;
    const int cpiece = threadIdx.x & 15;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      q.piece[t] = u32x4{0, 0, 0, 0};
      if (rows_idx.idx[t] >= 0)
        q.piece[t] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.q) +
                                                     int64_t(rows_idx.idx[t]) * kD + 8 * cpiece);
    }
    return q;
  };
  auto store_q = [&](const QRegs<NT>& q) {
    const int rr = threadIdx.x >> 4, cpiece = threadIdx.x & 15;
#pragma unroll
    for (int t = 0; t < NT; ++t) *reinterpret_cast<u32x4*>(&sm_q[t][rr][8 * cpiece]) = q.piece[t];
  };

  // ---- tile loads: buffer loads, block base in SGPRs, two loop-invariant VGPR offsets ---------------------
  // `live` false (or a 16-token block past the segment end) gives a zero-sized descriptor: zeros, no traffic.
  // STREAM: the K/V of this launch is (almost all) read by one item only, so the loads are non-temporal -- the
  // lines do not displace what the caches hold and are not kept for a reader that never comes.  The policy is an
  // immediate of the load and a branch around loads would spoil the wait counts, hence one choice per launch.
  constexpr int kPolicy = STREAM ? kNonTemporal : 0;
  auto load_item_tile = [&](TileRegs<KVT>& tr, const ItemCtx& c, const ItemMeta& m, int k, bool live) {
    const int sub_a = c.sub0 + 2 * (wave + kWaves * k);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int sub = sub_a + b;
      const bool valid = live && k < c.my_tiles && sub < c.sub_end;
      const int id = meta_pick(m.ids, k & 63, b);
      const int64_t addr = c.head_base + int64_t(id) * blk_bytes + (sub & sub_mask) * sub_bytes;
      // a descriptor of size zero fetches nothing and returns zeros, whatever its base
      const __amdgpu_buffer_rsrc_t rs =
          __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(addr), 0, valid ? 0x7fffffff : 0, 0x00020000);
      if constexpr (KVT == PS_BF16) {
#pragma unroll
        for (int s = 0; s < 4; ++s)   // s = 2 T + h: tokens 8 T .. 8 T + 7, line h of their rows
          tr.k[b][s] = __builtin_amdgcn_raw_buffer_load_b128(rs, k_lane_off + 128 * (s & 1), 8 * (s >> 1) * tok_bytes, kPolicy);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          tr.v[4 * b + i] = __builtin_amdgcn_raw_buffer_load_b128(rs, v_lane_off, kv_bytes + i * tok_bytes, kPolicy);
      } else {
#pragma unroll
        for (int s = 0; s < 2; ++s)   // s = T: tokens 8 T .. 8 T + 7, whole rows
          tr.k[b][s] = __builtin_amdgcn_raw_buffer_load_b128(rs, k_lane_off, 8 * s * tok_bytes, kPolicy);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          tr.v[4 * b + i] = __builtin_amdgcn_raw_buffer_load_b64(rs, v_lane_off, kv_bytes + i * tok_bytes, kPolicy);
      }
    }
  };

  // ---- running state of the current item -------------------------------------------------------------------
  float m_run[NT], l_run[NT];
  f32x4 acc[NT][8];
  auto reset_state = [&]() {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      m_run[t] = neg_inf;
      l_run[t] = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };

  // all_rows_tag / full_tag: std::true_type promises that every row tile is in use / that the tile has all its
  // 32 tokens, which removes the uniform branches from the body so that the compiler can schedule the transposes
  // and conversions under the matrix instructions; std::false_type decides at run time.
  auto compute_tile = [&](TileRegs<KVT>& tr, const ItemCtx& c, const ItemMeta& meta, const RowLimit<NT>& rl, int k,
                          auto all_rows_tag, auto full_tag) {
    constexpr bool kAllRows = decltype(all_rows_tag)::value, kFull = decltype(full_tag)::value;
    const int tok0 = c.tok_begin + kTile * (wave + kWaves * k);  // first token of the tile
    const bool full = kFull || tok0 + kTile <= c.tok_end;
    // Per 16-token block: scores are raw dot products times sc_k (1/sqrt(d) in log2 units, times the block's K
    // scale); the block's V scale rides in the exponent of the probabilities (lvs = log2 of it), so that the
    // unscaled V codes can go into the matrix cores, and comes out of the row sums again through inv_v.
    float sc_k[2] = {p.scale_log2, p.scale_log2}, lvs[2] = {0.f, 0.f}, inv_v[2] = {1.f, 1.f};
    if constexpr (KVT == PS_FP8_E4M3) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        sc_k[b] *= meta_pick(meta.ksc, k, b);
        lvs[b] = meta_pick(meta.lvs, k, b);
        inv_v[b] = fast_exp2(-lvs[b]);
      }
    }

    // K operands
    bf16x8 ka[2][4];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if constexpr (KVT == PS_BF16) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          ka[b][2 * h] = as_bf16x8(k_even(tr.k[b][h], tr.k[b][2 + h]));
          ka[b][2 * h + 1] = as_bf16x8(k_odd(tr.k[b][h], tr.k[b][2 + h]));
        }
      } else {
        const u32x4 ev = k_even(tr.k[b][0], tr.k[b][1]), od = k_odd(tr.k[b][0], tr.k[b][1]);
        ka[b][0] = as_bf16x8(e4m3x8_to_bf16x8(ev.x, ev.y));
        ka[b][1] = as_bf16x8(e4m3x8_to_bf16x8(ev.z, ev.w));
        ka[b][2] = as_bf16x8(e4m3x8_to_bf16x8(od.x, od.y));
        ka[b][3] = as_bf16x8(e4m3x8_to_bf16x8(od.z, od.w));
      }
    }
    // scores and probabilities of every row tile first ...
    bf16x8 pb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      pb[t] = bf16x8{};
      if (kAllRows || t < c.nt_used) {
        bf16x8 qb[4];
#pragma unroll
        for (int st = 0; st < 4; ++st)
          qb[st] = as_bf16x8(*reinterpret_cast<const u32x4*>(&sm_q[t][n][k_step_elem<KVT>(st, kg)]));
        f32x4 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          s[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int st = 0; st < 4; ++st) s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[b][st], qb[st], s[b], 0, 0, 0);
        }
        if (MASKED || !full) {
          const int lim = MASKED ? rl.lim[t] : c.tok_end;
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (tok0 + 16 * b + 4 * kg + j >= lim) s[b][j] = neg_inf;
        }
        // The softmax reference m_run follows the row maximum lazily: it moves (and the accumulators are rescaled)
        // only when some score gets more than kLazy ahead of it, so probabilities stay below 2^kLazy instead of below 1
        // -- the same result by shift invariance of softmax.  The test is local to the lane (its own 8 scores, in log2
        // units; the scales are positive, so a block's maximum scales like its scores); only when it fires somewhere in
        // the wave is the maximum of each row put together across the row's four lanes, which must agree on m_run.
        // A row that has seen nothing yet has m_run = -inf and stays there until a score arrives.
        float mx = fmaxf(max_of4(s[0]) * sc_k[0], max_of4(s[1]) * sc_k[1]);
        if (__builtin_amdgcn_ballot_w64(mx > m_run[t] + kLazy) != 0) {
          mx = fmaxf(mx, lane_xor(mx, 16));
          mx = fmaxf(mx, lane_xor(mx, 32));
          const float m_new = (mx > m_run[t] + kLazy) ? mx : m_run[t];
          const float alpha = (m_new == m_run[t]) ? 1.f : fast_exp2(m_run[t] - m_new);   // -inf -> finite gives 0
          l_run[t] *= alpha;
#pragma unroll
          for (int cc = 0; cc < 8; ++cc) acc[t][cc] *= alpha;
          m_run[t] = m_new;
        }
        const float m_ref = (MASKED && m_run[t] == neg_inf) ? 0.f : m_run[t];   // keeps (-inf) - (-inf) out of the exponents
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const float shift = lvs[b] - m_ref;
          float lsum = 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float pw = fast_exp2(__builtin_fmaf(s[b][j], sc_k[b], shift));   // probability times the V scale
            lsum += pw;
            pb[t][4 * b + j] = (__bf16)pw;
          }
          l_run[t] += (KVT == PS_FP8_E4M3) ? lsum * inv_v[b] : lsum;
        }
      }
    }
    // V rows of this lane's 8 tokens, invalid tokens zeroed (their slots may hold anything)
    std::remove_reference_t<decltype(tr.v[0])> vraw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) vraw[i] = tr.v[i];
    if (!full) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tok = tok0 + 16 * (i >> 2) + 4 * kg + (i & 3);
        if (tok >= c.tok_end) vraw[i] = std::remove_reference_t<decltype(tr.v[0])>{};
      }
    }
    // ... then O^T += V^T P^T, one 16-column group of V at a time, transposed inside the lane:
    // vt = column cc of this lane's 8 token rows
    // (every row tile, used or not: the probabilities of an unused one are zero.  A uniform branch around single
    // matrix instructions here splits the products into many small basic blocks, and one such build returned wrong
    // sums for items that use fewer row tiles than the kernel carries -- the straight-line form is the one tested)
    auto accumulate = [&](int cc, const uint32_t (&w)[4]) {
      const bf16x8 vt = as_bf16x8(u32x4{w[0], w[1], w[2], w[3]});
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[t][cc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb[t], acc[t][cc], 0, 0, 0);
    };
    if constexpr (KVT == PS_BF16) {
#pragma unroll
      for (int cc = 0; cc < 8; ++cc) {
        uint32_t w[4];
#pragma unroll
        for (int i2 = 0; i2 < 4; ++i2) {
          // low (even cc) or high (odd cc) halves of a pair of token rows: one byte permute
          const uint32_t a = vraw[2 * i2][cc >> 1], b = vraw[2 * i2 + 1][cc >> 1];
          w[i2] = __builtin_amdgcn_perm(b, a, (cc & 1) ? 0x07060302u : 0x05040100u);
        }
        accumulate(cc, w);
      }
    } else {
      // e4m3: the transposition is done on the codes, before the conversion -- one byte permute gathers columns
      // (cc, cc + 1) of a pair of token rows, and each half of it converts into one operand register
#pragma unroll
      for (int cp = 0; cp < 4; ++cp) {
        uint32_t w0[4], w1[4];
#pragma unroll
        for (int i2 = 0; i2 < 4; ++i2) {
          const uint32_t a = vraw[2 * i2][cp >> 1], b = vraw[2 * i2 + 1][cp >> 1];
          const uint32_t pair = __builtin_amdgcn_perm(b, a, (cp & 1) ? 0x07030602u : 0x05010400u);
          w0[i2] = e4m3x2_to_bf16x2(pair, false);
          w1[i2] = e4m3x2_to_bf16x2(pair, true);
        }
        accumulate(2 * cp, w0);
        accumulate(2 * cp + 1, w1);
      }
    }
  };

  // merge the four waves of the item and write one partial state per row
  auto epilogue = [&](const ItemCtx& c) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < c.nt_used) {
        float l = l_run[t];
        l += lane_xor(l, 16);
        l += lane_xor(l, 32);
        if (kg == 0) {
          sm_m[wave][n] = m_run[t];
          sm_l[wave][n] = l;
        }
        // lane (n, kg), acc[cc][j] = O[row n][32 kg + 8 j + cc]
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          *reinterpret_cast<f32x4*>(&sm_o[wave][n][32 * kg + 8 * j]) =
              f32x4{acc[t][0][j], acc[t][1][j], acc[t][2][j], acc[t][3][j]};
          *reinterpret_cast<f32x4*>(&sm_o[wave][n][32 * kg + 8 * j + 4]) =
              f32x4{acc[t][4][j], acc[t][5][j], acc[t][6][j], acc[t][7][j]};
        }
        __syncthreads();
        const int r = threadIdx.x >> 4;  // row of the tile
        const int c0 = (threadIdx.x & 15) * 8;
        const int row = 16 * t + r;
        if (row < c.rows) {
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
          const int req = p.req_list[c.req_off + row / G];
          const int h = c.kv_head * G + row % G;
          const int64_t slot = int64_t(p.slot_base[req]) + c.split_local;
          float* o = p.ws_o + (slot * p.num_q_heads + h) * kD + c0;
          *reinterpret_cast<f32x4*>(o) = o0 * inv;
          *reinterpret_cast<f32x4*>(o + 4) = o1 * inv;
          if ((threadIdx.x & 15) == 0)
            p.ws_lse[slot * p.num_q_heads + h] = lsum > 0.f ? (mn + __builtin_amdgcn_logf(lsum)) * kLn2 : neg_inf;
        }
        __syncthreads();
      }
    }
  };

  // ---- walk the item list ------------------------------------------------------------------------------------
  // Software pipeline over items: `cur` streams; `nxt` has its block ids and query-row indices in registers
  // (fetched one iteration ago); the item after that gets its fetches issued now.
  stage_headers(j_first, min(kHdrRing, j_last - j_first));
  __syncthreads();
  ItemCtx cur = item_ctx(j_first);
  ItemMeta meta = fetch_meta(cur);
  RowLimit<NT> lim = fetch_limits(cur);
  // first tiles go out as soon as the block ids are here; the query rows follow while they fly
  TileRegs<KVT> buf[NB];
#pragma unroll
  for (int u = 0; u < NB - 1; ++u) load_item_tile(buf[u], cur, meta, u, true);
  store_q(load_q(q_row_index(cur)));
  bool has_next = j_first + 1 < j_last;
  ItemCtx nxt = cur;
  ItemMeta meta_nxt = kNoMeta;
  QIndex<NT> q_idx_nxt{};
  RowLimit<NT> lim_nxt{};
  if (has_next) {
    nxt = item_ctx(j_first + 1);
    meta_nxt = fetch_meta(nxt);
    lim_nxt = fetch_limits(nxt);
    q_idx_nxt = q_row_index(nxt);
  }
  __syncthreads();

  for (int j = j_first; j < j_last; ++j) {
    // query rows of the next item (their indices arrived long ago), fetches for the item after it
    QRegs<NT> q_nxt{};
    if (has_next) q_nxt = load_q(q_idx_nxt);
    const bool has_nn = j + 2 < j_last;
    ItemCtx nn = nxt;
    ItemMeta meta_nn = kNoMeta;
    QIndex<NT> q_idx_nn{};
    RowLimit<NT> lim_nn{};
    if (has_nn) {
      nn = item_ctx(j + 2);
      meta_nn = fetch_meta(nn);
      lim_nn = fetch_limits(nn);
      q_idx_nn = q_row_index(nn);
    }

    reset_state();
    // every item occupies at least one full turn of the ring, so its last NB - 1 slots always exist to
    // fetch ahead into the next item
    const int slots = max(NB, (cur.my_tiles + NB - 1) / NB * NB);
    int s0 = 0;
    // Turns before the last: every slot fetched ahead still belongs to this item, and every tile computed is a
    // complete one (the item's ragged tile, if any, is its last and falls into the last turn).
    auto full_turns = [&](auto all_rows_tag) {
      for (; s0 + NB < slots; s0 += NB) {
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          load_item_tile(buf[(u + NB - 1) % NB], cur, meta, s0 + u + NB - 1, true);
          compute_tile(buf[u], cur, meta, lim, s0 + u, all_rows_tag, std::true_type{});
        }
      }
    };
    if (NT == 1) full_turns(std::true_type{});
    else full_turns(std::false_type{});
    // last turn of the ring: its first fetch is the item's last slot, the others reach into the next item
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      if (u == 0) load_item_tile(buf[NB - 1], cur, meta, s0 + NB - 1, true);
      else load_item_tile(buf[u - 1], nxt, meta_nxt, u - 1, has_next);
      if (s0 + u < cur.my_tiles) compute_tile(buf[u], cur, meta, lim, s0 + u, std::false_type{}, std::false_type{});
    }

    epilogue(cur);   // ends with a barrier: sm_q and the consumed half of the header ring are free

    if (has_next) store_q(q_nxt);
    const int li = j + 1 - j_first;                     // items consumed so far
    if ((li % (kHdrRing / 2)) == 0) {                   // refill the half of the header ring just used up
      const int first = j_first + li + kHdrRing / 2;
      if (first < j_last) stage_headers(first, min(kHdrRing / 2, j_last - first));
    }
    __syncthreads();
    cur = nxt;
    meta = meta_nxt;
    lim = lim_nxt;
    lim_nxt = lim_nn;
    has_next = has_nn;
    nxt = nn;
    meta_nxt = meta_nn;
    q_idx_nxt = q_idx_nn;
  }
}

int32_t launch_mfma_attention(const AttnParams& p, const ps_geometry& g, int max_rows, int occ, bool masked, bool stream,
                              const ps_item* wg_items, const int32_t* wg_indptr, int num_wg, hipStream_t st) {
  if (num_wg <= 0) return PS_OK;
  const int spb = g.block_size / 16;
  if (g.head_dim != kD || g.q_dtype != PS_BF16 || g.block_size % 16 != 0 || (spb & (spb - 1)) != 0 || max_rows > 64)
    return PS_ERR_UNSUPPORTED;
  if (g.kv_dtype != PS_BF16 && g.kv_dtype != PS_FP8_E4M3) return PS_ERR_UNSUPPORTED;
  const dim3 grid(num_wg), block(256);
  const int nt = max_rows <= 16 ? 1 : (max_rows <= 32 ? 2 : 4);
#define PS_LAUNCH_AS(NT, KVT, NB, OCC, MASKED, STREAM) \
  hipLaunchKernelGGL((mfma_attention_kernel<NT, KVT, NB, OCC, MASKED, STREAM>), grid, block, 0, st, p, wg_items, wg_indptr)
#define PS_LAUNCH(NT, KVT, NB, OCC)                                \
  do {                                                             \
    if (masked) {                                                  \
      if (stream) PS_LAUNCH_AS(NT, KVT, NB, OCC, true, true);      \
      else PS_LAUNCH_AS(NT, KVT, NB, OCC, true, false);            \
    } else {                                                       \
      if (stream) PS_LAUNCH_AS(NT, KVT, NB, OCC, false, true);     \
      else PS_LAUNCH_AS(NT, KVT, NB, OCC, false, false);           \
    }                                                              \
  } while (0)
  // two tile buffers per wave everywhere (deeper rings measured no faster); `occ` is the residency the
  // plan sized the grid for (ps_mfma_occupancy)
  if (g.kv_dtype == PS_BF16) {
    if (nt == 1) { if (occ == 2) PS_LAUNCH(1, PS_BF16, 2, 2); else PS_LAUNCH(1, PS_BF16, 2, 1); }
    else if (nt == 2) PS_LAUNCH(2, PS_BF16, 2, 1);
    else PS_LAUNCH(4, PS_BF16, 2, 1);
  } else {
    if (nt == 1) { if (occ == 2) PS_LAUNCH(1, PS_FP8_E4M3, 2, 2); else PS_LAUNCH(1, PS_FP8_E4M3, 2, 1); }
    else if (nt == 2) { if (occ == 2) PS_LAUNCH(2, PS_FP8_E4M3, 2, 2); else PS_LAUNCH(2, PS_FP8_E4M3, 2, 1); }
    else PS_LAUNCH(4, PS_FP8_E4M3, 2, 1);
  }
#undef PS_LAUNCH
#undef PS_LAUNCH_AS
  return PS_OK;
}

}  // namespace psdev
