// Partial-prefill attention on the gfx950 matrix cores: many query rows per KV head against the cached context.
//
// When a context grows by a segment, only the new tokens are prefilled (System Design, execution pipeline step 1):
// every new token is a query row on its context's shared KV, the token at position t seeing the first t + 1
// tokens.  With G q heads per KV head a chunk of c new tokens is c * G rows per KV head -- hundreds, where a decode
// step has a few dozen -- so the work is a dense contraction and the matrix cores, not HBM, are the bound.
//
// One workgroup of eight waves takes one work item: a token range of one context and KV head, and up to 256 query
// rows that see into it.  The rows are split over the waves, 32 each (two 16-row tiles, the query rows resident in
// registers as MFMA B operands), and every wave walks the token range.  Two waves share a SIMD, so that the vector
// work of one (exponentials, conversions) runs under the matrix instructions of the other; a wave on its own issues
// one instruction every four cycles and cannot cover its own matrix instructions.
//
// K and V reach the waves through LDS, as ready-made A operands: per 32-token tile the eight waves fetch one eighth
// of it each (K straight in operand layout; V as pairs of token rows, transposed inside the lane with one byte
// permute per operand register; e4m3 codes converted to bf16 once), write it to a three-stage ring, and after one
// barrier per tile every wave reads the 8 K and 8 V operands of the tile back, 16 bytes per lane and operand, each
// lane exactly the slot of its own lane index (no bank conflicts).  A tile is thus fetched, transposed and
// converted once per 256 rows.  Global loads run three tiles ahead of the products (two tiles in registers, one in
// LDS).
//
// Per wave and tile the math is that of the decode kernel (S^T = K Q^T, online softmax with a lazily moving
// reference, O^T += V^T P^T).  A wave skips the tiles past what its own rows see; the per-row limit is applied only
// to tiles that reach past the wave's shortest row.  Nothing but the ring is shared between waves: no cross-wave
// merge, every wave writes the partial states of its own rows.
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "mfma_common.h"

namespace psdev {

namespace {

constexpr int kD = kHeadDim;
constexpr int kWaves = 8;         // per workgroup
constexpr int kNT = 2;            // 16-row tiles per wave
constexpr int kRowsPerWave = 16 * kNT;
constexpr int kTile = kTileTokens;
constexpr int kStages = 3;        // LDS ring: tile k read, tile k + 1 written, tile k - 1 possibly still read
constexpr float kLazy = kLazyRescale;

__device__ __forceinline__ int wave_max(int x) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) x = max(x, __builtin_amdgcn_ds_bpermute(((int(threadIdx.x) & 63) ^ m) << 2, x));
  return __builtin_amdgcn_readfirstlane(x);
}

}  // namespace

template <int KVT>
__global__ __launch_bounds__(64 * kWaves) void prefill_attention_kernel(AttnParams p, const ps_item* __restrict__ items) {
  __shared__ u32x4 sm_k[kStages][8][64];   // [stage][4 * block + k-step][lane]: K as that lane's A operand
  __shared__ u32x4 sm_v[kStages][8][64];   // [stage][16-column group][lane]: V^T as that lane's A operand
  __shared__ f32x4 sm_sc[kStages][2];      // e4m3: [stage][block] = (score scale in log2 units, log2 of the V scale, 1 / V scale, -)
  __shared__ int sm_see[kWaves];
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
  const int row_base = kRowsPerWave * wave;
  const int nt_used = max(0, min(kNT, (rows - row_base + 15) >> 4));   // 0: a wave without rows only fetches
  const float neg_inf = -__builtin_inff();

  // ---- this lane's query rows (row 16 t + n of the wave): request, visible length, and the row itself as the
  // four B operands of S^T = K Q^T (k-step st, lane group kg: elements 32 st + 8 kg .. + 7)
  int req_of[kNT], lim[kNT];
  bf16x8 qb[kNT][4];
  int lim_hi = 0, lim_lo = 0x7fffffff;
#pragma unroll
  for (int t = 0; t < kNT; ++t) {
    const int row = row_base + 16 * t + n;
    req_of[t] = -1;
    lim[t] = 0;   // a padding row sees nothing
#pragma unroll
    for (int st = 0; st < 4; ++st) qb[t][st] = as_bf16x8(u32x4{0, 0, 0, 0});
    if (row < rows) {
      const int req = p.req_list[req_off + row / G];
      req_of[t] = req;
      lim[t] = limited ? min(tok_end, p.visible[req]) : tok_end;
      const uint16_t* qrow = static_cast<const uint16_t*>(p.q) + (int64_t(req) * p.num_q_heads + kv_head * G + row % G) * kD;
#pragma unroll
      for (int st = 0; st < 4; ++st) qb[t][st] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 32 * st + 8 * kg));
      lim_hi = max(lim_hi, lim[t]);
      lim_lo = min(lim_lo, lim[t]);
    }
  }
  const int see_end = max(tok_begin, wave_max(lim_hi));   // no row of this wave sees a token at or past this one
  const int see_all = -wave_max(-lim_lo);                 // every row of this wave sees every token before this one
  if (lane == 0) sm_see[wave] = see_end;
  __syncthreads();
  int see_end_wg = tok_begin;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) see_end_wg = max(see_end_wg, sm_see[w]);
  see_end_wg = __builtin_amdgcn_readfirstlane(see_end_wg);
  const int n_tiles_wg = (see_end_wg - tok_begin + kTile - 1) / kTile;   // tiles the workgroup fetches
  const int n_tiles = nt_used > 0 ? (see_end - tok_begin + kTile - 1) / kTile : 0;   // tiles this wave multiplies
  const int n_whole = min(n_tiles, max(0, (see_all - tok_begin) / kTile));   // ... of which these need no per-row limit

  // ---- addressing: block base in SGPRs (a buffer descriptor per 16-token block), loop-invariant lane offsets
  const int sub_shift = __builtin_ctz(unsigned(p.block_size >> 4));
  const int sub_mask = (p.block_size >> 4) - 1;
  constexpr int kEsz = KVT == PS_BF16 ? 2 : 1;
  const int tok_bytes = int(p.s_tok) * kEsz;
  const int kv_bytes = int(p.s_kv) * kEsz;
  const int64_t head_base = reinterpret_cast<int64_t>(p.kv) + int64_t(kv_head) * p.s_head * kEsz;
  const uint32_t blk_bytes = uint32_t(p.s_block * kEsz);
  const int sub_bytes = 16 * tok_bytes;
  const int sub0 = tok_begin >> 4;
  const int sub_end = (see_end_wg + 15) >> 4;
  // What this wave fetches of every tile, all of it from one 16-token block (fblk) so that one block id and one
  // buffer descriptor per tile do.  K: operand (block fblk, k-step kst) -- token n of the block, the 8 elements of
  // lane group kg.  V: the pair of token rows (2 vp, 2 vp + 1) of the eight a lane group owns (rows 4 kg + i of
  // block 0, then of block 1), column half vh -- 4 of the lane's 8 columns.
  const int fblk = wave >> 2, kst = wave & 3;
  const int vp = 2 * fblk + (wave & 1), vh = (wave >> 1) & 1;
  const int vi = 2 * (wave & 1);
  const int k_lane_off = n * tok_bytes + (32 * kst + 8 * kg) * kEsz;
  const int v_lane_off = kv_bytes + (4 * kg + vi) * tok_bytes + (8 * n + 4 * vh) * kEsz;
  const int32_t* blk_seg = p.blk + blk_off;

  struct TileIds { int id; };   // of this wave's block of the tile
  auto fetch_ids = [&](int k) __attribute__((always_inline)) {   // wave-uniform
    // no branch around this load (the index is clamped into the range instead), so that the counting of
    // outstanding loads in the streaming loop stays exact; a block past the range is never fetched from
    TileIds r;
    const int sub = max(sub0, min(sub0 + 2 * k + fblk, sub_end - 1));
    r.id = __builtin_amdgcn_readfirstlane(blk_seg[sub >> sub_shift]);
    return r;
  };
  // this wave's share of a tile, as loaded
  struct Fetched {
    std::conditional_t<KVT == PS_BF16, u32x4, u32x2> k;         // 8 elements of one token
    std::conditional_t<KVT == PS_BF16, u32x2, uint32_t> v[2];   // 4 columns of two token rows
    f32x2 sc;                                                   // e4m3: K and V scale of the block
  };
  auto fetch = [&](Fetched& f, const TileIds& ids, int k) __attribute__((always_inline)) {
    const int sub = sub0 + 2 * k + fblk;
    const bool valid = sub < sub_end;   // a block past the range gets a zero-sized descriptor: zeros, no traffic
    const uint64_t addr = uint64_t(head_base) + uint64_t(uint32_t(ids.id)) * blk_bytes + uint32_t((sub & sub_mask) * sub_bytes);
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(addr), 0, valid ? 0x7fffffff : 0, 0x00020000);
    if constexpr (KVT == PS_BF16) {
      f.k = __builtin_amdgcn_raw_buffer_load_b128(rs, k_lane_off, 0, 0);
      f.v[0] = __builtin_amdgcn_raw_buffer_load_b64(rs, v_lane_off, 0, 0);
      f.v[1] = __builtin_amdgcn_raw_buffer_load_b64(rs, v_lane_off, tok_bytes, 0);
    } else {
      f.k = __builtin_amdgcn_raw_buffer_load_b64(rs, k_lane_off, 0, 0);
      f.v[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, v_lane_off, 0, 0);
      f.v[1] = __builtin_amdgcn_raw_buffer_load_b32(rs, v_lane_off, tok_bytes, 0);
      // (the block id is clamped into the range, so the scales of a tile past it are some block's: never used)
      f.sc = *reinterpret_cast<const f32x2*>(p.scales + (int64_t(ids.id) * p.num_kv_heads + kv_head) * 2);
    }
  };
  // ... and its way into the ring: K as it is (e4m3: converted), V transposed -- register vp of the operand of
  // column group cc holds column 8 n + cc of the token rows (2 vp, 2 vp + 1)
  auto publish = [&](const Fetched& f, int stage, int k) __attribute__((always_inline)) {
    if constexpr (KVT == PS_BF16) {
      sm_k[stage][4 * fblk + kst][lane] = f.k;
    } else {
      sm_k[stage][4 * fblk + kst][lane] = e4m3x8_to_bf16x8(f.k.x, f.k.y);
      // the block's scales, once per workgroup: the K scale folded into the score scale, the V scale as the exponent
      // offset of the probabilities and as the factor that takes it out of the row sums again
      if (kst == 0 && lane == 0) {
        const float lv = __builtin_amdgcn_logf(f.sc.y);
        sm_sc[stage][fblk] = f32x4{p.scale_log2 * f.sc.x, lv, fast_exp2(-lv), 0.f};
      }
    }
    // slots of tokens past the item's range may hold anything: zero them (their probabilities are zero)
    auto v0 = f.v[0], v1 = f.v[1];
    if (tok_begin + kTile * (k + 1) > tok_end) {   // (only the item's last tile can reach past its range)
      const int tok = tok_begin + kTile * k + 16 * fblk + 4 * kg + vi;
      if (tok >= tok_end) v0 = decltype(v0){};
      if (tok + 1 >= tok_end) v1 = decltype(v1){};
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(&sm_v[stage][4 * vh][lane]) + vp;
    if constexpr (KVT == PS_BF16) {
#pragma unroll
      for (int c = 0; c < 4; ++c)   // low (even column) or high (odd column) halves of the two rows: one byte permute
        dst[c * 64 * 4] = __builtin_amdgcn_perm(v1[c >> 1], v0[c >> 1], (c & 1) ? 0x07060302u : 0x05040100u);
    } else {
#pragma unroll
      for (int cp = 0; cp < 2; ++cp) {   // the codes of columns (2 cp, 2 cp + 1) of the two rows, then converted
        const uint32_t pair = __builtin_amdgcn_perm(v1, v0, cp ? 0x07030602u : 0x05010400u);
        dst[(2 * cp) * 64 * 4] = e4m3x2_to_bf16x2(pair, false);
        dst[(2 * cp + 1) * 64 * 4] = e4m3x2_to_bf16x2(pair, true);
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

  // One tile for this wave's rows, operands from the ring.
  // limited_tag: std::true_type applies the per-row limits (and guards rows that have seen nothing yet);
  // std::false_type promises that every row of the wave sees the whole tile.
  struct KOperands { u32x4 a[2][4]; };
  auto read_k = [&](int stage) __attribute__((always_inline)) {   // the 8 K operands of a stage, requested in one go
    KOperands ka;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int st = 0; st < 4; ++st) ka.a[b][st] = sm_k[stage][4 * b + st][lane];
    __builtin_amdgcn_sched_barrier(0);
    return ka;
  };
  struct VOperands { u32x4 a[8]; };
  auto read_v = [&](int stage) __attribute__((always_inline)) {   // the 8 V operands of a stage, requested in one go
    VOperands vt;
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) vt.a[cc] = sm_v[stage][cc][lane];
    __builtin_amdgcn_sched_barrier(0);
    return vt;
  };
  // O^T += V^T P^T, one 16-column group of V at a time
  auto pv = [&](const VOperands& vt, const bf16x8 (&pb)[kNT]) __attribute__((always_inline)) {
#pragma unroll
    for (int cc = 0; cc < 8; ++cc)
#pragma unroll
      for (int t = 0; t < kNT; ++t)
        acc[t][cc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vt.a[cc]), pb[t], acc[t][cc], 0, 0, 0);
  };
  auto multiply = [&](const KOperands& ka, int stage, int k, auto limited_tag) __attribute__((always_inline)) {
    constexpr bool kLimited = decltype(limited_tag)::value;
    const int tok0 = tok_begin + kTile * k;
    float sc_k[2], lvs[2], inv_v[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if constexpr (KVT == PS_FP8_E4M3) {
        const f32x4 q4 = sm_sc[stage][b];
        sc_k[b] = q4.x;
        lvs[b] = q4.y;
        inv_v[b] = q4.z;
      } else {
        sc_k[b] = p.scale_log2;
        lvs[b] = 0.f;
        inv_v[b] = 1.f;
      }
    }
    // raw scores S^T = K Q^T: per row tile two accumulation chains (one per 16-token block)
    f32x4 s[kNT][2];
#pragma unroll
    for (int t = 0; t < kNT; ++t)
#pragma unroll
      for (int b = 0; b < 2; ++b) s[t][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int t = 0; t < kNT; ++t)
          s[t][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka.a[b][st]), qb[t][st], s[t][b], 0, 0, 0);
    // the V operands are requested now, all eight, so that they arrive under the softmax (left to itself the
    // compiler requests each one right before its products, and the wave sits out the LDS latency eight times)
    const VOperands vt = read_v(stage);
    if constexpr (kLimited) {
#pragma unroll
      for (int t = 0; t < kNT; ++t)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (tok0 + 16 * b + 4 * kg + j >= lim[t]) s[t][b][j] = neg_inf;
    }
    // The softmax reference m_run follows the row maximum lazily: it moves (and the accumulators are rescaled)
    // only when some score gets more than kLazy ahead of it, so probabilities stay below 2^kLazy instead of below 1
    // -- the same result by shift invariance of softmax.  The test is local to the lane (its own scores, in log2
    // units; the scales are positive, so a block's maximum scales like its scores) and one vote covers the row
    // tiles; only when it fires somewhere in the wave is the maximum of each row put together across the row's
    // four lanes, which must agree on m_run.  A row that has seen nothing yet has m_run = -inf and stays there
    // until a score arrives.
    // Where no per-row limit applies the test is made on the exponents themselves (score minus reference, which the
    // probabilities need anyway): one exceeds kLazy exactly when its score is that far ahead, and a row that has
    // seen nothing yet (reference -inf) gets +inf there and votes too.  Only the rare branch goes back to the raw
    // scores, and recomputes the exponents against the new reference.
    auto raw_max = [&](int t) { return fmaxf(max_of4(s[t][0]) * sc_k[0], max_of4(s[t][1]) * sc_k[1]); };
    auto move_reference = [&](int t, float mx) __attribute__((always_inline)) {
      float row_mx = fmaxf(mx, lane_xor(mx, 16));
      row_mx = fmaxf(row_mx, lane_xor(row_mx, 32));
      const float m_new = (row_mx > m_run[t] + kLazy) ? row_mx : m_run[t];
      const float alpha = (m_new == m_run[t]) ? 1.f : fast_exp2(m_run[t] - m_new);   // -inf -> finite gives 0
      l_run[t] *= alpha;
#pragma unroll
      for (int cc = 0; cc < 8; ++cc) acc[t][cc] *= alpha;
      m_run[t] = m_new;
    };
    f32x4 e[kNT][2];   // exponents: score in log2 units, plus log2 of the block's V scale, minus the reference
    if constexpr (kLimited) {
      float mx[kNT];
      bool ahead = false;
#pragma unroll
      for (int t = 0; t < kNT; ++t) {
        mx[t] = raw_max(t);
        ahead |= mx[t] > m_run[t] + kLazy;
      }
      if (__builtin_amdgcn_ballot_w64(ahead) != 0) {
#pragma unroll
        for (int t = 0; t < kNT; ++t) move_reference(t, mx[t]);
      }
#pragma unroll
      for (int t = 0; t < kNT; ++t) {
        const float m_ref = (m_run[t] == neg_inf) ? 0.f : m_run[t];   // keeps (-inf) - (-inf) out of the exponents
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int j = 0; j < 4; ++j) e[t][b][j] = __builtin_fmaf(s[t][b][j], sc_k[b], lvs[b] - m_ref);
      }
    } else {
      bool ahead = false;
#pragma unroll
      for (int t = 0; t < kNT; ++t) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int j = 0; j < 4; ++j) e[t][b][j] = __builtin_fmaf(s[t][b][j], sc_k[b], lvs[b] - m_run[t]);
        if constexpr (KVT == PS_BF16) {   // no V scale in the exponents: one fold over both blocks
          const float seed = max_of4(e[t][0]);
          ahead |= fmaxf(fmaxf(fmaxf(fmaxf(seed, e[t][1][0]), e[t][1][1]), e[t][1][2]), e[t][1][3]) > kLazy;
        } else {
          ahead |= (max_of4(e[t][0]) > kLazy + lvs[0]) | (max_of4(e[t][1]) > kLazy + lvs[1]);
        }
      }
      if (__builtin_amdgcn_ballot_w64(ahead) != 0) {
#pragma unroll
        for (int t = 0; t < kNT; ++t) {
          move_reference(t, raw_max(t));
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) e[t][b][j] = __builtin_fmaf(s[t][b][j], sc_k[b], lvs[b] - m_run[t]);
        }
      }
    }
    bf16x8 pb[kNT];
#pragma unroll
    for (int t = 0; t < kNT; ++t) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float lsum = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float pw = fast_exp2(e[t][b][j]);   // probability times the V scale
          lsum += pw;
          pb[t][4 * b + j] = (__bf16)pw;
        }
        l_run[t] += (KVT == PS_FP8_E4M3) ? lsum * inv_v[b] : lsum;
      }
    }
    pv(vt, pb);
  };

  // ---- stream the token range.  In iteration k the wave publishes its share of tile k + 1 (fetched two iterations
  // earlier), requests tile k + 3, multiplies tile k, and meets the others at the barrier: after it tile k + 1 is
  // complete in the ring and nobody reads tile k - 1 any more, whose stage the next iteration overwrites.  No branch
  // surrounds a load, so the counting of outstanding loads stays exact; every wave runs every iteration (and every
  // barrier), whether it has rows or not.
  Fetched fa, fb;
  fetch(fa, fetch_ids(0), 0);
  fetch(fb, fetch_ids(1), 1);
  TileIds ids_nxt = fetch_ids(2);
  publish(fa, 0, 0);
  fetch(fa, ids_nxt, 2);
  ids_nxt = fetch_ids(3);
  __syncthreads();
  int st_cur = 0, st_nxt = 1, st_prv = 2;   // ring stages of tiles k, k + 1, k - 1
  // ids_nxt: the block id of tile k + 3, asked for one iteration ago
  // what_tag: std::false_type / std::true_type = multiply without / with the per-row limits; void* = only fetch
  auto one_tile = [&](int k, Fetched& f_pub, auto what_tag) __attribute__((always_inline)) {
    constexpr bool kMultiply = !std::is_pointer<decltype(what_tag)>::value;
    KOperands ka;
    if constexpr (kMultiply) ka = read_k(st_cur);   // on their way while the wave does its share of the fetching
    publish(f_pub, st_nxt, k + 1);
    fetch(f_pub, ids_nxt, k + 3);
    ids_nxt = fetch_ids(k + 4);
    if constexpr (kMultiply) multiply(ka, st_cur, k, what_tag);
    const int st_free = st_prv;
    st_prv = st_cur;
    st_cur = st_nxt;
    st_nxt = st_free;
    __syncthreads();
  };
  // Two tiles per round, so that the fetch registers keep their roles.  Three loops rather than tests inside one (a
  // branch around the products would have the accumulators copied where its sides meet): the tiles every row of the
  // wave sees whole, then the rest of what the wave sees with the per-row limits (a tile past it is masked out
  // entirely), then the tiles only other waves need.  Every wave passes the same number of barriers.
  // (Measured and dropped, all with parity green: giving the two waves of a SIMD different orders of the steps of a
  // tile -- P V of the tile before first, or the fetching after the products instead of before -- so that they would
  // not ask for the matrix cores at the same time: 5-9 % slower than leaving both in the same order; four-wave
  // workgroups, two per item and per CU, which do not wait for each other but fetch every tile twice: 4 % slower; a
  // four-stage ring with the scores of tile k + 1 issued one matrix instruction at a time between the exponentials
  // of tile k: 9 % slower; a four-stage ring filled two tiles ahead with a barrier every second tile: 6 % slower
  // with bf16 KV, 4 % faster with e4m3.)
  int k = 0;
  for (; k + 2 <= n_whole; k += 2) {
    one_tile(k, fb, std::false_type{});
    one_tile(k + 1, fa, std::false_type{});
  }
  for (; k < n_tiles; k += 2) {
    one_tile(k, fb, std::true_type{});
    one_tile(k + 1, fa, std::true_type{});
  }
  for (; k < n_tiles_wg; k += 2) {
    one_tile(k, fb, static_cast<void*>(nullptr));
    one_tile(k + 1, fa, static_cast<void*>(nullptr));
  }

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
  const dim3 grid(num_items), block(64 * kWaves);
  if (g.kv_dtype == PS_BF16)
    hipLaunchKernelGGL((prefill_attention_kernel<PS_BF16>), grid, block, 0, st, p, items);
  else if (g.kv_dtype == PS_FP8_E4M3)
    hipLaunchKernelGGL((prefill_attention_kernel<PS_FP8_E4M3>), grid, block, 0, st, p, items);
  else
    return PS_ERR_UNSUPPORTED;
  return PS_OK;
}

}  // namespace psdev
