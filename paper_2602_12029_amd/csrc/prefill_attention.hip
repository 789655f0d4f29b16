// Partial-prefill attention on the gfx950 matrix cores: many query rows per KV head against the cached context.
//
// When a context grows by a segment, only the new tokens are prefilled (System Design, execution pipeline step 1):
// every new token is a query row on its context's shared KV, the token at position t seeing the first t + 1
// tokens.  With G q heads per KV head a chunk of c new tokens is c * G rows per KV head -- hundreds, where a decode
// step has a few dozen -- so the work is a dense contraction and the matrix cores, not HBM, are the bound.
//
// One workgroup of eight waves takes one work item: a token range of one context and KV head, and up to 256 query
// rows that see into it.  The rows are split over the waves, 32 each (the query rows resident in registers as MFMA
// B operands), and every wave walks the token range.  Two waves share a SIMD, so that the vector work of one
// (exponentials, conversions) runs under the matrix instructions of the other.
//
// The products are v_mfma_f32_32x32x16_bf16: 32 tokens x 32 rows per instruction.  On this chip it keeps the matrix
// core busy for 32 cycles and the SIMD's vector port for 8 of them, so six plain vector instructions fit into its
// shadow, where the 16x16x32 form (16 cycles, 8 of them on the port) leaves room for two: the same flops take half
// the issue slots, and issue slots are what this kernel runs out of.
//
// K and V reach the waves through LDS, as ready-made A operands: per 32-token tile the eight waves fetch one eighth
// of it each (K straight in operand layout; V as pairs of token rows, transposed inside the lane with one byte
// permute per operand register; e4m3 codes converted to bf16 once), write it to a three-stage ring, and after one
// barrier per tile every wave reads the 8 K and 8 V operands of the tile back, 16 bytes per lane and operand, each
// lane exactly the slot of its own lane index (no bank conflicts).  A tile is thus fetched, transposed and
// converted once per 256 rows.  Global loads run four tiles ahead of the products (two tiles in registers, two in
// LDS), and a tile's K operands are requested from the ring while the tile before it is multiplied.
//
// Per wave and tile: S^T = K Q^T (A = K: lane (m, g) holds elements 16 st + 8 g .. + 7 of token m for k-step st; B =
// Q^T likewise for query row n), whose result leaves lane (n, g) with the scores of row n against tokens
// 8 (r / 4) + 4 g + r % 4, r = 0 .. 15; online softmax with a lazily moving reference; O^T += V^T P^T with the
// probabilities as B operand exactly as they lie (registers 8 ks .. 8 ks + 7 for the 16-token step ks), V^T written
// to the ring so that position j of lane group g in step ks is token 16 ks + 8 (j / 4) + 4 g + j % 4.  A wave skips
// the tiles past what its own rows see; the per-row limit is applied only to tiles that reach past the wave's
// shortest row.  Nothing but the ring is shared between waves: no cross-wave merge, every wave writes the partial
// states of its own rows.
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "mfma_common.h"

namespace psdev {

namespace {

constexpr int kD = kHeadDim;
constexpr int kWaves = 8;         // per workgroup
constexpr int kRowsPerWave = 32;  // one 32-row tile per wave
constexpr int kTile = kTileTokens;
constexpr int kStages = 3;        // LDS ring: tile k read (V), tile k + 1 read (K, one tile ahead), tile k + 2 written
constexpr float kLazy = kLazyRescale;
constexpr float kLazyTop = 256.f;   // 2^kLazy
static_assert(kLazyRescale == 8.f, "kLazyTop is 2^kLazyRescale");

typedef __attribute__((ext_vector_type(16))) float f32x16;

// largest of eight scores, folded from the constant -inf so that three-input maxima do (see max_of4)
__device__ __forceinline__ float max_of8(const f32x16& s, int first) {
  float m = -__builtin_inff();
#pragma unroll
  for (int i = 0; i < 8; ++i) m = fmaxf(m, s[first + i]);
  return m;
}

__device__ __forceinline__ int wave_max(int x) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) x = max(x, __builtin_amdgcn_ds_bpermute(((int(threadIdx.x) & 63) ^ m) << 2, x));
  return __builtin_amdgcn_readfirstlane(x);
}

}  // namespace

template <int KVT>
__global__ __launch_bounds__(64 * kWaves) void prefill_attention_kernel(AttnParams p, const ps_item* __restrict__ items) {
  __shared__ u32x4 sm_k[kStages][8][64];   // [stage][k-step][lane]: K as that lane's A operand
  __shared__ u32x4 sm_v[kStages][8][64];   // [stage][2 * column class + 16-token step][lane]: V^T as that lane's A operand
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
  const int n = lane & 15;   // fetching: token within a 16-token block
  const int kg = lane >> 4;  // fetching: 8-element chunk of a 32-element piece (K), row / column class (V)
  const int g = lane >> 5;   // products: half of a k-step's 16 contraction indices
  const int G = p.group;
  const int rows = n_req * G;
  const int row_base = kRowsPerWave * wave;
  const bool has_rows = rows > row_base;   // a wave without rows only fetches
  const float neg_inf = -__builtin_inff();

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
  int sub_end = (tok_end + 15) >> 4;   // (narrowed below to what some row of the workgroup sees)
  // What this wave fetches of every tile, all of it from one 16-token block (fblk) so that one block id and one
  // buffer descriptor per tile do.  K: token n of the block, elements 32 kst + 8 kg .. + 7 -- that is lane
  // (16 fblk + n, kg % 2) of the operand of k-step 2 kst + kg / 2.  V: the pair of token rows (vrow, vrow + 1), columns
  // 8 n + 4 (kg % 2) + x, x = 0 .. 3 -- the pair is register wave % 4 of lane (n + 16 (kg % 2), kg / 2) = this very
  // lane in the operand of column class x and step fblk; the operand's row lane % 32 is thus column
  // 8 (lane % 16) + 4 (lane / 16 % 2) + x, which the epilogue undoes.
  const int fblk = wave >> 2, kst = wave & 3;
  const int vreg = wave & 3;
  const int vrow = 4 * (kg >> 1) + 8 * ((wave >> 1) & 1) + 2 * (wave & 1);
  const int k_lane_off = n * tok_bytes + (32 * kst + 8 * kg) * kEsz;
  const int v_lane_off = kv_bytes + vrow * tok_bytes + (8 * n + 4 * (kg & 1)) * kEsz;
  const int k_op = 2 * kst + (kg >> 1), k_slot = 16 * fblk + n + 32 * (kg & 1);
  // (constant address space: the table is read-only for the kernel's lifetime, which keeps the load a scalar one
  // whatever stands around it)
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr blk_seg = (const_i32_ptr)(p.blk + blk_off);

  struct TileIds { int id; };   // of this wave's block of the tile
  auto fetch_ids = [&](int k) __attribute__((always_inline)) {   // wave-uniform
    // no branch around this load (the index is clamped into the range instead), so that the counting of
    // outstanding loads in the streaming loop stays exact; a block past the range is never fetched from
    TileIds r;
    const int sub = max(sub0, min(sub0 + 2 * k + fblk, sub_end - 1));
    r.id = blk_seg[sub >> sub_shift];
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
  // The first two tiles and the block ids of the next two are requested at once, from the item's header alone: what
  // the rows see (request list -> visible lengths) is another two round trips to memory, which these need not wait for.
  Fetched fa, fb;
  fetch(fa, fetch_ids(0), 0);
  fetch(fb, fetch_ids(1), 1);
  const TileIds ids2 = fetch_ids(2), ids3 = fetch_ids(3);

  // ---- this lane's query row (row lane % 32 of the wave): request, visible length, and the row itself as the
  // eight B operands of S^T = K Q^T (k-step st, lane group g: elements 16 st + 8 g .. + 7)
  int req_of = -1, lim = 0;   // a padding row sees nothing
  bf16x8 qb[8];
#pragma unroll
  for (int st = 0; st < 8; ++st) qb[st] = as_bf16x8(u32x4{0, 0, 0, 0});
  int lim_hi = 0, lim_lo = 0x7fffffff;
  {
    const int row = row_base + (lane & 31);
    if (row < rows) {
      const int req = p.req_list[req_off + row / G];
      req_of = req;
      lim = limited ? min(tok_end, p.visible[req]) : tok_end;
      const uint16_t* qrow = static_cast<const uint16_t*>(p.q) + (int64_t(req) * p.num_q_heads + kv_head * G + row % G) * kD;
#pragma unroll
      for (int st = 0; st < 8; ++st) qb[st] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 16 * st + 8 * g));
      lim_hi = lim;
      lim_lo = lim;
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
  const int n_tiles = has_rows ? (see_end - tok_begin + kTile - 1) / kTile : 0;   // tiles this wave multiplies
  const int n_whole = min(n_tiles, max(0, (see_all - tok_begin) / kTile));   // ... of which these need no per-row limit

  sub_end = (see_end_wg + 15) >> 4;   // blocks past it are not fetched: nobody sees them

  // ... and its way into the ring: K as it is (e4m3: converted), V transposed -- register vreg of this lane's slot
  // in the operand of column class x holds column 8 n + 4 (kg % 2) + x of the token rows (vrow, vrow + 1)
  // ragged_tag: std::true_type = the tile may be the item's last, which can reach past its range
  auto publish = [&](const Fetched& f, int stage, int k, auto ragged_tag) __attribute__((always_inline)) {
    if constexpr (KVT == PS_BF16) {
      sm_k[stage][k_op][k_slot] = f.k;
    } else {
      sm_k[stage][k_op][k_slot] = e4m3x8_to_bf16x8(f.k.x, f.k.y);
      // the block's scales, once per workgroup: the K scale folded into the score scale, the V scale as the exponent
      // offset of the probabilities and as the factor that takes it out of the row sums again
      if (kst == 0 && lane == 0) {
        const float lv = __builtin_amdgcn_logf(f.sc.y);
        sm_sc[stage][fblk] = f32x4{p.scale_log2 * f.sc.x, lv, fast_exp2(-lv), 0.f};
      }
    }
    // slots of tokens past the item's range may hold anything: zero them (their probabilities are zero)
    auto v0 = f.v[0], v1 = f.v[1];
    if (decltype(ragged_tag)::value && tok_begin + kTile * (k + 1) > tok_end) {   // (only the item's last tile can)
      const int tok = tok_begin + kTile * k + 16 * fblk + vrow;
      if (tok >= tok_end) v0 = decltype(v0){};
      if (tok + 1 >= tok_end) v1 = decltype(v1){};
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(&sm_v[stage][fblk][lane]) + vreg;   // operand 2 x + fblk
    if constexpr (KVT == PS_BF16) {
#pragma unroll
      for (int x = 0; x < 4; ++x)   // low (even column) or high (odd column) halves of the two rows: one byte permute
        dst[x * 2 * 64 * 4] = __builtin_amdgcn_perm(v1[x >> 1], v0[x >> 1], (x & 1) ? 0x07060302u : 0x05040100u);
    } else {
#pragma unroll
      for (int cp = 0; cp < 2; ++cp) {   // the codes of columns (2 cp, 2 cp + 1) of the two rows, then converted
        const uint32_t pair = __builtin_amdgcn_perm(v1, v0, cp ? 0x07030602u : 0x05010400u);
        dst[(2 * cp) * 2 * 64 * 4] = e4m3x2_to_bf16x2(pair, false);
        dst[(2 * cp + 1) * 2 * 64 * 4] = e4m3x2_to_bf16x2(pair, true);
      }
    }
  };

  float m_run = neg_inf, l_run = 0.f;
  f32x16 acc[4];   // O^T, one block of 32 columns per column class
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[x][r] = 0.f;

  // One tile for this wave's rows, operands from the ring.
  // limited_tag: std::true_type applies the per-row limits (and guards rows that have seen nothing yet);
  // std::false_type promises that every row of the wave sees the whole tile.
  struct KOperands { u32x4 a[8]; };
  auto read_k = [&](int stage) __attribute__((always_inline)) {   // the 8 K operands of a stage, requested in one go
    KOperands ka;
#pragma unroll
    for (int st = 0; st < 8; ++st) ka.a[st] = sm_k[stage][st][lane];
    __builtin_amdgcn_sched_barrier(0);
    return ka;
  };
  struct VOperands { u32x4 a[8]; };
  auto read_v = [&](int stage) __attribute__((always_inline)) {   // the 8 V operands of a stage, requested in one go
    VOperands vt;
#pragma unroll
    for (int op = 0; op < 8; ++op) vt.a[op] = sm_v[stage][op][lane];
    __builtin_amdgcn_sched_barrier(0);
    return vt;
  };
  // O^T += V^T P^T: the two 16-token steps of the tile, one column class at a time
  auto pv = [&](const VOperands& vt, const bf16x8 (&pb)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int x = 0; x < 4; ++x)
        acc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vt.a[2 * x + ks]), pb[ks], acc[x], 0, 0, 0);
  };
  // raw scores S^T = K Q^T: register r of this lane = its row against token 8 (r / 4) + 4 g + r % 4 of the tile
  // (registers 0 .. 7 the first 16-token block, 8 .. 15 the second)
  auto scores = [&](const KOperands& ka) __attribute__((always_inline)) {
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int st = 0; st < 8; ++st) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka.a[st]), qb[st], s, 0, 0, 0);
    return s;
  };
  // softmax of a tile's scores and its P V products
  auto finish = [&](f32x16 s, const VOperands& vt, int stage, int k, auto limited_tag) __attribute__((always_inline)) {
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
    if constexpr (kLimited) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (tok0 + 8 * (r >> 2) + 4 * g + (r & 3) >= lim) s[r] = neg_inf;
    }
    // The softmax reference m_run follows the row maximum lazily: it moves (and the accumulators are rescaled)
    // only when some score gets far ahead of it, so probabilities stay below 2^kLazy instead of below 1 -- the same
    // result by shift invariance of softmax.  The test is local to the lane and one wave vote decides; only when it
    // fires somewhere in the wave is the maximum of the row put together across the row's two lanes, which must
    // agree on m_run.  A row that has seen nothing yet has m_run = -inf and stays there until a score arrives.
    auto raw_max = [&]() { return fmaxf(max_of8(s, 0) * sc_k[0], max_of8(s, 8) * sc_k[1]); };
    auto move_reference = [&](float mx, float ahead_by) __attribute__((always_inline)) {
      const float row_mx = fmaxf(mx, lane_xor(mx, 32));
      const float m_new = (row_mx > m_run + ahead_by) ? row_mx : m_run;
      const float alpha = (m_new == m_run) ? 1.f : fast_exp2(m_run - m_new);   // -inf -> finite gives 0
      l_run *= alpha;
#pragma unroll
      for (int x = 0; x < 4; ++x) acc[x] *= alpha;
      m_run = m_new;
    };
    f32x16 e;   // exponents: score in log2 units, plus log2 of the block's V scale, minus the reference
    float pw[16], lsum[2];   // probabilities times the V scale; their sums per block
    auto probabilities = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        lsum[b] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          pw[8 * b + j] = fast_exp2(e[8 * b + j]);
          lsum[b] += pw[8 * b + j];
        }
      }
    };
    float total;   // this lane's 16 probabilities, summed
    if constexpr (kLimited) {
      // per-row limits: the test is made on the raw scores (in log2 units; the scales are positive, so a block's
      // maximum scales like its scores)
      const float mx = raw_max();
      if (__builtin_amdgcn_ballot_w64(mx > m_run + kLazy) != 0) move_reference(mx, kLazy);
      const float m_ref = (m_run == neg_inf) ? 0.f : m_run;   // keeps (-inf) - (-inf) out of the exponents
#pragma unroll
      for (int r = 0; r < 16; ++r) e[r] = __builtin_fmaf(s[r], sc_k[r >> 3], lvs[r >> 3] - m_ref);
      probabilities();
      total = (KVT == PS_FP8_E4M3) ? lsum[0] * inv_v[0] + lsum[1] * inv_v[1] : lsum[0] + lsum[1];
    } else {
      // Every row sees the whole tile: the test is made on the sum of the lane's probabilities, which the row sum
      // needs anyway -- a probability above 2^kLazy (or an infinite one: a row that has seen nothing yet has the
      // reference -inf) shows in it, and a sum above 2^kLazy means that one of its 16 terms is above 2^(kLazy - 4),
      // so in the rare branch the reference moves for every row that is that far ahead, after which the row's
      // probabilities are at most 1 and the test is quiet again.  No maximum is taken on the common path.
#pragma unroll
      for (int r = 0; r < 16; ++r) e[r] = __builtin_fmaf(s[r], sc_k[r >> 3], lvs[r >> 3] - m_run);
      probabilities();
      total = (KVT == PS_FP8_E4M3) ? lsum[0] * inv_v[0] + lsum[1] * inv_v[1] : lsum[0] + lsum[1];
      if (__builtin_amdgcn_ballot_w64(!(total <= kLazyTop)) != 0) {
        move_reference(raw_max(), kLazy - 4.f);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] = __builtin_fmaf(s[r], sc_k[r >> 3], lvs[r >> 3] - m_run);
        probabilities();
        total = (KVT == PS_FP8_E4M3) ? lsum[0] * inv_v[0] + lsum[1] * inv_v[1] : lsum[0] + lsum[1];
      }
    }
    l_run += total;
    bf16x8 pb[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int j = 0; j < 8; ++j) pb[b][j] = (__bf16)pw[8 * b + j];
    pv(vt, pb);
  };

  // ---- stream the token range.  The ring holds three tiles: in iteration k the wave multiplies tile k (its K
  // operands already in registers, requested during iteration k - 1), requests the K operands of tile k + 1 (complete
  // in the ring since the last barrier), publishes its share of tile k + 2 (fetched two iterations earlier) into the
  // stage tile k - 1 left, requests tile k + 4 from memory, and meets the others at the barrier.  The products of a
  // tile thus start right behind the barrier instead of waiting for operands that all eight waves ask for at once.
  // No branch surrounds a load, so the counting of outstanding loads stays exact; every wave runs every iteration
  // (and every barrier), whether it has rows or not.
  publish(fa, 0, 0, std::true_type{});
  fetch(fa, ids2, 2);
  publish(fb, 1, 1, std::true_type{});
  fetch(fb, ids3, 3);
  TileIds ids_nxt = fetch_ids(4);   // the block id of tile k + 4, asked for one iteration ahead
  __syncthreads();
  int st_cur = 0, st_nxt = 1, st_wr = 2;   // ring stages of tiles k, k + 1, k + 2
  KOperands ka_even, ka_odd;               // K operands of the even / odd tile in flight
  if (n_tiles > 0) ka_even = read_k(0);
  // what_tag: std::false_type / std::true_type = multiply without / with the per-row limits; void* = only fetch
  auto one_tile = [&](int k, Fetched& f_pub, const KOperands& ka, KOperands& ka_next, auto what_tag,
                      auto ragged_tag) __attribute__((always_inline)) {
    constexpr bool kMultiply = !std::is_pointer<decltype(what_tag)>::value;
    // (the fetching stands in front of the score products in program order and the compiler weaves it into them:
    // a wave issues in order, so vector work finds room under matrix instructions only between them -- with the
    // products first and everything else behind a scheduling barrier the kernel is 3-13 % slower)
    if constexpr (kMultiply) ka_next = read_k(st_nxt);   // on their way while this tile is multiplied
    publish(f_pub, st_wr, k + 2, ragged_tag);
    fetch(f_pub, ids_nxt, k + 4);
    ids_nxt = fetch_ids(k + 5);
    if constexpr (kMultiply) {
      const f32x16 s = scores(ka);
      // the V operands are requested now, all eight, so that they arrive under the softmax (left to itself the
      // compiler requests each one right before its products, and the wave sits out the LDS latency eight times)
      const VOperands vt = read_v(st_cur);
      finish(s, vt, st_cur, k, what_tag);
    }
    const int st_free = st_cur;
    st_cur = st_nxt;
    st_nxt = st_wr;
    st_wr = st_free;
    __syncthreads();
  };
  // Two tiles per round, so that the fetch and operand registers keep their roles.  Three loops rather than tests
  // inside one (a branch around the products would have the accumulators copied where its sides meet): the tiles
  // every row of the wave sees whole, then the rest of what the wave sees with the per-row limits (a tile past it
  // is masked out entirely), then the tiles only other waves need.  Every wave passes the same number of barriers.
  // (Measured and dropped, all with parity green: giving the two waves of a SIMD different orders of the steps of a
  // tile, or different priorities -- whichever phase or wave is favoured, 15-30 % slower than equal priorities;
  // four-wave workgroups, two per item and per CU, which do not wait for each other but fetch every tile twice: 4 %
  // slower; the scores of tile k + 1 issued one matrix instruction at a time between the exponentials of tile k: 9 %
  // slower with the 16x16x32 products, and with the 32x32x16 ones, where the compiler weaves the two by itself, 2 %
  // faster with bf16 KV and 4 % slower with e4m3 than requesting the K operands a tile ahead, which the registers
  // do not allow next to it; four waves of 64 rows, one per SIMD, every operand read feeding two matrix instructions:
  // 18-29 % slower, a wave alone on its SIMD has nobody to cover its waits.)
  // (the first loop also stops short of the item's last complete tiles, so that the tiles it publishes -- two and
  // three ahead -- are complete ones and need no zeroing of rows past the range)
  const int n_fast = min(n_whole, (tok_end - tok_begin) / kTile - 2);
  int k = 0;
  for (; k + 2 <= n_fast; k += 2) {
    one_tile(k, fa, ka_even, ka_odd, std::false_type{}, std::false_type{});
    one_tile(k + 1, fb, ka_odd, ka_even, std::false_type{}, std::false_type{});
  }
  for (; k < n_tiles; k += 2) {
    one_tile(k, fa, ka_even, ka_odd, std::true_type{}, std::true_type{});
    one_tile(k + 1, fb, ka_odd, ka_even, std::true_type{}, std::true_type{});
  }
  for (; k < n_tiles_wg; k += 2) {
    one_tile(k, fa, ka_even, ka_odd, static_cast<void*>(nullptr), std::true_type{});
    one_tile(k + 1, fb, ka_odd, ka_even, static_cast<void*>(nullptr), std::true_type{});
  }

  // ---- one partial state per row, straight from the accumulators: register r of column class x is column
  // 64 (r / 4 % 2) + 32 g + 8 (r % 4) + 4 (r / 8) + x of this lane's row
  if (has_rows) {
    float l = l_run;
    l += lane_xor(l, 32);
    if (req_of >= 0) {
      const float inv = l > 0.f ? 1.f / l : 0.f;
      const int row = row_base + (lane & 31);
      const int h = kv_head * G + row % G;
      const int64_t slot = int64_t(p.slot_base[req_of]) + split_local;
      float* o = p.ws_o + (slot * p.num_q_heads + h) * kD + 32 * g;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        *reinterpret_cast<f32x4*>(o + 64 * ((r >> 2) & 1) + 8 * (r & 3) + 4 * (r >> 3)) =
            f32x4{acc[0][r], acc[1][r], acc[2][r], acc[3][r]} * inv;
      if (g == 0)
        p.ws_lse[slot * p.num_q_heads + h] = l > 0.f ? (m_run + __builtin_amdgcn_logf(l)) * kLn2 : neg_inf;
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
