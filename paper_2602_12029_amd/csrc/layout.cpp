// Host side of the library: block pool, the refcounted two-segment block table (ps_kv_layout) and
// the split plan.  Pure C++ -- no HIP calls -- so it is testable without a GPU.
//
// Sharing rule implemented here: a prompt's prefix blocks are allocated once and referenced by every
// request on that prompt (each decode module starts from the same base cache, Method Eq. 6), and
// only the model-specific segment is private (Efficiency Analysis Eq. 9).
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <map>
#include <tuple>
#include <new>
#include <numeric>
#include <queue>
#include <set>
#include <utility>

#include "ps_internal.h"

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

int32_t check_geometry(const ps_geometry& g) {
  if (g.num_q_heads <= 0 || g.num_kv_heads <= 0 || g.head_dim <= 0 || g.block_size <= 0) return PS_ERR_SHAPE;
  if (g.num_q_heads % g.num_kv_heads != 0) return PS_ERR_SHAPE;
  if (g.q_dtype != PS_F32 && g.q_dtype != PS_BF16) return PS_ERR_UNSUPPORTED;
  if (g.kv_dtype != PS_F32 && g.kv_dtype != PS_BF16 && g.kv_dtype != PS_FP8_E4M3) return PS_ERR_UNSUPPORTED;
  const int64_t esz = g.kv_dtype == PS_F32 ? 4 : (g.kv_dtype == PS_BF16 ? 2 : 1);
  const int64_t strides[4] = {g.kv_stride_block, g.kv_stride_head, g.kv_stride_kv, g.kv_stride_tok};
  for (int64_t s : strides)
    if (s <= 0 || (s * esz) % 16 != 0) return PS_ERR_SHAPE;
  if (g.kv_stride_tok < g.head_dim) return PS_ERR_SHAPE;
  return PS_OK;
}

}  // namespace

int32_t (*ps_device_num_cus_hook)() = nullptr;

bool ps_mfma_supported(const ps_geometry& g) {
  // The matrix-core kernels address a (block, head) slice through a buffer descriptor with 32-bit byte offsets
  // (V plane + token row + column), so the slice must span less than 2 GiB; a pool with K and V planes further
  // apart than that goes to the wavefront kernel, which computes 64-bit addresses.
  const int64_t esz = g.kv_dtype == PS_BF16 ? 2 : 1;
  const int64_t slice_span = (g.kv_stride_kv + int64_t(g.block_size) * g.kv_stride_tok) * esz;
  return g.q_dtype == PS_BF16 && (g.kv_dtype == PS_BF16 || g.kv_dtype == PS_FP8_E4M3) && g.head_dim == 128 &&
         g.block_size % 16 == 0 && ((g.block_size / 16) & (g.block_size / 16 - 1)) == 0 &&  // 16, 32, 64, ...
         (g.num_q_heads / g.num_kv_heads) <= 64 && slice_span < (int64_t(1) << 31);
}

// ---------------------------------------------------------------------------------------------------
// Split plan: cut every segment into token chunks of (nearly) equal size, one workgroup each; a
// request's partial states are numbered prefix chunks first, then its suffix chunks.
int32_t ps_plan_build(ps_layout* lay, const ps_plan_options* user) {
  ps_plan_options opt{};
  if (user) opt = *user;
  if (opt.prefix_chunk_tokens < 0 || opt.suffix_chunk_tokens < 0 || opt.num_cus < 0) return PS_ERR_INVALID_ARG;
  auto bad_variant = [](int32_t v) { return v != PS_VARIANT_AUTO && v != PS_VARIANT_WAVE && v != PS_VARIANT_MFMA; };
  if (bad_variant(opt.prefix_variant) || bad_variant(opt.suffix_variant)) return PS_ERR_INVALID_ARG;
  if (opt.kv_cache_policy < PS_KV_POLICY_AUTO || opt.kv_cache_policy > PS_KV_POLICY_CACHEABLE) return PS_ERR_INVALID_ARG;
  const ps_geometry& g = lay->geo;
  const bool mfma_ok = ps_mfma_supported(g);
  if ((opt.prefix_variant == PS_VARIANT_MFMA || opt.suffix_variant == PS_VARIANT_MFMA) && !mfma_ok)
    return PS_ERR_UNSUPPORTED;
  const int32_t group = g.num_q_heads / g.num_kv_heads;
  // compute units to spread the work over: the caller's figure, else the current device's, else MI355X's
  int32_t num_cus = opt.num_cus;
  if (num_cus == 0 && ps_device_num_cus_hook) num_cus = ps_device_num_cus_hook();
  if (num_cus <= 0) num_cus = kPsDefaultNumCus;

  // chunk boundaries fall on block boundaries and on the 32-token MFMA tile
  const int64_t granule = std::lcm<int64_t>(g.block_size, 32);
  int64_t total = 0;
  for (int32_t l : lay->prefix_len) total += l;
  for (int32_t l : lay->suffix_len) total += l;
  for (int32_t l : lay->root_len) total += l;
  total *= g.num_kv_heads;
  // Aim for about one full-size chunk per compute unit: long items amortise the per-item merge and keep
  // the number of partial states (workspace traffic) low; the many small suffix items fill the gaps.  Where the
  // kernel runs two workgroups per compute unit the aim is 0.6 of that, 1.2 times a workgroup's share: with
  // segments of unequal lengths the heaviest workgroups otherwise run on alone at the end of the launch (measured on
  // 20 to 60 concurrent sessions with contexts of 1024 to 6144 tokens: 2 to 10 % faster, none slower by more than
  // 0.5 %; any factor from 0.5 to 0.8 does about as well).
  // Shared segments of (nearly) equal lengths are cut as before: whole segments then pair up evenly on the compute
  // units by themselves, and the 4096-token prefixes of the 8B-shaped configuration are 2-3 % slower in halves.
  int32_t widest = group;   // rows of the widest item per KV head, for the kernel's residency
  {
    const int32_t cap = (g.kv_dtype == PS_FP8_E4M3 ? 32 : 64) / group;   // requests per item (see max_req below)
    for (size_t p = 0; p + 1 < lay->group_indptr.size(); ++p)
      widest = std::max(widest, std::min(std::max(1, cap), lay->group_indptr[p + 1] - lay->group_indptr[p]) * group);
    for (size_t t = 0; t + 1 < lay->root_group_indptr.size(); ++t)
      widest = std::max(widest, std::min(std::max(1, cap), lay->root_group_indptr[t + 1] - lay->root_group_indptr[t]) * group);
  }
  const bool two_per_cu = mfma_ok && ps_mfma_occupancy(widest, g.kv_dtype) == 2;
  int32_t shortest = INT32_MAX, longest = 0;   // of the shared segments
  for (int32_t l : lay->prefix_len) { shortest = std::min(shortest, l); longest = std::max(longest, l); }
  const bool unequal = longest > 0 && int64_t(longest) * 10 > int64_t(shortest) * 11;
  const int64_t ideal = std::max<int64_t>(1, ceil_div(two_per_cu && unequal ? total * 3 / 5 : total, int64_t(num_cus)));
  auto pick = [&](int32_t asked) -> int64_t {
    if (asked > 0) return round_up(asked, granule);
    return std::min<int64_t>(std::max<int64_t>(round_up(ideal, granule), round_up(256, granule)), round_up(kPsMfmaMaxChunk, granule));
  };
  auto resolve = [&](int32_t v) { return v == PS_VARIANT_AUTO ? (mfma_ok ? PS_VARIANT_MFMA : PS_VARIANT_WAVE) : v; };
  const int64_t mfma_cap = std::max<int64_t>(granule, kPsMfmaMaxChunk / granule * granule);
  int64_t prefix_chunk = pick(opt.prefix_chunk_tokens);
  int64_t suffix_chunk = pick(opt.suffix_chunk_tokens);
  if (resolve(opt.prefix_variant) == PS_VARIANT_MFMA) prefix_chunk = std::min(prefix_chunk, mfma_cap);
  if (resolve(opt.suffix_variant) == PS_VARIANT_MFMA) suffix_chunk = std::min(suffix_chunk, mfma_cap);

  lay->opt = opt;
  lay->prefix_variant = resolve(opt.prefix_variant);
  lay->suffix_variant = resolve(opt.suffix_variant);
  lay->prefix_chunk = int32_t(prefix_chunk);
  lay->suffix_chunk = int32_t(suffix_chunk);

  // equal-sized chunks of a segment of `len` tokens: returns the chunk size used
  auto chunking = [&](int64_t len, int64_t chunk, int32_t* n) -> int64_t {
    if (len <= 0) { *n = 0; return chunk; }
    const int64_t count = ceil_div(len, chunk);
    const int64_t size = round_up(ceil_div(len, count), granule);
    *n = int32_t(ceil_div(len, size));
    return size;
  };
  // ... of a shared segment that goes to the prefill kernel: one that is only a little longer than a number of chunks
  // (by up to a quarter chunk) is not cut once more -- two halves of a context just over the aim cost an item, a
  // partial state per row and a merge more than they balance (partial-prefill batches whose contexts straddle the
  // aim: 7 % faster whole; decode batches of 60-80 sessions 1-2 % slower with the same rule, so they keep the plain
  // one).
  // (the prefill kernel walks a range of any length -- one scalar block id per tile -- so its items are not held to
  // the persistent kernel's 64 tiles per wave: the aim for them is the uncapped share, at most 32768 tokens)
  const int64_t wide_chunk = opt.prefix_chunk_tokens > 0 ? prefix_chunk
                             : std::min<int64_t>(std::max<int64_t>(round_up(ideal, granule), round_up(256, granule)), round_up(32768, granule));
  auto chunking_shared = [&](int64_t len, int64_t chunk, int32_t* n) -> int64_t {
    if (len <= 0) { *n = 0; return chunk; }
    if (opt.prefix_chunk_tokens > 0) return chunking(len, chunk, n);   // a chunk size the caller asked for is taken as it is
    const int64_t count = std::max<int64_t>(1, ceil_div(len - chunk / 4, chunk));
    const int64_t size = round_up(ceil_div(len, count), granule);
    *n = int32_t(ceil_div(len, size));
    return size;
  };

  const int32_t P = lay->num_prompts, R = lay->num_requests;
  // Visible prefix lengths (partial prefill: a query row may see only the leading part of its prompt's shared
  // prefix).  A request takes part in the prefix chunks that begin below its visible length, so its prefix splits
  // are the first ceil(visible / chunk size) of its prompt's; an item's token range ends at the largest visible
  // length among its rows, and it is marked where some row sees less than that.
  const bool limited = !lay->visible.empty();
  auto visible_of = [&](int32_t r) { return limited ? lay->visible[size_t(r)] : lay->prefix_len[size_t(lay->req_prompt[size_t(r)])]; };
  std::vector<int32_t> nsplit_root(R, 0), nsplit_prefix(R), nsplit_suffix(R);
  lay->suffix_chunk_size.assign(size_t(R), 0);
  lay->suffix_chunks.assign(size_t(R), 0);
  std::vector<ps_item> prefix_items, suffix_items;
  // Rows an item carries per KV head: up to 64 (four row tiles).  With e4m3 KV a sharing group is cut at 32 rows where
  // the matrix-core kernel runs: the two-tile kernel keeps two workgroups per compute unit and measured 19 % faster
  // on 64-row groups than the four-tile one (bf16 KV the other way round: the four-tile kernel is 9-12 % faster).
  const bool narrow_items = g.kv_dtype == PS_FP8_E4M3 && resolve(opt.prefix_variant) == PS_VARIANT_MFMA;
  const int32_t max_req = std::max(1, (narrow_items ? 32 : 64) / group);
  const int32_t total_prefix_blocks = int32_t(lay->prefix_blk.size());
  lay->max_rows_prefix = 0;
  lay->any_masked = false;
  lay->req_list.assign(lay->group_req.begin(), lay->group_req.end());
  for (int32_t r = 0; r < R; ++r) lay->req_list.push_back(r);
  lay->req_list.insert(lay->req_list.end(), lay->root_group_req.begin(), lay->root_group_req.end());
  const bool prefix_mfma = resolve(opt.prefix_variant) == PS_VARIANT_MFMA;
  // Root segments: read whole by every request below the root (all models of all its prompts), so the sharing group
  // is large.  In a decode batch it goes out in ordinary items of at most 64 rows, packed into the one persistent
  // launch with everything else (the root's K/V is then fetched once per 64 rows, mostly from the last-level cache;
  // a separate launch for a handful of root items would leave most of the chip idle while it runs).  In a
  // partial-prefill batch (visible lengths set) large groups go to the prefill kernel, roots included.
  const int32_t root_blk0 = int32_t(lay->prefix_blk.size() + lay->suffix_blk.size());   // roots close the block array
  lay->planned_root_blk0 = root_blk0;
  for (int32_t t = 0; t < lay->num_roots; ++t) {
    int32_t n = 0;
    const int32_t g0 = lay->root_group_indptr[size_t(t)], count = lay->root_group_indptr[size_t(t) + 1] - g0;
    const bool wide = limited && prefix_mfma && int64_t(count) * group > 64;
    // (a root is seen whole by every request below it, so all its chunks go the same way)
    const int64_t size = wide ? chunking_shared(lay->root_len[size_t(t)], wide_chunk, &n) : chunking(lay->root_len[size_t(t)], prefix_chunk, &n);
    for (int32_t i = 0; i < count; ++i) nsplit_root[size_t(lay->root_group_req[size_t(g0 + i)])] = n;
    const bool row_split = limited && prefix_mfma && int64_t(count) * group > 64;
    const int32_t per_item = row_split ? std::max(1, 256 / group) : max_req;
    // Row groups outside, KV heads inside: items of equal cost reach the workgroups in this order (LPT, lowest
    // index on ties) and workgroup i runs on XCD i mod 8, so with a multiple of eight KV heads the row groups that
    // read one (range, head) start together on one XCD and share its L2.
    for (int32_t c = 0; c < n; ++c)
      for (int32_t m0 = 0; m0 < count; m0 += per_item)
        for (int32_t h = 0; h < g.num_kv_heads; ++h) {
          ps_item it{};
          it.blk_off = root_blk0 + lay->root_blk_indptr[size_t(t)];
          it.tok_begin = int32_t(c * size);
          it.tok_end = int32_t(std::min<int64_t>(lay->root_len[size_t(t)], (c + 1) * size));
          it.req_off = 2 * R + g0 + m0;
          it.n_req = std::min(per_item, count - m0);
          it.kv_head = h;
          it.split_local = c;
          it.kind = kPsItemRoot | (row_split ? kPsItemRowSplit : 0) | (count > per_item ? kPsItemReread : 0);
          if (!row_split) lay->max_rows_prefix = std::max(lay->max_rows_prefix, it.n_req * group);
          prefix_items.push_back(it);
        }
  }
  // The prefill kernel runs one workgroup per item, one item per compute unit at a time, and its items are long: with
  // a few items per compute unit the last round of the launch is badly filled (704 items of 132 tiles on 256 compute
  // units: three rounds for the work of 2.75).  The contexts whose items come last -- the shortest, the launch goes
  // heaviest first -- are therefore cut into more pieces, as many as fill the last round best; the others stay whole
  // (one partial state per row).
  std::vector<int32_t> tail_cut(size_t(P), 1);
  if (limited && prefix_mfma && opt.prefix_chunk_tokens == 0) {
    struct wide_prompt { int32_t p; int64_t items, tiles; };
    std::vector<wide_prompt> wp;
    int64_t n_items = 0, work = 0;
    for (int32_t p = 0; p < P; ++p) {
      const int64_t reqs = lay->group_indptr[p + 1] - lay->group_indptr[p];
      if (reqs * group <= 64 || lay->prefix_len[p] <= 0) continue;
      int32_t n0 = 0;
      const int64_t size0 = chunking_shared(lay->prefix_len[p], wide_chunk, &n0);
      const int64_t per_item = std::max(1, 256 / group);
      const wide_prompt e{p, ceil_div(reqs, per_item) * g.num_kv_heads * n0, ceil_div(std::min<int64_t>(size0, lay->prefix_len[p]), 32)};
      wp.push_back(e);
      n_items += e.items;
      work += e.items * e.tiles;
    }
    if (n_items > 0) {
      const int64_t mean_tiles = std::max<int64_t>(1, work / n_items);
      const int64_t rounds = work / num_cus / mean_tiles;          // rounds the whole items fill completely
      const int64_t rest = n_items - rounds * num_cus;             // items of the last, partly filled round
      // time of the last round in tiles, an item costing about twelve tiles beyond its own (launch, the dependent
      // reads of its start, filling the ring, its stores; measured: pieces of 33 tiles gained nothing on 132-tile items)
      constexpr int64_t kItemOverheadTiles = 12;
      int64_t best_cut = 1, best_cost = INT64_MAX, whole_cost = 0;
      for (int64_t cut : {1, 2, 3, 4, 6, 8}) {
        if (mean_tiles / cut < 16) break;                          // pieces of at least 512 tokens
        const int64_t cost = ceil_div(rest * cut, int64_t(num_cus)) * (ceil_div(mean_tiles, cut) + kItemOverheadTiles);
        if (cut == 1) whole_cost = cost;
        if (cost < best_cost) { best_cost = cost; best_cut = cut; }
      }
      // (worth it from 3 % of a compute unit's work on: the pieces cost their rows a partial state and a merge each)
      if (rest > 0 && best_cut > 1 && (whole_cost - best_cost) * 100 >= 3 * (work / num_cus)) {
        std::stable_sort(wp.begin(), wp.end(), [](const wide_prompt& x, const wide_prompt& y) { return x.tiles < y.tiles; });
        int64_t taken = 0;
        for (size_t i = 0; i < wp.size() && taken < rest; ++i) {
          tail_cut[size_t(wp[i].p)] = int32_t(best_cut);
          taken += wp[i].items;
        }
      }
    }
  }
  std::vector<int32_t> members;
  for (int32_t p = 0; p < P; ++p) {
    int32_t n = 0;
    const int32_t g0 = lay->group_indptr[p], g1 = lay->group_indptr[p + 1];
    const bool wide = limited && prefix_mfma && int64_t(g1 - g0) * group > 64;   // goes to the prefill kernel
    int64_t size = wide ? chunking_shared(lay->prefix_len[p], wide_chunk, &n) : chunking(lay->prefix_len[p], prefix_chunk, &n);
    if (wide && tail_cut[size_t(p)] > 1 && n > 0) {
      size = round_up(ceil_div(int64_t(lay->prefix_len[p]), int64_t(n) * tail_cut[size_t(p)]), granule);
      n = int32_t(ceil_div(int64_t(lay->prefix_len[p]), size));
    }
    if (size > mfma_cap && prefix_mfma) {
      // chunks longer than the persistent kernel's items hold are fine only while every one of them goes to the
      // prefill kernel: a chunk that too few requests see into (64 rows or fewer) would be an ordinary item
      for (int32_t c = 0; c < n && size > mfma_cap; ++c) {
        int64_t seen_by = 0;
        for (int32_t i = g0; i < g1; ++i) seen_by += visible_of(lay->group_req[size_t(i)]) > c * size;
        if (seen_by * group <= 64) size = chunking(lay->prefix_len[p], prefix_chunk, &n);
      }
    }
    for (int32_t i = g0; i < g1; ++i) {
      const int32_t r = lay->group_req[size_t(i)];
      nsplit_prefix[size_t(r)] = int32_t(ceil_div(visible_of(r), size));
    }
    for (int32_t c = 0; c < n; ++c) {
      // the requests that see into this chunk, in group order: the whole group unless lengths were limited
      int32_t list0 = g0, count = g1 - g0;
      if (limited) {
        members.clear();
        for (int32_t i = g0; i < g1; ++i)
          if (visible_of(lay->group_req[size_t(i)]) > c * size) members.push_back(lay->group_req[size_t(i)]);
        count = int32_t(members.size());
        if (count != g1 - g0) {
          list0 = int32_t(lay->req_list.size());
          lay->req_list.insert(lay->req_list.end(), members.begin(), members.end());
        }
      }
      // Partial prefill on the matrix cores: a sharing group with more rows than one 64-row item holds (the new
      // tokens of a context) goes out in items of up to 256 rows, which the prefill kernel splits over its waves
      // by rows, so that a K/V tile is fetched once per 256 rows instead of once per 64.
      const bool row_split = limited && prefix_mfma && int64_t(count) * group > 64;
      const int32_t per_item = row_split ? std::max(1, 256 / group) : max_req;
      for (int32_t m0 = 0; m0 < count; m0 += per_item)      // row groups outside, heads inside (see the roots)
        for (int32_t h = 0; h < g.num_kv_heads; ++h) {
          ps_item it{};
          it.blk_off = lay->prefix_blk_indptr[p];
          it.tok_begin = int32_t(c * size);
          it.req_off = list0 + m0;
          it.n_req = std::min(per_item, count - m0);
          int32_t v_max = 0, v_min = INT32_MAX;
          for (int32_t i = 0; i < it.n_req; ++i) {
            const int32_t v = visible_of(lay->req_list[size_t(it.req_off + i)]);
            v_max = std::max(v_max, v);
            v_min = std::min(v_min, v);
          }
          it.tok_end = int32_t(std::min<int64_t>(std::min<int64_t>(lay->prefix_len[p], (c + 1) * size), v_max));
          it.kv_head = h;
          it.split_local = c;   // the root's splits are added below, once every request's count is known
          it.kind = (v_min < it.tok_end ? kPsItemMasked : 0) | (row_split ? kPsItemRowSplit : 0) |
                    (count > per_item ? kPsItemReread : 0);
          if (it.kind & kPsItemMasked) lay->any_masked = true;
          if (!row_split) lay->max_rows_prefix = std::max(lay->max_rows_prefix, it.n_req * group);
          prefix_items.push_back(it);
        }
    }
  }
  for (int32_t r = 0; r < R; ++r) {
    int32_t n = 0;
    const int64_t size = chunking(lay->suffix_len[r], suffix_chunk, &n);
    nsplit_suffix[r] = n;
    lay->suffix_chunk_size[size_t(r)] = int32_t(size);
    lay->suffix_chunks[size_t(r)] = n;
    for (int32_t c = 0; c < n; ++c)
      for (int32_t h = 0; h < g.num_kv_heads; ++h) {
        ps_item it{};
        it.blk_off = total_prefix_blocks + lay->suffix_blk_indptr[r];
        it.tok_begin = int32_t(c * size);
        it.tok_end = int32_t(std::min<int64_t>(lay->suffix_len[r], (c + 1) * size));
        it.req_off = R + r;  // identity part of the request list
        it.n_req = 1;
        it.kv_head = h;
        it.split_local = nsplit_root[size_t(r)] + nsplit_prefix[size_t(r)] + c;
        it.kind = kPsItemSuffix;
        suffix_items.push_back(it);
      }
  }
  // a request's partial states: root splits, then prefix splits, then suffix splits (every request of a prefix item
  // is on the same prompt, hence below the same root)
  for (ps_item& it : prefix_items)
    if (!(it.kind & kPsItemRoot)) it.split_local += nsplit_root[size_t(lay->req_list[size_t(it.req_off)])];
  auto by_cost = [](const ps_item& a, const ps_item& b) { return (a.tok_end - a.tok_begin) > (b.tok_end - b.tok_begin); };
  auto rs_first = [&](const ps_item& a, const ps_item& b) {   // row-split items lead, heaviest (tokens x rows) first
    const bool ra = a.kind & kPsItemRowSplit, rb = b.kind & kPsItemRowSplit;
    if (ra != rb) return ra;
    if (ra) return int64_t(a.tok_end - a.tok_begin) * a.n_req > int64_t(b.tok_end - b.tok_begin) * b.n_req;
    return by_cost(a, b);
  };
  std::stable_sort(prefix_items.begin(), prefix_items.end(), rs_first);
  std::stable_sort(suffix_items.begin(), suffix_items.end(), by_cost);
  lay->num_rowsplit_items = 0;
  for (const ps_item& it : prefix_items) lay->num_rowsplit_items += (it.kind & kPsItemRowSplit) ? 1 : 0;
  if (lay->num_rowsplit_items > 8) {
    // XCD-aware launch order of the prefill kernel.  Workgroup i of a launch runs on XCD i mod 8, and each XCD has
    // its own L2.  The row groups that read the same K/V range (same segment, token begin and KV head: a family)
    // are therefore placed eight apart, on one XCD, and next to each other in that XCD's sequence, so that they run
    // at the same time and the range comes out of HBM once instead of once per row group.  Families go, heaviest
    // first, to the XCD with the fewest items so far.
    const int n_rs = lay->num_rowsplit_items;
    typedef std::tuple<int32_t, int32_t, int32_t> range_key;             // (segment, token begin, KV head)
    std::map<range_key, size_t> family_of;
    std::vector<std::vector<ps_item>> family;                             // in order of first (= heaviest) member
    for (int i = 0; i < n_rs; ++i) {
      const ps_item& it = prefix_items[size_t(i)];
      const auto at = family_of.emplace(range_key{it.blk_off, it.tok_begin, it.kv_head}, family.size());
      if (at.second) family.emplace_back();
      family[at.first->second].push_back(it);
    }
    std::vector<std::vector<ps_item>> column(8);
    for (const auto& members : family) {
      size_t target = 0;
      for (size_t c = 1; c < 8; ++c)
        if (column[c].size() < column[target].size()) target = c;
      column[target].insert(column[target].end(), members.begin(), members.end());
    }
    int out = 0;
    for (size_t row = 0; out < n_rs; ++row)
      for (size_t c = 0; c < 8; ++c)
        if (row < column[c].size()) prefix_items[size_t(out++)] = column[c][row];
  }
  // (what the persistent kernel is given must fit its per-wave tile directory; the cuts above see to it)
  if (prefix_mfma)
    for (const ps_item& it : prefix_items)
      if (!(it.kind & kPsItemRowSplit) && it.tok_end - it.tok_begin > mfma_cap) return PS_ERR_INVALID_ARG;
  lay->num_prefix_items = int32_t(prefix_items.size());
  lay->items = std::move(prefix_items);
  lay->items.insert(lay->items.end(), suffix_items.begin(), suffix_items.end());

  lay->slot_base.assign(R + 1, 0);
  int64_t slots = 0;
  for (int32_t r = 0; r < R; ++r) {
    slots += nsplit_root[r] + nsplit_prefix[r] + nsplit_suffix[r];
    if (slots > INT32_MAX) return PS_ERR_INVALID_ARG;
    lay->slot_base[r + 1] = int32_t(slots);
  }
  lay->num_slots = slots;

  // Schedules for the persistent MFMA kernel: longest-processing-time-first packing of a set of items
  // onto the resident workgroups (cost = tokens + a fixed per-item charge), each list longest first.
  typedef ps_layout::packed_set packed;
  auto pack = [&](int begin, int end) {
    packed out;
    const int count = end - begin;
    for (int i = begin; i < end; ++i) out.max_rows = std::max(out.max_rows, lay->items[size_t(i)].n_req * group);
    out.occ = ps_mfma_occupancy(out.max_rows, g.kv_dtype);
    // Cache policy of the launch: K/V that one item reads is best streamed past the caches, K/V that several row
    // groups read (kPsItemReread) should stay in them.  The policy is per launch, so it goes by the share of the
    // set's tokens that lie in re-read items: streaming while that is under a quarter (measured: a root shared by 8
    // row groups next to 3/4 of ordinary traffic gains 1.5 % from streaming, two row groups per prompt at 46 % of
    // the tokens lose 5 %).
    int64_t tokens_all = 0, tokens_reread = 0;
    for (int i = begin; i < end; ++i) {
      const ps_item& it = lay->items[size_t(i)];
      tokens_all += it.tok_end - it.tok_begin;
      if (it.kind & kPsItemReread) tokens_reread += it.tok_end - it.tok_begin;
    }
    out.stream = opt.kv_cache_policy == PS_KV_POLICY_AUTO ? 4 * tokens_reread < tokens_all
                                                           : opt.kv_cache_policy == PS_KV_POLICY_STREAM;
    const int num_wg = std::max(1, std::min(count, num_cus * out.occ));
    std::vector<int> order(size_t(count), 0);
    std::iota(order.begin(), order.end(), begin);
    auto cost = [&](int i) { return int64_t(lay->items[size_t(i)].tok_end - lay->items[size_t(i)].tok_begin) + 64; };
    auto heavier = [&](int a, int b) { return cost(a) > cost(b); };
    // the shared items and the suffix items are each in descending cost already; a range that spans both is the
    // stable merge of two sorted runs
    const int split = std::min(std::max(lay->num_prefix_items, begin), end) - begin;
    if (!std::is_sorted(order.begin(), order.begin() + split, heavier)) std::stable_sort(order.begin(), order.begin() + split, heavier);
    if (!std::is_sorted(order.begin() + split, order.end(), heavier)) std::stable_sort(order.begin() + split, order.end(), heavier);
    std::inplace_merge(order.begin(), order.begin() + split, order.end(), heavier);
    // least-loaded workgroup first, lowest index on ties: a min-heap of (assigned cost, workgroup)
    typedef std::pair<int64_t, int> slot;
    std::priority_queue<slot, std::vector<slot>, std::greater<slot>> load;
    for (int w = 0; w < num_wg; ++w) load.push({0, w});
    std::vector<int> wg_of(size_t(count), 0), fill(size_t(num_wg) + 1, 0);
    for (int n = 0; n < count; ++n) {
      const slot least = load.top();
      load.pop();
      wg_of[size_t(n)] = least.second;
      ++fill[size_t(least.second) + 1];
      load.push({least.first + cost(order[size_t(n)]), least.second});
    }
    for (int w = 0; w < num_wg; ++w) fill[size_t(w) + 1] += fill[size_t(w)];
    out.indptr.assign(fill.begin(), fill.end());
    out.items.resize(size_t(count));
    for (int n = 0; n < count; ++n)      // a workgroup's items keep the order in which they were assigned
      out.items[size_t(fill[size_t(wg_of[size_t(n)])]++)] = lay->items[size_t(order[size_t(n)])];
    if (count == 0) out.indptr.assign(1, 0);
    return out;
  };
  const int n_items = int(lay->items.size());
  const bool pre_mfma = lay->prefix_variant == PS_VARIANT_MFMA, suf_mfma = lay->suffix_variant == PS_VARIANT_MFMA;
  const int first_packed = lay->num_rowsplit_items;   // row-split items run in the prefill kernel, one workgroup each
  lay->pk_prefix = pre_mfma ? pack(first_packed, lay->num_prefix_items) : packed{};
  lay->pk_suffix = suf_mfma ? pack(lay->num_prefix_items, n_items) : packed{};
  lay->pk_all = (pre_mfma && suf_mfma) ? pack(first_packed, n_items) : packed{};
  return ps_blob_build(lay);
}

// Lays the tables out for the device: everything the kernels read, as one int32 blob.
int32_t ps_blob_build(ps_layout* lay) {
  typedef ps_layout::packed_set packed;
  const ps_geometry& g = lay->geo;
  const int32_t R = lay->num_requests;
  const int32_t total_prefix_blocks = int32_t(lay->prefix_blk.size());
  const int32_t root_blk0 = int32_t(lay->prefix_blk.size() + lay->suffix_blk.size());
  const packed &pk_prefix = lay->pk_prefix, &pk_suffix = lay->pk_suffix, &pk_all = lay->pk_all;
  const bool limited = !lay->visible.empty();
  auto visible_of = [&](int32_t r) { return limited ? lay->visible[size_t(r)] : lay->prefix_len[size_t(lay->req_prompt[size_t(r)])]; };
  // device blob: [block ids: prefix ++ suffix ++ root][request list: group_req ++ identity ++ root groups ++ per-chunk
  // subsets][items]
  // [slot_base][visible][schedules]
  // [per-block source offsets and valid counts][destinations of the last append]
  auto pad4 = [](int64_t n) { return (n + 3) / 4 * 4; };
  lay->off_blk = 0;
  lay->off_req = pad4(lay->off_blk + int64_t(lay->prefix_blk.size() + lay->suffix_blk.size() + lay->root_blk.size()));
  lay->off_items = pad4(lay->off_req + int64_t(lay->req_list.size()));
  lay->off_slot = pad4(lay->off_items + 8 * int64_t(lay->items.size()));
  lay->off_visible = pad4(lay->off_slot + R + 1);
  int64_t words = pad4(lay->off_visible + R);
  auto place = [&](ps_layout::schedule& s, const packed& pk) {
    s = ps_layout::schedule{};
    if (pk.items.empty()) return;
    s.num_wg = int32_t(pk.indptr.size()) - 1;
    s.max_rows = pk.max_rows;
    s.occ = pk.occ;
    s.stream = pk.stream;
    s.off_items = words;
    words = pad4(words + 8 * int64_t(pk.items.size()));
    s.off_indptr = words;
    words = pad4(words + int64_t(pk.indptr.size()));
  };
  place(lay->sched_prefix, pk_prefix);
  place(lay->sched_suffix, pk_suffix);
  place(lay->sched_all, pk_all);
  // per-block directory for the cache-writing kernels
  const int64_t num_blk_entries = int64_t(lay->prefix_blk.size() + lay->suffix_blk.size() + lay->root_blk.size());
  lay->off_ent_tok0 = words;
  lay->off_ent_valid = pad4(lay->off_ent_tok0 + num_blk_entries);
  lay->off_dest = pad4(lay->off_ent_valid + num_blk_entries);
  lay->off_ent_order = pad4(lay->off_dest + R);
  words = pad4(lay->off_ent_order + num_blk_entries);
  // (the tables grow by a few words per decode step: room to spare keeps the buffer -- and its mapped pages -- in
  // place instead of taking a fresh allocation every step)
  const size_t blob_words = size_t(std::max<int64_t>(words, 4));
  if (lay->blob.capacity() < blob_words) lay->blob.reserve(blob_words + blob_words / 4 + 1024);
  lay->blob.assign(blob_words, 0);
  int32_t* b = lay->blob.data();
  {
    const int32_t B = g.block_size;
    // skip: per segment, leading blocks that are not to be written (adopted from another layout); the ragged source
    // then holds only the tokens after them
    auto fill_entries = [&](const std::vector<int32_t>& indptr, const std::vector<int32_t>& len, int32_t* tok0_out,
                            int32_t* valid_out, const std::vector<int32_t>* skip) {
      int64_t tok = 0;
      for (size_t s = 0; s + 1 < indptr.size(); ++s) {
        const int64_t skipped = skip ? int64_t((*skip)[s + 1] - (*skip)[s]) * B : 0;
        for (int32_t i = indptr[s]; i < indptr[s + 1]; ++i) {
          const int64_t first = int64_t(i - indptr[s]) * B;
          if (tok + first > INT32_MAX) return false;
          const bool kept = first < skipped;
          tok0_out[i] = kept ? 0 : int32_t(tok + first - skipped);
          valid_out[i] = kept ? 0 : int32_t(std::min<int64_t>(B, len[s] - first));
        }
        tok += len[s] - skipped;
      }
      return true;
    };
    // The shared segments (prefixes, roots) never change after the layout is made, so their part of the directory is
    // worked out once and copied from then on; the private part follows the appends.
    const size_t n_fixed = lay->prefix_blk.size() + lay->root_blk.size();
    if (lay->ent_fixed_tok0.size() != n_fixed) {
      lay->ent_fixed_tok0.assign(n_fixed, 0);
      lay->ent_fixed_valid.assign(n_fixed, 0);
      int32_t* root_tok0 = lay->ent_fixed_tok0.data() + lay->prefix_blk.size();
      int32_t* root_valid = lay->ent_fixed_valid.data() + lay->prefix_blk.size();
      if (!fill_entries(lay->prefix_blk_indptr, lay->prefix_len, lay->ent_fixed_tok0.data(), lay->ent_fixed_valid.data(),
                        lay->adopt_indptr.empty() ? nullptr : &lay->adopt_indptr) ||
          (lay->num_roots && !fill_entries(lay->root_blk_indptr, lay->root_len, root_tok0, root_valid, nullptr))) {
        lay->ent_fixed_tok0.clear();
        lay->ent_fixed_valid.clear();
        return PS_ERR_INVALID_ARG;
      }
      // An ingest walks the shared blocks in the order of their addresses in the pool, not of the tokens: the pool's
      // blocks are scattered, and scattered reads (the source, now) cost less than scattered writes (measured on the
      // staging copies: 5.8 against 5.2 TB/s).
      auto by_block = [&](const std::vector<int32_t>& blk, int32_t* order) {
        std::iota(order, order + blk.size(), 0);
        std::sort(order, order + blk.size(), [&](int32_t a, int32_t b2) { return blk[size_t(a)] < blk[size_t(b2)]; });
      };
      lay->ent_fixed_order.resize(n_fixed);
      by_block(lay->prefix_blk, lay->ent_fixed_order.data());
      by_block(lay->root_blk, lay->ent_fixed_order.data() + lay->prefix_blk.size());
    }
    std::copy(lay->ent_fixed_tok0.begin(), lay->ent_fixed_tok0.begin() + total_prefix_blocks, b + lay->off_ent_tok0);
    std::copy(lay->ent_fixed_valid.begin(), lay->ent_fixed_valid.begin() + total_prefix_blocks, b + lay->off_ent_valid);
    std::copy(lay->ent_fixed_tok0.begin() + total_prefix_blocks, lay->ent_fixed_tok0.end(), b + lay->off_ent_tok0 + root_blk0);
    std::copy(lay->ent_fixed_valid.begin() + total_prefix_blocks, lay->ent_fixed_valid.end(), b + lay->off_ent_valid + root_blk0);
    if (!fill_entries(lay->suffix_blk_indptr, lay->suffix_len, b + lay->off_ent_tok0 + total_prefix_blocks,
                      b + lay->off_ent_valid + total_prefix_blocks, nullptr))
      return PS_ERR_INVALID_ARG;
    lay->append_dest.resize(size_t(R), -1);
    std::copy(lay->append_dest.begin(), lay->append_dest.end(), b + lay->off_dest);
    // (entries of the concatenated block array: the shared kinds by block, the private segments as stored)
    std::copy(lay->ent_fixed_order.begin(), lay->ent_fixed_order.begin() + total_prefix_blocks, b + lay->off_ent_order);
    std::iota(b + lay->off_ent_order + total_prefix_blocks, b + lay->off_ent_order + root_blk0, total_prefix_blocks);
    for (size_t i = 0; i < lay->root_blk.size(); ++i)
      b[lay->off_ent_order + root_blk0 + int64_t(i)] = root_blk0 + lay->ent_fixed_order[size_t(total_prefix_blocks) + i];
  }
  auto fill = [&](const ps_layout::schedule& s, const packed& pk) {
    if (pk.items.empty()) return;
    std::memcpy(b + s.off_items, pk.items.data(), pk.items.size() * sizeof(ps_item));
    std::copy(pk.indptr.begin(), pk.indptr.end(), b + s.off_indptr);
  };
  fill(lay->sched_prefix, pk_prefix);
  fill(lay->sched_suffix, pk_suffix);
  fill(lay->sched_all, pk_all);
  std::copy(lay->prefix_blk.begin(), lay->prefix_blk.end(), b + lay->off_blk);
  std::copy(lay->suffix_blk.begin(), lay->suffix_blk.end(), b + lay->off_blk + lay->prefix_blk.size());
  std::copy(lay->root_blk.begin(), lay->root_blk.end(), b + lay->off_blk + root_blk0);
  std::copy(lay->req_list.begin(), lay->req_list.end(), b + lay->off_req);
  for (int32_t r = 0; r < R; ++r) b[lay->off_visible + r] = visible_of(r);
  if (!lay->items.empty()) std::memcpy(b + lay->off_items, lay->items.data(), lay->items.size() * sizeof(ps_item));
  std::copy(lay->slot_base.begin(), lay->slot_base.end(), b + lay->off_slot);
  return PS_OK;
}

namespace {

// Drops every reference the layout holds; blocks that reach zero join the free-list tail in ascending id.
// PS_ERR_REFCOUNT leaves the pool unchanged.
int32_t drop_references(ps_pool* pool, const ps_layout* lay) {
  std::vector<int64_t> drop(size_t(pool->num_blocks), 0);
  for (int32_t t = 0; t < lay->num_roots; ++t) {
    const int32_t k = lay->root_group_indptr[size_t(t) + 1] - lay->root_group_indptr[size_t(t)];
    for (int32_t i = lay->root_blk_indptr[size_t(t)]; i < lay->root_blk_indptr[size_t(t) + 1]; ++i) {
      const int32_t b = lay->root_blk[size_t(i)];
      if (b < 0 || b >= pool->num_blocks) return PS_ERR_REFCOUNT;
      drop[size_t(b)] += k;
    }
  }
  for (int32_t p = 0; p < lay->num_prompts; ++p) {
    const int32_t k = lay->group_indptr[size_t(p) + 1] - lay->group_indptr[size_t(p)];
    for (int32_t i = lay->prefix_blk_indptr[size_t(p)]; i < lay->prefix_blk_indptr[size_t(p) + 1]; ++i) {
      const int32_t b = lay->prefix_blk[size_t(i)];
      if (b < 0 || b >= pool->num_blocks) return PS_ERR_REFCOUNT;
      drop[size_t(b)] += k;
    }
  }
  for (int32_t b : lay->suffix_blk) {
    if (b < 0 || b >= pool->num_blocks) return PS_ERR_REFCOUNT;
    drop[size_t(b)] += 1;
  }
  for (int32_t b = 0; b < pool->num_blocks; ++b)
    if (pool->refcount[size_t(b)] < drop[size_t(b)]) return PS_ERR_REFCOUNT;
  for (int32_t b = 0; b < pool->num_blocks; ++b) {
    if (!drop[size_t(b)]) continue;
    pool->refcount[size_t(b)] -= int32_t(drop[size_t(b)]);
    if (pool->refcount[size_t(b)] == 0) pool->free_list.push_back(b);
  }
  return PS_OK;
}

// Takes the blocks of every segment by the canonical policy (roots, prompts, requests; head of the free list).  The
// caller has checked that the free list is long enough.
void take_blocks(ps_pool* pool, ps_layout* lay) {
  const int32_t B = lay->geo.block_size;
  auto take = [&](int32_t refs) {
    const int32_t blk = pool->free_list.front();
    pool->free_list.pop_front();
    pool->refcount[size_t(blk)] += refs;
    return blk;
  };
  lay->root_blk.clear();
  lay->prefix_blk.clear();
  lay->suffix_blk.clear();
  lay->root_blk_indptr.assign(size_t(lay->num_roots) + 1, 0);
  for (int32_t t = 0; t < lay->num_roots; ++t) {
    const int32_t k = lay->root_group_indptr[size_t(t) + 1] - lay->root_group_indptr[size_t(t)];
    const int64_t n = ceil_div(lay->root_len[size_t(t)], B);
    for (int64_t i = 0; i < n; ++i) lay->root_blk.push_back(take(k));
    lay->root_blk_indptr[size_t(t) + 1] = int32_t(lay->root_blk.size());
  }
  lay->prefix_blk_indptr.assign(size_t(lay->num_prompts) + 1, 0);
  const bool adopting = !lay->adopt_indptr.empty();
  for (int32_t p = 0; p < lay->num_prompts; ++p) {
    const int32_t k = lay->group_indptr[size_t(p) + 1] - lay->group_indptr[size_t(p)];
    const int64_t n = ceil_div(lay->prefix_len[size_t(p)], B);
    const int32_t a0 = adopting ? lay->adopt_indptr[size_t(p)] : 0, a1 = adopting ? lay->adopt_indptr[size_t(p) + 1] : 0;
    for (int64_t i = 0; i < n; ++i) {
      if (i < a1 - a0) {   // a cached block another layout holds: one more reference per request, like a fresh one
        const int32_t blk = lay->adopt_blk[size_t(a0 + i)];
        pool->refcount[size_t(blk)] += k;
        lay->prefix_blk.push_back(blk);
      } else {
        lay->prefix_blk.push_back(take(k));
      }
    }
    lay->prefix_blk_indptr[size_t(p) + 1] = int32_t(lay->prefix_blk.size());
  }
  lay->suffix_blk_indptr.assign(size_t(lay->num_requests) + 1, 0);
  for (int32_t r = 0; r < lay->num_requests; ++r) {
    const int64_t n = ceil_div(lay->suffix_len[size_t(r)], B);
    for (int64_t i = 0; i < n; ++i) lay->suffix_blk.push_back(take(1));
    lay->suffix_blk_indptr[size_t(r) + 1] = int32_t(lay->suffix_blk.size());
  }
}

int64_t blocks_of(const ps_layout* lay) {   // blocks the layout references, adopted ones included
  const int32_t B = lay->geo.block_size;
  int64_t n = 0;
  for (int32_t l : lay->root_len) n += ceil_div(l, B);
  for (int32_t l : lay->prefix_len) n += ceil_div(l, B);
  for (int32_t l : lay->suffix_len) n += ceil_div(l, B);
  return n;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
extern "C" {

int32_t ps_pool_create(int32_t num_blocks, const int32_t* free_order, ps_pool** out) {
  if (!out || num_blocks < 0) return PS_ERR_INVALID_ARG;
  ps_pool* p = new (std::nothrow) ps_pool();
  if (!p) return PS_ERR_OOM;
  p->num_blocks = num_blocks;
  p->refcount.assign(size_t(num_blocks), 0);
  if (free_order) {
    std::vector<char> seen(size_t(num_blocks), 0);
    for (int32_t i = 0; i < num_blocks; ++i) {
      const int32_t b = free_order[i];
      if (b < 0 || b >= num_blocks || seen[size_t(b)]) { delete p; return PS_ERR_INVALID_ARG; }
      seen[size_t(b)] = 1;
      p->free_list.push_back(b);
    }
  } else {
    for (int32_t i = 0; i < num_blocks; ++i) p->free_list.push_back(i);
  }
  *out = p;
  return PS_OK;
}

int32_t ps_pool_destroy(ps_pool* pool) {
  delete pool;
  return PS_OK;
}

int32_t ps_pool_num_free(const ps_pool* pool, int32_t* out) {
  if (!pool || !out) return PS_ERR_INVALID_ARG;
  *out = int32_t(pool->free_list.size());
  return PS_OK;
}

int32_t ps_pool_free_list(const ps_pool* pool, int32_t* out, int32_t capacity, int32_t* count) {
  if (!pool || !count || capacity < 0 || (capacity > 0 && !out)) return PS_ERR_INVALID_ARG;
  *count = int32_t(pool->free_list.size());
  if (capacity < *count) return PS_ERR_INVALID_ARG;
  std::copy(pool->free_list.begin(), pool->free_list.end(), out);
  return PS_OK;
}

int32_t ps_pool_refcounts(const ps_pool* pool, const int32_t** refcount) {
  if (!pool || !refcount) return PS_ERR_INVALID_ARG;
  *refcount = pool->refcount.data();
  return PS_OK;
}

}  // extern "C"

namespace {

int32_t build_layout(ps_pool* pool, const ps_geometry* geometry, int32_t num_roots, const int32_t* root_len,
                     int32_t num_prompts, const int32_t* prompt_root, const int32_t* prefix_len,
                     const int32_t* adopt_indptr, const int32_t* adopt_blk, int32_t num_requests,
                     const int32_t* req_prompt, const int32_t* req_model, const int32_t* suffix_len, ps_layout** out) {
  if (!pool || !geometry || !out || num_roots < 0 || num_prompts < 0 || num_requests < 0) return PS_ERR_INVALID_ARG;
  if ((num_prompts && !prefix_len) || (num_requests && (!req_prompt || !req_model || !suffix_len)))
    return PS_ERR_INVALID_ARG;
  if (num_roots && (!root_len || !prompt_root)) return PS_ERR_INVALID_ARG;
  if (int32_t st = check_geometry(*geometry)) return st;
  const int32_t B = geometry->block_size;

  std::vector<int32_t> members_count(size_t(num_prompts), 0);
  std::set<std::pair<int32_t, int32_t>> seen;
  for (int32_t r = 0; r < num_requests; ++r) {
    if (req_prompt[r] < 0 || req_prompt[r] >= num_prompts || req_model[r] < 0 || suffix_len[r] < 0)
      return PS_ERR_INVALID_ARG;
    if (!seen.insert({req_prompt[r], req_model[r]}).second) return PS_ERR_INVALID_ARG;
    ++members_count[size_t(req_prompt[r])];
  }
  // requests below every root: all requests of the prompts that begin with it
  std::vector<int32_t> below_count(size_t(num_roots), 0), root_prompts(size_t(num_roots), 0);
  for (int32_t p = 0; p < num_prompts && num_roots; ++p) {
    const int32_t t = prompt_root[p];
    if (t < -1 || t >= num_roots) return PS_ERR_INVALID_ARG;
    if (t >= 0) {
      below_count[size_t(t)] += members_count[size_t(p)];
      ++root_prompts[size_t(t)];
    }
  }
  int64_t needed = 0;
  for (int32_t t = 0; t < num_roots; ++t) {
    if (root_len[t] < 0 || root_prompts[size_t(t)] == 0) return PS_ERR_INVALID_ARG;
    needed += ceil_div(root_len[t], B);
  }
  for (int32_t p = 0; p < num_prompts; ++p) {
    if (prefix_len[p] < 0 || members_count[size_t(p)] == 0) return PS_ERR_INVALID_ARG;
    needed += ceil_div(prefix_len[p], B);
  }
  for (int32_t r = 0; r < num_requests; ++r) needed += ceil_div(suffix_len[r], B);
  if (adopt_indptr) {
    // adopted blocks: full blocks of the prompt's prefix, alive (referenced by some layout) and named once
    if (adopt_indptr[0] != 0 || (adopt_indptr[num_prompts] > 0 && !adopt_blk)) return PS_ERR_INVALID_ARG;
    std::set<int32_t> named;
    for (int32_t p = 0; p < num_prompts; ++p) {
      const int32_t n = adopt_indptr[p + 1] - adopt_indptr[p];
      if (n < 0 || int64_t(n) * B > prefix_len[p]) return PS_ERR_INVALID_ARG;
      for (int32_t i = adopt_indptr[p]; i < adopt_indptr[p + 1]; ++i) {
        const int32_t blk = adopt_blk[i];
        if (blk < 0 || blk >= pool->num_blocks || pool->refcount[size_t(blk)] <= 0 || !named.insert(blk).second)
          return PS_ERR_INVALID_ARG;
      }
      needed -= n;
    }
  }
  if (needed > int64_t(pool->free_list.size())) return PS_ERR_OOM;

  ps_layout* lay = new (std::nothrow) ps_layout();
  if (!lay) return PS_ERR_OOM;
  lay->geo = *geometry;
  lay->num_prompts = num_prompts;
  lay->num_requests = num_requests;
  lay->prefix_len.assign(prefix_len, prefix_len + num_prompts);
  lay->suffix_len.assign(suffix_len, suffix_len + num_requests);
  lay->req_prompt.assign(req_prompt, req_prompt + num_requests);
  lay->req_model.assign(req_model, req_model + num_requests);
  if (adopt_indptr && adopt_indptr[num_prompts] > 0) {
    lay->adopt_indptr.assign(adopt_indptr, adopt_indptr + num_prompts + 1);
    lay->adopt_blk.assign(adopt_blk, adopt_blk + adopt_indptr[num_prompts]);
  }
  lay->num_roots = num_roots;
  if (num_roots) {
    lay->root_len.assign(root_len, root_len + num_roots);
    lay->prompt_root.assign(prompt_root, prompt_root + num_prompts);
  }

  // sharing groups: a prompt's requests in ascending request index; a root's likewise
  lay->group_indptr.assign(size_t(num_prompts) + 1, 0);
  for (int32_t p = 0; p < num_prompts; ++p) lay->group_indptr[size_t(p) + 1] = lay->group_indptr[size_t(p)] + members_count[size_t(p)];
  lay->group_req.assign(size_t(num_requests), 0);
  {
    std::vector<int32_t> cursor(lay->group_indptr.begin(), lay->group_indptr.end() - 1);
    for (int32_t r = 0; r < num_requests; ++r) lay->group_req[size_t(cursor[size_t(req_prompt[r])]++)] = r;
  }
  lay->root_group_indptr.assign(size_t(num_roots) + 1, 0);
  for (int32_t t = 0; t < num_roots; ++t)
    lay->root_group_indptr[size_t(t) + 1] = lay->root_group_indptr[size_t(t)] + below_count[size_t(t)];
  lay->root_group_req.assign(size_t(lay->root_group_indptr.back()), 0);
  if (num_roots) {
    std::vector<int32_t> cursor(lay->root_group_indptr.begin(), lay->root_group_indptr.end() - 1);
    for (int32_t r = 0; r < num_requests; ++r) {
      const int32_t t = prompt_root[req_prompt[r]];
      if (t >= 0) lay->root_group_req[size_t(cursor[size_t(t)]++)] = r;
    }
  }

  take_blocks(pool, lay);

  if (int32_t st = ps_plan_build(lay, nullptr)) {
    // cannot fail with default options, but never leave references behind
    ps_layout_release(pool, lay);
    return st;
  }
  *out = lay;
  return PS_OK;
}

}  // namespace

extern "C" {

int32_t ps_kv_layout_tree(ps_pool* pool, const ps_geometry* geometry, int32_t num_roots, const int32_t* root_len,
                          int32_t num_prompts, const int32_t* prompt_root, const int32_t* prefix_len,
                          int32_t num_requests, const int32_t* req_prompt, const int32_t* req_model,
                          const int32_t* suffix_len, ps_layout** out) {
  return build_layout(pool, geometry, num_roots, root_len, num_prompts, prompt_root, prefix_len, nullptr, nullptr,
                      num_requests, req_prompt, req_model, suffix_len, out);
}

int32_t ps_kv_layout(ps_pool* pool, const ps_geometry* geometry, int32_t num_prompts, const int32_t* prefix_len,
                     int32_t num_requests, const int32_t* req_prompt, const int32_t* req_model,
                     const int32_t* suffix_len, ps_layout** out) {
  return build_layout(pool, geometry, 0, nullptr, num_prompts, nullptr, prefix_len, nullptr, nullptr, num_requests,
                      req_prompt, req_model, suffix_len, out);
}

int32_t ps_kv_layout_adopt(ps_pool* pool, const ps_geometry* geometry, int32_t num_prompts, const int32_t* prefix_len,
                           const int32_t* adopt_indptr, const int32_t* adopt_blk, int32_t num_requests,
                           const int32_t* req_prompt, const int32_t* req_model, const int32_t* suffix_len,
                           ps_layout** out) {
  if (num_prompts > 0 && !adopt_indptr) return PS_ERR_INVALID_ARG;
  return build_layout(pool, geometry, 0, nullptr, num_prompts, nullptr, prefix_len, adopt_indptr, adopt_blk,
                      num_requests, req_prompt, req_model, suffix_len, out);
}

int32_t ps_layout_root_tables(const ps_layout* lay, int32_t* num_roots, const int32_t** root_blk_indptr,
                              const int32_t** root_blk, const int32_t** root_group_indptr,
                              const int32_t** root_group_req) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (num_roots) *num_roots = lay->num_roots;
  if (root_blk_indptr) *root_blk_indptr = lay->root_blk_indptr.data();
  if (root_blk) *root_blk = lay->root_blk.data();
  if (root_group_indptr) *root_group_indptr = lay->root_group_indptr.data();
  if (root_group_req) *root_group_req = lay->root_group_req.data();
  return PS_OK;
}

int32_t ps_layout_release(ps_pool* pool, ps_layout* lay) {
  if (!pool || !lay) return PS_ERR_INVALID_ARG;
  if (!lay->parked)
    if (int32_t st = drop_references(pool, lay)) return st;
  delete lay;
  return PS_OK;
}

int32_t ps_blocks_needed(int32_t block_size, int32_t num_roots, const int32_t* root_len, int32_t num_prompts,
                         const int32_t* prefix_len, int32_t num_requests, const int32_t* suffix_len, int64_t* out) {
  if (!out || block_size <= 0 || num_roots < 0 || num_prompts < 0 || num_requests < 0) return PS_ERR_INVALID_ARG;
  if ((num_roots && !root_len) || (num_prompts && !prefix_len) || (num_requests && !suffix_len)) return PS_ERR_INVALID_ARG;
  int64_t n = 0;
  auto add = [&](const int32_t* len, int32_t count) {
    for (int32_t i = 0; i < count; ++i) {
      if (len[i] < 0) return false;
      n += ceil_div(len[i], block_size);
    }
    return true;
  };
  if (!add(root_len, num_roots) || !add(prefix_len, num_prompts) || !add(suffix_len, num_requests)) return PS_ERR_INVALID_ARG;
  *out = n;
  return PS_OK;
}

int32_t ps_layout_park(ps_pool* pool, ps_layout* lay) {
  if (!pool || !lay || lay->parked) return PS_ERR_INVALID_ARG;
  if (int32_t st = drop_references(pool, lay)) return st;
  lay->parked = true;
  lay->adopt_indptr.clear();   // a resumed layout holds fresh blocks only: its image carries the adopted contents
  lay->ent_fixed_tok0.clear();   // ... so the directory of the shared segments is worked out again
  lay->ent_fixed_valid.clear();
  lay->ent_fixed_order.clear();
  lay->adopt_blk.clear();
  std::fill(lay->root_blk.begin(), lay->root_blk.end(), -1);
  std::fill(lay->prefix_blk.begin(), lay->prefix_blk.end(), -1);
  std::fill(lay->suffix_blk.begin(), lay->suffix_blk.end(), -1);
  std::fill(lay->append_dest.begin(), lay->append_dest.end(), -1);
  return PS_OK;
}

int32_t ps_layout_resume(ps_pool* pool, ps_layout* lay) {
  if (!pool || !lay || !lay->parked) return PS_ERR_INVALID_ARG;
  if (blocks_of(lay) > int64_t(pool->free_list.size())) return PS_ERR_OOM;
  take_blocks(pool, lay);
  lay->parked = false;
  return ps_plan_build(lay, &lay->opt);   // options that were accepted before cannot fail
}

int32_t ps_layout_state(const ps_layout* lay, int64_t* num_blocks, int32_t* parked) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (num_blocks) *num_blocks = blocks_of(lay);
  if (parked) *parked = lay->parked ? 1 : 0;
  return PS_OK;
}

int32_t ps_stage_layout(const ps_layout* lay, int64_t* block_bytes, int64_t* scales_offset_bytes, int64_t* total_bytes) {
  if (!lay) return PS_ERR_INVALID_ARG;
  const ps_geometry& g = lay->geo;
  const int64_t esz = g.kv_dtype == PS_F32 ? 4 : (g.kv_dtype == PS_BF16 ? 2 : 1);
  const int64_t per_block = int64_t(g.num_kv_heads) * 2 * g.block_size * g.head_dim * esz;
  const int64_t n = blocks_of(lay);
  const int64_t scales_off = round_up(n * per_block, 256);
  if (block_bytes) *block_bytes = per_block;
  if (scales_offset_bytes) *scales_offset_bytes = scales_off;
  if (total_bytes) *total_bytes = g.kv_dtype == PS_FP8_E4M3 ? scales_off + n * g.num_kv_heads * 2 * 4 : std::max<int64_t>(n * per_block, 16);
  return PS_OK;
}

int32_t ps_layout_tables(const ps_layout* lay, const int32_t** prefix_blk_indptr, const int32_t** prefix_blk,
                         const int32_t** group_indptr, const int32_t** group_req,
                         const int32_t** suffix_blk_indptr, const int32_t** suffix_blk) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (prefix_blk_indptr) *prefix_blk_indptr = lay->prefix_blk_indptr.data();
  if (prefix_blk) *prefix_blk = lay->prefix_blk.data();
  if (group_indptr) *group_indptr = lay->group_indptr.data();
  if (group_req) *group_req = lay->group_req.data();
  if (suffix_blk_indptr) *suffix_blk_indptr = lay->suffix_blk_indptr.data();
  if (suffix_blk) *suffix_blk = lay->suffix_blk.data();
  return PS_OK;
}

int32_t ps_layout_lengths(const ps_layout* lay, const int32_t** prefix_len, const int32_t** suffix_len) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (prefix_len) *prefix_len = lay->prefix_len.data();
  if (suffix_len) *suffix_len = lay->suffix_len.data();
  return PS_OK;
}

int32_t ps_layout_append(ps_pool* pool, ps_layout* lay, const int32_t* active, const int32_t** dest) {
  if (!pool || !lay || lay->parked) return PS_ERR_INVALID_ARG;
  const int32_t R = lay->num_requests, B = lay->geo.block_size;
  if (int64_t(pool->num_blocks) * B > INT32_MAX) return PS_ERR_INVALID_ARG;  // slot indices are int32
  auto is_active = [&](int32_t r) { return !active || active[r] != 0; };
  int64_t needed = 0;
  for (int32_t r = 0; r < R; ++r) {
    if (!is_active(r)) continue;
    if (lay->suffix_len[size_t(r)] == INT32_MAX) return PS_ERR_INVALID_ARG;
    if (lay->suffix_len[size_t(r)] % B == 0) ++needed;
  }
  if (needed > int64_t(pool->free_list.size())) return PS_ERR_OOM;
  // requests in ascending index; one whose private length is a multiple of the block size (none yet, or the
  // last block is full) takes the block at the head of the free list
  std::vector<int32_t> blk, indptr(size_t(R) + 1, 0);
  blk.reserve(lay->suffix_blk.size() + size_t(needed));
  lay->append_dest.assign(size_t(R), -1);
  for (int32_t r = 0; r < R; ++r) {
    const size_t first = blk.size();
    blk.insert(blk.end(), lay->suffix_blk.begin() + lay->suffix_blk_indptr[size_t(r)],
               lay->suffix_blk.begin() + lay->suffix_blk_indptr[size_t(r) + 1]);
    if (is_active(r)) {
      const int32_t pos = lay->suffix_len[size_t(r)];
      if (pos % B == 0) {
        const int32_t b = pool->free_list.front();
        pool->free_list.pop_front();
        pool->refcount[size_t(b)] += 1;
        blk.push_back(b);
      }
      lay->append_dest[size_t(r)] = blk[first + size_t(pos / B)] * B + pos % B;
      lay->suffix_len[size_t(r)] = pos + 1;
    }
    indptr[size_t(r) + 1] = int32_t(blk.size());
  }
  lay->suffix_blk.swap(blk);
  lay->suffix_blk_indptr.swap(indptr);
  // A step that leaves the chunk structure of every private segment as it is (same number of chunks, same chunk
  // size where there are several) only moves token ends and block offsets: the plan -- items, their order, the
  // packing onto workgroups -- is kept and patched, and only the tables are laid out again.  Anything else (a first
  // token, a segment outgrowing its chunks) plans afresh.
  bool same_structure = lay->suffix_chunks.size() == size_t(R) && lay->suffix_chunk > 0;
  const int64_t granule = std::lcm<int64_t>(B, 32);
  for (int32_t r = 0; r < R && same_structure; ++r) {
    if (!is_active(r)) continue;
    const int64_t len = lay->suffix_len[size_t(r)];
    const int64_t count = ceil_div(len, lay->suffix_chunk);
    const int64_t size = round_up(ceil_div(len, count), granule);
    const int64_t n = ceil_div(len, size);
    if (len <= 1 || n != lay->suffix_chunks[size_t(r)] || (n > 1 && size != lay->suffix_chunk_size[size_t(r)]))
      same_structure = false;
    else
      lay->suffix_chunk_size[size_t(r)] = int32_t(size);
  }
  if (same_structure) {
    const int32_t prefix_blocks = int32_t(lay->prefix_blk.size());
    const int32_t root_shift = int32_t(lay->prefix_blk.size() + lay->suffix_blk.size()) - lay->planned_root_blk0;
    auto patch = [&](std::vector<ps_item>& items) {
      for (ps_item& it : items) {
        if (it.kind & kPsItemSuffix) {
          const int32_t r = it.req_off - R;   // private-suffix items index the identity part of the request list
          it.blk_off = prefix_blocks + lay->suffix_blk_indptr[size_t(r)];
          it.tok_end = std::min(lay->suffix_len[size_t(r)], it.tok_begin + lay->suffix_chunk_size[size_t(r)]);
        } else if (it.kind & kPsItemRoot) {
          it.blk_off += root_shift;
        }
      }
    };
    patch(lay->items);
    patch(lay->pk_prefix.items);
    patch(lay->pk_suffix.items);
    patch(lay->pk_all.items);
    lay->planned_root_blk0 += root_shift;
    if (int32_t st = ps_blob_build(lay)) return st;
  } else {
    if (int32_t st = ps_plan_build(lay, &lay->opt)) return st;
  }
  if (dest) *dest = lay->append_dest.data();
  return PS_OK;
}

int32_t ps_layout_set_visible(ps_layout* lay, const int32_t* prefix_visible) {
  if (!lay) return PS_ERR_INVALID_ARG;
  std::vector<int32_t> v;
  if (prefix_visible) {
    v.assign(prefix_visible, prefix_visible + lay->num_requests);
    for (int32_t r = 0; r < lay->num_requests; ++r)
      if (v[size_t(r)] < 0 || v[size_t(r)] > lay->prefix_len[size_t(lay->req_prompt[size_t(r)])]) return PS_ERR_INVALID_ARG;
  }
  lay->visible.swap(v);
  if (int32_t st = ps_plan_build(lay, &lay->opt)) {
    lay->visible.swap(v);              // cannot fail with options that were accepted before; keep the old state
    ps_plan_build(lay, &lay->opt);
    return st;
  }
  return PS_OK;
}

int32_t ps_layout_request_list(const ps_layout* lay, int32_t* count, const int32_t** list) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (count) *count = int32_t(lay->req_list.size());
  if (list) *list = lay->req_list.data();
  return PS_OK;
}

int32_t ps_layout_replan(ps_layout* lay, const ps_plan_options* options) {
  if (!lay) return PS_ERR_INVALID_ARG;
  return ps_plan_build(lay, options);
}

int32_t ps_layout_plan(const ps_layout* lay, int32_t* num_items, const int32_t** items, const int32_t** slot_base,
                       int32_t* prefix_variant, int32_t* suffix_variant) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (num_items) *num_items = int32_t(lay->items.size());
  if (items) *items = reinterpret_cast<const int32_t*>(lay->items.data());
  if (slot_base) *slot_base = lay->slot_base.data();
  if (prefix_variant) *prefix_variant = lay->prefix_variant;
  if (suffix_variant) *suffix_variant = lay->suffix_variant;
  return PS_OK;
}

int32_t ps_layout_schedule(const ps_layout* lay, int32_t which, int32_t* num_workgroups, const int32_t** items,
                           const int32_t** indptr) {
  if (!lay || which < 0 || which > 2) return PS_ERR_INVALID_ARG;
  const ps_layout::schedule& s = which == 0 ? lay->sched_prefix : (which == 1 ? lay->sched_suffix : lay->sched_all);
  if (num_workgroups) *num_workgroups = s.num_wg;
  if (items) *items = s.num_wg ? lay->blob.data() + s.off_items : nullptr;
  if (indptr) *indptr = s.num_wg ? lay->blob.data() + s.off_indptr : nullptr;
  return PS_OK;
}

int64_t ps_layout_device_bytes(const ps_layout* lay) { return lay ? int64_t(lay->blob.size()) * 4 : -1; }

int64_t ps_workspace_bytes(const ps_layout* lay) {
  if (!lay) return -1;
  const int64_t rows = lay->num_slots * lay->geo.num_q_heads;
  return std::max<int64_t>(16, rows * (lay->geo.head_dim + 1) * 4);
}

int32_t ps_workspace_layout(const ps_layout* lay, int64_t* num_slots, int64_t* lse_offset_bytes) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (num_slots) *num_slots = lay->num_slots;
  if (lse_offset_bytes) *lse_offset_bytes = lay->num_slots * lay->geo.num_q_heads * int64_t(lay->geo.head_dim) * 4;
  return PS_OK;
}

const char* ps_strerror(int32_t status) {
  switch (status) {
    case PS_OK: return "ok";
    case PS_ERR_INVALID_ARG: return "invalid argument";
    case PS_ERR_SHAPE: return "geometry cannot be addressed (head counts, strides or alignment)";
    case PS_ERR_OOM: return "not enough free KV blocks (or host memory); nothing was allocated";
    case PS_ERR_REFCOUNT: return "refcount underflow or double release";
    case PS_ERR_UNSUPPORTED: return "no kernel for this dtype / head_dim / block_size combination";
    case PS_ERR_DEVICE: return "HIP call failed (see ps_last_hip_error)";
    case PS_ERR_TOO_LARGE: return "the batch's partial states exceed the library's static workspace (PS_STATIC_WORKSPACE_BYTES)";
    default: return "unknown status";
  }
}

}  // extern "C"
