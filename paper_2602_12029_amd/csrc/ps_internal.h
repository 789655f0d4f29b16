// Internal host-side structures shared by the layout/planner and the launch code.
#pragma once
#include <cstdint>
#include <deque>
#include <vector>

#include "prefillshare.h"

struct ps_pool {
  int32_t num_blocks = 0;
  std::deque<int32_t> free_list;
  std::vector<int32_t> refcount;
};

// One unit of attention work: a token range of one KV segment for one KV head, applied to the
// query rows of n_req requests (all G q heads of the head's group each).
struct ps_item {
  int32_t blk_off;      // index of the segment's first block in the concatenated block array
  int32_t tok_begin;
  int32_t tok_end;
  int32_t req_off;      // index of the first request in the request list
  int32_t n_req;
  int32_t kv_head;
  int32_t split_local;  // partial-state slot of request r is slot_base[r] + split_local
  int32_t kind;         // bit 0: 0 prefix, 1 suffix; bit 1: some row of the item sees less than tok_end
};
// bit 2: up to 256 rows, split over the four waves of a workgroup by rows instead of by tokens (partial prefill)
// bit 3: a root segment (a context several prompts begin with), read by every request below the root
// bit 4: other items (further row groups of the same sharing group) read the same K/V range: keep it cacheable
constexpr int32_t kPsItemSuffix = 1, kPsItemMasked = 2, kPsItemRowSplit = 4, kPsItemRoot = 8, kPsItemReread = 16;
static_assert(sizeof(ps_item) == 32, "ps_item is 8 int32");

struct ps_layout {
  ps_geometry geo{};
  int32_t num_prompts = 0, num_requests = 0;
  std::vector<int32_t> prefix_len, suffix_len, req_prompt, req_model;
  std::vector<int32_t> prefix_blk_indptr, prefix_blk, group_indptr, group_req, suffix_blk_indptr, suffix_blk;
  // blocks adopted from another layout (the cached beginning of a prompt's prefix): adopt_indptr[P+1], ids; empty
  // when nothing is adopted.  They are the first blocks of the prompt's prefix list and are not written by ingest.
  std::vector<int32_t> adopt_indptr, adopt_blk;
  // parked: the blocks were handed back to the pool (their contents staged elsewhere by the caller); the block
  // arrays keep their shape but name no blocks until ps_layout_resume
  bool parked = false;
  // optional third level: roots (contexts several prompts begin with); prompt_root[p] = -1: none
  int32_t num_roots = 0;
  std::vector<int32_t> root_len, prompt_root, root_blk_indptr, root_blk, root_group_indptr, root_group_req;
  // per request: how many leading tokens of its prompt's prefix it attends to; empty = all of them
  std::vector<int32_t> visible;
  bool any_masked = false;           // the plan holds an item with kPsItemMasked
  // request list the items index into: group_req, then the identity list (suffix items), then root_group_req,
  // then the subsets of a sharing group that see into a prefix chunk (only where visible lengths cut a group)
  std::vector<int32_t> req_list;

  // split plan
  ps_plan_options opt{};
  int32_t prefix_variant = PS_VARIANT_WAVE, suffix_variant = PS_VARIANT_WAVE;
  int32_t prefix_chunk = 0, suffix_chunk = 0;
  int32_t max_rows_prefix = 0;       // largest n_req * G over prefix items
  std::vector<ps_item> items;        // row-split shared items, then the other shared (root, prefix) items, then suffix items
  int32_t num_rowsplit_items = 0;    // launched one workgroup each by the prefill kernel, outside the schedules
  int32_t num_prefix_items = 0;      // all shared items: root and prefix, row-split ones included
  std::vector<int32_t> slot_base;    // [R+1]
  int64_t num_slots = 0;

  // persistent-kernel schedules: for a set of items, the items regrouped by workgroup (8 int32 each,
  // workgroup w owns [indptr[w], indptr[w+1])) -- one schedule per launchable set
  struct schedule {
    int64_t off_items = 0, off_indptr = 0;  // blob offsets in words
    int32_t num_wg = 0, max_rows = 0, occ = 1;  // occ: workgroups per compute unit the grid was sized for
    bool stream = true;   // K/V loads of the launch are non-temporal (little of the set's K/V is read by several items)
  };
  schedule sched_prefix, sched_suffix, sched_all;
  // the schedules' contents as packed by the planner (copied into the blob; kept so that a decode step that changes
  // no chunk structure can patch token counts and block offsets instead of planning again)
  struct packed_set {
    std::vector<ps_item> items;
    std::vector<int32_t> indptr;
    int32_t max_rows = 0, occ = 1;
    bool stream = true;
  };
  packed_set pk_prefix, pk_suffix, pk_all;
  // per request: tokens per suffix chunk and number of suffix chunks in the current plan; where the root blocks
  // started in the concatenated block array when the plan was made
  std::vector<int32_t> suffix_chunk_size, suffix_chunks;
  int32_t planned_root_blk0 = 0;
  // upload staging (abi.hip): two pinned host buffers used alternately, so that ps_layout_upload returns as soon as
  // its copy is enqueued and the tables may change again right away; released with the layout
  struct upload_staging;
  mutable upload_staging* staging = nullptr;
  mutable void (*staging_free)(upload_staging*) = nullptr;
  ~ps_layout() {
    if (staging && staging_free) staging_free(staging);
  }
  // directory entries (first source token, valid tokens) of the shared segments' blocks: prefixes, then roots
  std::vector<int32_t> ent_fixed_tok0, ent_fixed_valid;
  // ... and the order in which an ingest walks them: by physical block, within each kind
  std::vector<int32_t> ent_fixed_order;

  // where the token of the most recent ps_layout_append went: block * B + slot per request, -1 = none
  std::vector<int32_t> append_dest;

  // device table blob (int32 words) and section offsets in words
  std::vector<int32_t> blob;
  int64_t off_blk = 0, off_req = 0, off_items = 0, off_slot = 0;
  int64_t off_visible = 0;           // int32[R]: effective visible prefix length of every request
  // for the cache-writing kernels, per entry of the concatenated block array: index of its first token in the
  // ragged source tensor of its kind (prefixes back to back / suffixes back to back) and its number of valid
  // tokens; then append_dest; then, per entry position, the entry an ingest or a stage-in takes there (every kind
  // keeps its range of positions)
  int64_t off_ent_tok0 = 0, off_ent_valid = 0, off_dest = 0, off_ent_order = 0;
};

// Waves per SIMD the MFMA kernel is built for, by the widest row group it must carry.
inline int ps_mfma_occupancy(int max_rows, int kv_dtype) {
  // two workgroups per compute unit where the kernel fits in 256 VGPRs: one 16-row tile, or e4m3 KV
  // (half-size tile buffers) with up to two
  if (max_rows <= 16) return 2;
  if (max_rows <= 32 && kv_dtype == PS_FP8_E4M3) return 2;
  return 1;
}
constexpr int kPsMfmaMaxChunk = 8192;  // tokens per MFMA work item (64 tiles per wave: their block ids fill two registers)

// Compute units of the current device, or 0 if none can be asked.  Null in a build without the device side of the
// library (the planner then assumes kPsDefaultNumCus); abi.hip installs it when the library is loaded.
extern int32_t (*ps_device_num_cus_hook)();
constexpr int32_t kPsDefaultNumCus = 256;   // MI355X

// layout.cpp
int32_t ps_plan_build(ps_layout* lay, const ps_plan_options* opt);
int32_t ps_blob_build(ps_layout* lay);
bool ps_mfma_supported(const ps_geometry& g);
