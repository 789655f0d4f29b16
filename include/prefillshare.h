/*
 * prefillshare.h -- C ABI of the shared-prefix decode attention library for MI355X (gfx950).
 *
 * Setting (PrefillShare, arXiv 2602.12029): a frozen base module prefills a prompt once and
 * produces the shared cache C_base (Method, Eq. 5); each of several task-specific decode modules
 * starts from C <- C_base and appends its own keys/values while decoding (Method, Eq. 6; Background
 * Eq. 2 and Eq. 4).  On the decode GPU a prompt's prefix KV is therefore stored once and read by
 * every model, and each (prompt, model) request owns only its model-specific segment (Efficiency
 * Analysis, Eq. 9: Mem = O(L_shared + N * L_unique)).  This library is the attention of one decode
 * step of one layer for a batch of such requests: a query token per request attends over
 * [shared prefix ; private suffix].
 *
 * Conventions
 *   - Every function returns an int32 status (PS_OK or a PS_ERR_* code); nothing throws.
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory on the
 *     current device.  The caller owns all device memory (KV pool, scales, Q, O, workspace, the
 *     uploaded table blob); the library owns only the opaque host objects it creates.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are enqueued
 *     asynchronously and never synchronise; ps_layout_upload stages the tables in pinned host
 *     memory the layout owns (two buffers, used alternately) and returns once the copy is enqueued.
 *   - q and out are [R][Hq][d] contiguous in q_dtype.  The KV pool is addressed as
 *         elem(block, kv_head, which, slot, c) = block*kv_stride_block + kv_head*kv_stride_head
 *                                               + which*kv_stride_kv + slot*kv_stride_tok + c
 *     (which: 0 = K, 1 = V; strides in elements; the head_dim axis is contiguous; every stride must
 *     be a multiple of 16 bytes; where kv_stride_kv + block_size*kv_stride_tok reaches 2 GiB the
 *     matrix-core kernels do not apply and the plan uses the wavefront kernel).  kv_scales (fp8 only) is [num_blocks][Hkv][2] fp32: K scale, V scale.
 *   - q head h reads KV head h / (Hq / Hkv).  Every stored token of both segments is attended to,
 *     unless ps_layout_set_visible limits how much of the shared prefix a request sees.  Scores are
 *     scaled by 1/sqrt(head_dim).
 *   - A partial state of a set of tokens is (o: the softmax-weighted value average over that set,
 *     fp32[d]; lse: natural-log sum of exp(score) over that set, fp32).  The empty set is (0, -inf).
 */
#ifndef PREFILLSHARE_H
#define PREFILLSHARE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PS_OK = 0,
  PS_ERR_INVALID_ARG = 1, /* NULL pointer, negative size, index out of range, duplicate request   */
  PS_ERR_SHAPE = 2,       /* geometry the kernels cannot address (Hq % Hkv, strides, alignment)    */
  PS_ERR_OOM = 3,         /* the pool has too few free blocks; nothing was allocated              */
  PS_ERR_REFCOUNT = 4,    /* release would drive a refcount below zero (wrong pool)               */
  PS_ERR_UNSUPPORTED = 5, /* dtype / head_dim / block_size combination without a kernel           */
  PS_ERR_DEVICE = 6,      /* a HIP call failed; ps_last_hip_error() returns its code              */
  PS_ERR_TOO_LARGE = 7    /* the batch needs more than a fixed-size buffer of the library holds    */
};

enum { PS_F32 = 0, PS_BF16 = 1, PS_FP8_E4M3 = 2 /* OCP e4m3fn, KV only */ };

/* kernel family used for a pass */
enum { PS_VARIANT_AUTO = 0, PS_VARIANT_WAVE = 1 /* fp32 wavefront-reduction */, PS_VARIANT_MFMA = 2 };

typedef struct ps_pool ps_pool;     /* host: free list + refcounts of the physical blocks          */
typedef struct ps_layout ps_layout; /* host: block tables, sharing groups and split plan of a batch */

typedef struct ps_geometry {
  int32_t num_q_heads, num_kv_heads, head_dim, block_size;
  int32_t q_dtype, kv_dtype;
  int64_t kv_stride_block, kv_stride_head, kv_stride_kv, kv_stride_tok; /* in elements */
} ps_geometry;

typedef struct ps_plan_options {
  int32_t prefix_chunk_tokens; /* tokens of a shared prefix handled by one workgroup; 0 = choose  */
  int32_t suffix_chunk_tokens; /* same for private suffixes; 0 = choose                           */
  int32_t prefix_variant;      /* PS_VARIANT_*                                                    */
  int32_t suffix_variant;      /* PS_VARIANT_*                                                    */
  int32_t num_cus;             /* compute units to plan for; 0 = those of the current device (256
                                  on MI355X, which is also assumed where no device is visible)    */
  int32_t kv_cache_policy;     /* PS_KV_POLICY_*: how the matrix-core decode kernel loads K/V     */
} ps_plan_options;

/* K/V loads of the matrix-core decode kernel.  STREAM: non-temporal (the bytes are wanted once: they
 * do not displace what the caches hold); CACHEABLE: ordinary loads (several row groups of a sharing
 * group read the same range and should meet in L2); AUTO: per launch, STREAM unless a quarter or more
 * of the launch's tokens lie in ranges that several items read.  The results are the same bits. */
enum { PS_KV_POLICY_AUTO = 0, PS_KV_POLICY_STREAM = 1, PS_KV_POLICY_CACHEABLE = 2 };

/* ---- block pool (pool of cached KV blocks, Background "Prefix Caching") -------------------------
 * ps_pool_create: num_blocks >= 0; free_order = host permutation of [0, num_blocks) giving the
 * initial free-list order, or NULL for ascending.  *out receives the pool. */
int32_t ps_pool_create(int32_t num_blocks, const int32_t* free_order, ps_pool** out);
int32_t ps_pool_destroy(ps_pool* pool);
int32_t ps_pool_num_free(const ps_pool* pool, int32_t* out);
/* Copies the free list (head first) into host out[capacity]; *count receives its length. */
int32_t ps_pool_free_list(const ps_pool* pool, int32_t* out, int32_t capacity, int32_t* count);
/* *refcount points at the pool's own int32[num_blocks]; valid until ps_pool_destroy. */
int32_t ps_pool_refcounts(const ps_pool* pool, const int32_t** refcount);

/* ---- ps_kv_layout: the refcounted two-segment block table (Eq. 6 "C <- C_base", Eq. 9) ----------
 * Builds the table of one decode batch.  Host inputs: prefix_len[P]; for each request its prompt
 * index, model index and private suffix length (tokens; 0 allowed).  Policy: prompts in ascending
 * index take ceil(Lp/B) blocks each from the head of the free list, then requests in ascending index
 * take ceil(Ls/B) private blocks each; a prefix block's refcount rises by the number of requests on
 * that prompt, a private block's by 1.  A partially filled last prefix block stays shared and
 * read-only; a private segment always starts in a fresh block.  Also derives a split plan (how the
 * segments are cut into workgroup-sized chunks) with default options.
 * Errors: PS_ERR_INVALID_ARG (NULL, negative length, unknown prompt, duplicate (prompt, model), a
 * prompt with no request), PS_ERR_SHAPE / PS_ERR_UNSUPPORTED (geometry), PS_ERR_OOM (pool untouched). */
int32_t ps_kv_layout(ps_pool* pool, const ps_geometry* geometry,
                     int32_t num_prompts, const int32_t* prefix_len,
                     int32_t num_requests, const int32_t* req_prompt, const int32_t* req_model,
                     const int32_t* suffix_len, ps_layout** out);
/* ps_kv_layout_tree: the same table with a third sharing level.  Several prompts may begin with one context
 * (Background, "Multi-Model Inference and Prefix Caching": a common system prompt or a shared document in front of
 * each session's own history); such a root is stored once, as a prompt's prefix is stored once for its models (Eq. 9
 * applied one level up).  Host inputs as above plus root_len[num_roots] and prompt_root[P] (index of the root prompt
 * p begins with, -1 = none); prefix_len[p] is then the prompt's own part, and request r on prompt p attends over
 * [root ; prefix p ; suffix r].  Policy: roots in ascending index take ceil(L/B) blocks each first, then prompts and
 * requests as in ps_kv_layout; a root block's refcount rises by the number of requests below the root; a root's
 * partially filled last block stays shared and read-only, and a prompt's own prefix starts in a fresh block.
 * num_roots = 0 is ps_kv_layout.  Additional errors: PS_ERR_INVALID_ARG for a root index out of range or a root no
 * prompt begins with.  A request's partial states are numbered root splits, prefix splits, suffix splits. */
int32_t ps_kv_layout_tree(ps_pool* pool, const ps_geometry* geometry, int32_t num_roots, const int32_t* root_len,
                          int32_t num_prompts, const int32_t* prompt_root, const int32_t* prefix_len,
                          int32_t num_requests, const int32_t* req_prompt, const int32_t* req_model,
                          const int32_t* suffix_len, ps_layout** out);
/* ps_kv_layout_adopt: ps_kv_layout for a batch that continues cached contexts.  Prefix-aware routing sends a session
 * back to the worker that holds its cache, so that the cache is extended rather than rebuilt (System Design,
 * prefix-aware routing), and the context grows as X(i) = [X(i-1); Y(i)] (System Design, execution pipeline): the
 * layout of the next step -- the partial prefill of Y(i), or the next decode batch over X(i) -- adopts the blocks that
 * already hold the beginning of its prompts.  adopt_indptr[P+1], adopt_blk[..]: for prompt p the physical ids of its first
 * n = adopt_indptr[p+1] - adopt_indptr[p] prefix blocks, taken over from a layout that still holds them.  Only full
 * blocks are adopted (n * block_size <= prefix_len[p]); each gains one reference per request on the prompt, like a
 * block from the free list, and stays alive until the last layout referencing it is released; the other
 * ceil(Lp/B) - n blocks come from the free list as usual.  ps_kv_ingest(which = 0) on such a layout leaves the adopted
 * blocks alone: its source holds, per prompt, only the tokens from n * block_size on.  A parked layout gives up its
 * adoptions: its image holds the adopted blocks' contents and a resume takes fresh blocks for all of them.
 * Additional errors: PS_ERR_INVALID_ARG for an adopted id that is out of range, not referenced by any layout, or
 * named twice, and for more adopted blocks than the prefix has full blocks. */
int32_t ps_kv_layout_adopt(ps_pool* pool, const ps_geometry* geometry, int32_t num_prompts, const int32_t* prefix_len,
                           const int32_t* adopt_indptr, const int32_t* adopt_blk, int32_t num_requests,
                           const int32_t* req_prompt, const int32_t* req_model, const int32_t* suffix_len,
                           ps_layout** out);
/* Host views of the root level (valid until release; any output pointer may be NULL): root_blk_indptr[T+1],
 * root_blk[..], root_group_indptr[T+1], root_group_req[..] (the requests below a root, ascending). */
int32_t ps_layout_root_tables(const ps_layout* layout, int32_t* num_roots, const int32_t** root_blk_indptr,
                              const int32_t** root_blk, const int32_t** root_group_indptr,
                              const int32_t** root_group_req);
/* Drops the batch's references (blocks reaching zero join the free-list tail in ascending id) and
 * destroys the layout.  PS_ERR_REFCOUNT leaves pool and layout unchanged. */
int32_t ps_layout_release(ps_pool* pool, ps_layout* layout);
/* Host views of the tables (int32, CSR), valid until release.  Any output pointer may be NULL.
 * prefix_blk_indptr[P+1], prefix_blk[..], group_indptr[P+1], group_req[R] (a prompt's requests,
 * ascending), suffix_blk_indptr[R+1], suffix_blk[..]. */
int32_t ps_layout_tables(const ps_layout* layout,
                         const int32_t** prefix_blk_indptr, const int32_t** prefix_blk,
                         const int32_t** group_indptr, const int32_t** group_req,
                         const int32_t** suffix_blk_indptr, const int32_t** suffix_blk);

/* Host views of the segment lengths in tokens (prefix_len[P], suffix_len[R]); suffix_len changes with
 * ps_layout_append.  Valid until release. */
int32_t ps_layout_lengths(const ps_layout* layout, const int32_t** prefix_len, const int32_t** suffix_len);

/* ---- split plan -------------------------------------------------------------------------------
 * Re-derives the plan with explicit options (NULL = defaults).  Invalidates earlier uploads of this
 * layout's table blob and the sizes reported below. */
int32_t ps_layout_replan(ps_layout* layout, const ps_plan_options* options);
/* Plan introspection (host, valid until the next replan/release).  items is int32[num_items][8]:
 * {first block index in the concatenated (prefix ++ suffix ++ root) block array, token begin, token end,
 *  first index into the request list, number of requests, kv head, split index within the request's
 *  partial states, 0 = prefix / 1 = suffix}.  slot_base is int32[R+1]: request r owns partial-state
 * slots [slot_base[r], slot_base[r+1]), prefix splits first. */
int32_t ps_layout_plan(const ps_layout* layout, int32_t* num_items, const int32_t** items,
                       const int32_t** slot_base, int32_t* prefix_variant, int32_t* suffix_variant);
/* The request list the items index into (host view, valid until the next replan/release): a prompt's
 * requests in ascending order for every prompt (group_req), then 0..R-1 (private-suffix items), then
 * root_group_req, then, where visible lengths keep part of a sharing group out of a prefix chunk, the sub-lists of those
 * chunks.  The last field of an item is a bit set: bit 0 = private suffix, bit 1 = some row of the item
 * sees fewer tokens than the item's token end, bit 2 = an item of up to 256 rows (the new tokens of a
 * context in a partial prefill, the requests below a root), which a workgroup of the prefill kernel splits
 * over its waves by rows (such items lead the item array and are not part of the schedules below), bit 3 =
 * a root segment, bit 4 = further items (other row groups of the same sharing group) read the same K/V
 * range (see PS_KV_POLICY_AUTO). */
int32_t ps_layout_request_list(const ps_layout* layout, int32_t* count, const int32_t** list);

/* Schedule of the persistent matrix-core kernel for one launchable set of items (which: 0 = prefix items,
 * 1 = suffix items, 2 = both): the set's items regrouped by workgroup, int32[n][8] in the item format
 * above, workgroup w owning rows [indptr[w], indptr[w+1]).  Items are packed longest-first onto
 * num_cus x (resident workgroups per compute unit) workgroups.  *num_workgroups is 0 where the set does not
 * run on the matrix-core kernel.  Host views, valid until the next replan/release. */
int32_t ps_layout_schedule(const ps_layout* layout, int32_t which, int32_t* num_workgroups,
                           const int32_t** items, const int32_t** indptr);

/* Size of the int32 table blob, and its copy to device memory (at least that many bytes, 16-byte
 * aligned) on `stream`.  The copy is asynchronous: the layout may be changed (ps_layout_append,
 * ps_layout_replan) as soon as the call returns; kernels that use dev_tables must follow on the same
 * stream or be ordered behind it by the caller.  The third upload of a layout waits on the host for the
 * first one's copy, the fourth for the second's, and so on. */
int64_t ps_layout_device_bytes(const ps_layout* layout);
int32_t ps_layout_upload(const ps_layout* layout, void* dev_tables, void* stream);
/* Partial-state workspace: fp32 o[num_slots][Hq][d] followed, at lse_offset_bytes, by fp32
 * lse[num_slots][Hq]. */
int64_t ps_workspace_bytes(const ps_layout* layout);
int32_t ps_workspace_layout(const ps_layout* layout, int64_t* num_slots, int64_t* lse_offset_bytes);

/* ---- attention passes (device pointers; asynchronous on `stream`) ---------------------------------
 * What all of them compute (Background Eq. 2 and Eq. 4: a decode step attends to the whole cache; Method Eq. 6: the
 * cache of a decode module is C_base followed by the entries the module appended itself): for request r on prompt p
 * and q head h, softmax attention of the one query row over [shared prefix of p ; private suffix of r].
 *
 * ps_prefix_attention (Method Eq. 5-6: C_base is produced once and every decode module starts from it; Efficiency
 * Analysis Eq. 9: it is stored once): for every prompt, KV head and chunk of the prompt's shared prefix, streams the
 * chunk's K/V blocks once and applies them to the queries of every request on that prompt and every q head of the
 * KV head's group; writes one partial state per (request, q head, prefix split).
 * ps_suffix_attention (Method Eq. 6, the entries a decode module appended; the N * L_unique term of Eq. 9): the same
 * over each request's private blocks (flash-decoding split over tokens).
 * Both write only their own slots of `workspace` (device, ps_workspace_bytes, 16-byte aligned, caller-owned).
 * Errors: PS_ERR_INVALID_ARG (null layout / tables / workspace, null q or kv_pool with work to do, null kv_scales
 * for an e4m3 pool, a parked layout), PS_ERR_UNSUPPORTED (no kernel for the geometry), PS_ERR_DEVICE. */
int32_t ps_prefix_attention(const ps_layout* layout, const void* dev_tables, const void* q,
                            const void* kv_pool, const float* kv_scales, void* workspace, void* stream);
int32_t ps_suffix_attention(const ps_layout* layout, const void* dev_tables, const void* q,
                            const void* kv_pool, const float* kv_scales, void* workspace, void* stream);
/* ps_prefix_suffix_attention: both passes; where they run the same kernel family the two work lists go
 * out as one launch (this is the attention part of ps_decode_attention). */
int32_t ps_prefix_suffix_attention(const ps_layout* layout, const void* dev_tables, const void* q,
                                   const void* kv_pool, const float* kv_scales, void* workspace, void* stream);
/* ps_merge_states (softmax algebra over the concatenated cache of Background Eq. 2: the attention over
 * [prefix ; suffix] is the weighted combination of the attentions over its parts): per (request, q head) combines
 * the request's partial states, lse = log sum_i exp(lse_i), o = sum_i exp(lse_i - lse) o_i, and writes
 * out[R][Hq][d] in q_dtype (bf16: round to nearest even) and, if out_lse != NULL, lse as fp32 [R][Hq].  A request
 * with no tokens at all gets o = 0, lse = -inf.  `workspace` may have been filled by the two passes or by the
 * caller in the documented format. */
int32_t ps_merge_states(const ps_layout* layout, const void* dev_tables, const void* workspace,
                        void* out, float* out_lse, void* stream);
/* ps_decode_attention (Background Eq. 2 / Eq. 4, Method Eq. 6: one decode step's attention over the whole cache):
 * the whole step -- ps_prefix_suffix_attention, then ps_merge_states -- on one stream. */
int32_t ps_decode_attention(const ps_layout* layout, const void* dev_tables, const void* q,
                            const void* kv_pool, const float* kv_scales, void* workspace,
                            void* out, float* out_lse, void* stream);
/* ps_decode_attention_static: ps_decode_attention for callers that cannot allocate device memory -- code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The partial states go to a buffer of
 * PS_STATIC_WORKSPACE_BYTES that lives in the library's device image (one per GPU, held until the process ends)
 * instead of a caller-provided workspace; everything else is as in ps_decode_attention (the caller still passes the
 * uploaded tables, q, the pool, out).  The call allocates nothing, on the host or on the device.
 * PS_ERR_TOO_LARGE: ps_workspace_bytes(layout) exceeds PS_STATIC_WORKSPACE_BYTES; nothing is launched.
 * Every call on a GPU uses that GPU's one buffer: calls that overlap on one GPU (two streams, two threads) race, and
 * the caller must order them.  Nothing in the buffer needs clearing between calls (the attention passes write every
 * partial state of the batch before the merge reads it); it keeps the last call's contents. */
#define PS_STATIC_WORKSPACE_BYTES (64ll << 20)
int32_t ps_decode_attention_static(const ps_layout* layout, const void* dev_tables, const void* q,
                                   const void* kv_pool, const float* kv_scales, void* out, float* out_lse,
                                   void* stream);

/* ---- partial prefill: per-request visible prefix length ------------------------------------------------
 * When a context grows by a segment, the prefill worker extends the shared cache only for the newly
 * appended tokens (System Design, execution pipeline step 1; Appendix B.1: a cache hit on the old context,
 * KV states computed for the new tokens only).  The attention of such a chunk is this library's step with
 * one request per new token: the chunk's keys/values are stored as the continuation of the prompt's shared
 * prefix, and the request of the token at position t of the context sees the first t + 1 tokens of it --
 * causal attention written as a length.
 *
 * ps_layout_set_visible (host): prefix_visible = int32[R], request r attends to the first prefix_visible[r]
 * tokens of its prompt's shared prefix (0 <= prefix_visible[r] <= prefix length) and to its whole private
 * suffix; NULL restores full visibility.  Re-derives the split plan with the options last used (a request
 * gets partial states only for the prefix chunks it sees into), so earlier uploads of the table blob and the
 * sizes reported by ps_layout_device_bytes / ps_workspace_bytes are invalid afterwards.  Block tables and
 * refcounts do not change.  Where the matrix-core kernels apply and a sharing group has more than 64 query
 * rows per KV head (the new tokens of a context), the group goes out in items of up to 256 rows that run in the
 * prefill kernel.  PS_ERR_INVALID_ARG: a length out of range; the layout is unchanged. */
int32_t ps_layout_set_visible(ps_layout* layout, const int32_t* prefix_visible);

/* ---- cache growth -------------------------------------------------------------------------------------
 * A decode step returns the step's new cache entries, which are appended to the decode module's own cache
 * (Method Eq. 6; Background Eq. 2 and Eq. 4); the shared prefix cache comes from a prefill worker and is
 * handed to the decode workers (Method Eq. 5; System Design, execution pipeline steps 1 and 3).
 *
 * ps_layout_append (host): one step of table growth.  active = int32[R], non-zero where the request appends a
 * token, or NULL = every request.  Requests in ascending index; a request whose private length is a multiple
 * of the block size (no private block yet, or its last one is full) first takes the block at the head of the
 * free list (refcount 1); then its private length grows by one.  Shared prefix blocks are never written.
 * Re-derives the split plan with the options last used, so earlier uploads of the table blob and the sizes
 * reported by ps_layout_device_bytes / ps_workspace_bytes are invalid afterwards.  *dest (may be NULL)
 * receives a host view int32[R], valid until the next append/release: block * block_size + slot where the
 * request's new token belongs, -1 for inactive requests.  PS_ERR_OOM: too few free blocks, nothing changed.
 * PS_ERR_INVALID_ARG also for pools with more than 2^31 slots. */
int32_t ps_layout_append(ps_pool* pool, ps_layout* layout, const int32_t* active, const int32_t** dest);

/* ps_kv_append (device, asynchronous): stores the tokens reserved by the last ps_layout_append.  dev_tables
 * must be an upload made after that call.  new_k, new_v: device [R][Hkv][d] contiguous, bf16 for bf16 and
 * e4m3 pools, float32 for float32 pools; rows of inactive requests are ignored.  bf16 / float32 pools
 * store the bits.  e4m3 pools, per (block, KV head) and separately for K and V, with a = max |x| of the new
 * token in float32: the tile's scale becomes max(old scale, a / 448) (slot 0 of a fresh block: a / 448, or 1
 * if a = 0); if it grew, the tokens already in the tile are re-encoded from their stored values,
 * (decode(code) * old) / new in float32; the new token is stored as the round-to-nearest-even e4m3fn code of
 * x / scale.  kv_scales is read and written. */
int32_t ps_kv_append(const ps_layout* layout, const void* dev_tables, const void* new_k, const void* new_v,
                     void* kv_pool, float* kv_scales, void* stream);

/* ps_kv_ingest (device, asynchronous): stores whole segments handed over as contiguous tensors.  which: 0 =
 * every prompt's shared prefix, 1 = every request's private suffix, 2 = every root.  src_k, src_v: device, token-major
 * [T][Hkv][d] with T = the sum of the segment lengths of that kind, segments back to back in index order;
 * element (t, h, c) at t * src_stride_tok + h * src_stride_head + c (strides in elements, multiples of 16
 * bytes, base pointers 16-byte aligned); bf16 for bf16 and e4m3 pools, float32 for float32 pools.  Token j of
 * a segment goes to slot j % block_size of the segment's block j / block_size; slots past the segment's
 * length are not written.  e4m3 pools: per (block, KV head), separately for K and V, a = max |x| over the
 * tile's valid tokens, scale = a / 448 in float32 (1 if a = 0), code = round-to-nearest-even e4m3fn of
 * x / scale (float32 division); kv_scales is written.  PS_ERR_UNSUPPORTED: head_dim not a multiple of 8
 * (4 for float32), or an e4m3 tile of more than 16384 elements. */
int32_t ps_kv_ingest(const ps_layout* layout, const void* dev_tables, int32_t which, const void* src_k,
                     const void* src_v, int64_t src_stride_tok, int64_t src_stride_head, void* kv_pool,
                     float* kv_scales, void* stream);

/* ---- staging of cold KV and admission (Appendix B.2, "KV transfer and staging at high concurrency") -------------
 * When the resident KV of the decode side exceeds the GPU's capacity, the caches of sessions that are not scheduled
 * are staged in CPU memory and reloaded when their sessions run again; admission control and reservation of KV blocks
 * are the alternatives the paper names.  The unit here is a batch layout: it is *parked* (its blocks copied to a
 * staging image, its references dropped, the blocks back in the pool) and later *resumed* (blocks taken again by the
 * ordinary policy -- in general other physical blocks -- and the image copied back).
 *
 * ps_blocks_needed (host): blocks a batch would take, sum over roots, prompts and requests of ceil(len / block_size)
 * (Eq. 9); a batch can be admitted if this does not exceed ps_pool_num_free.  root_len may be NULL with num_roots = 0.
 * ps_layout_state (host): the blocks this layout takes (the same count from its current lengths) and whether it is
 * parked.
 * ps_stage_layout (host): the staging image of this layout: its blocks in table order (prefix blocks, suffix
 * blocks, root blocks: the order of the concatenated block array), each block whole and dense,
 * [kv_head][K|V][slot][head_dim] in the pool's element type (*block_bytes each); e4m3 pools append the blocks'
 * scales [block][kv_head][K|V] float32 at *scales_offset_bytes; *total_bytes is the size to allocate.
 * ps_kv_stage_out / ps_kv_stage_in (device, asynchronous on `stream`): copy the layout's blocks to / from `image`
 * (16-byte aligned; device memory, or pinned host memory that the device can address -- then the copy crosses PCIe
 * inside the kernel).  dev_tables must be a current upload.  Bits are copied, nothing is converted.
 * ps_layout_park (host): drops the layout's references as ps_layout_release does (blocks that reach zero join the
 * free-list tail in ascending id) but keeps the layout; call it after ps_kv_stage_out has completed.  Every device
 * call and ps_layout_append on a parked layout return PS_ERR_INVALID_ARG; ps_layout_release still works.
 * ps_layout_resume (host): takes blocks again (roots, prompts, requests, from the head of the free list as it is
 * now) and re-derives the plan with the options last used; upload the tables again, then ps_kv_stage_in.
 * PS_ERR_OOM: the batch does not fit; pool and layout unchanged, still parked. */
int32_t ps_blocks_needed(int32_t block_size, int32_t num_roots, const int32_t* root_len, int32_t num_prompts,
                         const int32_t* prefix_len, int32_t num_requests, const int32_t* suffix_len, int64_t* out);
int32_t ps_layout_state(const ps_layout* layout, int64_t* num_blocks, int32_t* parked);
int32_t ps_stage_layout(const ps_layout* layout, int64_t* block_bytes, int64_t* scales_offset_bytes,
                        int64_t* total_bytes);
int32_t ps_kv_stage_out(const ps_layout* layout, const void* dev_tables, const void* kv_pool, const float* kv_scales,
                        void* image, void* stream);
int32_t ps_kv_stage_in(const ps_layout* layout, const void* dev_tables, const void* image, void* kv_pool,
                       float* kv_scales, void* stream);
int32_t ps_layout_park(ps_pool* pool, ps_layout* layout);
int32_t ps_layout_resume(ps_pool* pool, ps_layout* layout);

const char* ps_strerror(int32_t status);
int32_t ps_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PREFILLSHARE_H */
