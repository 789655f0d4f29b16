// Host-callable launchers of the device passes (defined in the .hip files).
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace psdev {

bool wave_supported(const ps_geometry& g);
int32_t launch_wave_attention(const AttnParams& p, const ps_geometry& g, int item_begin, int n_items, hipStream_t st);
// Persistent launch: workgroup w walks wg_items[wg_indptr[w] .. wg_indptr[w+1]).
// `masked`: the set holds items whose rows see different token counts (per-request visible prefix lengths).
// `stream`: K/V tile loads are non-temporal (the set's K/V is read by one item each, or nearly so).
int32_t launch_mfma_attention(const AttnParams& p, const ps_geometry& g, int max_rows, int occ, bool masked, bool stream,
                              const ps_item* wg_items, const int32_t* wg_indptr, int num_wg, hipStream_t st);
// Partial prefill: one workgroup per row-split item (up to 256 query rows, split over the waves by rows).
int32_t launch_prefill_attention(const AttnParams& p, const ps_geometry& g, const ps_item* items, int num_items,
                                 hipStream_t st);
// Cache writes: whole segments of one kind (0 = shared prefixes, 1 = private suffixes) from ragged contiguous
// sources, and the one token per request reserved by the last ps_layout_append.
int32_t launch_kv_ingest(const ps_layout* lay, const void* dev_tables, int which, const void* src_k, const void* src_v,
                         int64_t src_s_tok, int64_t src_s_head, void* kv, float* scales, hipStream_t st);
int32_t launch_kv_append(const ps_layout* lay, const void* dev_tables, const void* new_k, const void* new_v, void* kv,
                         float* scales, hipStream_t st);
// Whole blocks of a layout, in table order, to (to_image) or from a dense staging image; e4m3 scales follow the
// blocks at scales_offset_bytes.
int32_t launch_kv_stage(const ps_layout* lay, const void* dev_tables, bool to_image, void* kv, float* scales,
                        void* image, int64_t scales_offset_bytes, hipStream_t st);
// Measurement aid: reads `bytes` (whole 8 KiB units of it) once with the load footprint `pattern` names.
int32_t launch_probe_read(const void* buf, int64_t bytes, int pattern, int num_workgroups, hipStream_t st);
int32_t launch_merge(const int32_t* slot_base, const float* ws_o, const float* ws_lse, void* out, float* out_lse,
                     int num_requests, const ps_geometry& g, hipStream_t st);

}  // namespace psdev
