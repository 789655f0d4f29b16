// Device-facing entry points of the C ABI: table upload and the attention passes.
#include <hip/hip_runtime.h>

#include <cmath>

#include "device_common.h"
#include "launch.h"

namespace {

thread_local int32_t g_last_hip_error = 0;

int32_t check_hip(hipError_t e) {
  if (e == hipSuccess) return PS_OK;
  g_last_hip_error = int32_t(e);
  return PS_ERR_DEVICE;
}

psdev::AttnParams make_params(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv,
                              const float* scales, void* workspace) {
  const int32_t* t = static_cast<const int32_t*>(dev_tables);
  const ps_geometry& g = lay->geo;
  psdev::AttnParams p{};
  p.blk = t + lay->off_blk;
  p.req_list = t + lay->off_req;
  p.items = reinterpret_cast<const ps_item*>(t + lay->off_items);
  p.slot_base = t + lay->off_slot;
  p.q = q;
  p.kv = kv;
  p.scales = scales;
  p.ws_o = static_cast<float*>(workspace);
  p.ws_lse = p.ws_o + lay->num_slots * g.num_q_heads * int64_t(g.head_dim);
  p.num_q_heads = g.num_q_heads;
  p.num_kv_heads = g.num_kv_heads;
  p.group = g.num_q_heads / g.num_kv_heads;
  p.block_size = g.block_size;
  p.s_block = g.kv_stride_block;
  p.s_head = g.kv_stride_head;
  p.s_kv = g.kv_stride_kv;
  p.s_tok = g.kv_stride_tok;
  p.scale_log2 = float(1.4426950408889634 / std::sqrt(double(g.head_dim)));
  return p;
}

int32_t launch_range(const ps_layout* lay, const psdev::AttnParams& p, int variant, int begin, int count,
                     hipStream_t st) {
  if (count <= 0) return PS_OK;
  int32_t rc;
  if (variant == PS_VARIANT_MFMA) {
    // widest row group in the range decides how many 16-row tiles the kernel carries
    const int group = lay->geo.num_q_heads / lay->geo.num_kv_heads;
    int max_rows = 0;
    if (begin < lay->num_prefix_items) max_rows = lay->max_rows_prefix;
    if (begin + count > lay->num_prefix_items) max_rows = max_rows > group ? max_rows : group;
    rc = psdev::launch_mfma_attention(p, lay->geo, max_rows, begin, count, st);
  } else
  {
    rc = psdev::launch_wave_attention(p, lay->geo, begin, count, st);
  }
  if (rc != PS_OK) return rc;
  return check_hip(hipGetLastError());
}

int32_t check_pass_args(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv,
                        const float* scales, const void* workspace) {
  if (!lay || !dev_tables || !workspace) return PS_ERR_INVALID_ARG;
  if (!lay->items.empty() && (!q || !kv)) return PS_ERR_INVALID_ARG;
  if (lay->geo.kv_dtype == PS_FP8_E4M3 && !scales && !lay->items.empty()) return PS_ERR_INVALID_ARG;
  return PS_OK;
}

}  // namespace

extern "C" {

int32_t ps_last_hip_error(void) { return g_last_hip_error; }

int32_t ps_layout_upload(const ps_layout* lay, void* dev_tables, void* stream) {
  if (!lay || !dev_tables) return PS_ERR_INVALID_ARG;
  return check_hip(hipMemcpyAsync(dev_tables, lay->blob.data(), lay->blob.size() * sizeof(int32_t),
                                  hipMemcpyHostToDevice, static_cast<hipStream_t>(stream)));
}

int32_t ps_prefix_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                            const float* kv_scales, void* workspace, void* stream) {
  if (int32_t st = check_pass_args(lay, dev_tables, q, kv_pool, kv_scales, workspace)) return st;
  const psdev::AttnParams p = make_params(lay, dev_tables, q, kv_pool, kv_scales, workspace);
  return launch_range(lay, p, lay->prefix_variant, 0, lay->num_prefix_items, static_cast<hipStream_t>(stream));
}

int32_t ps_suffix_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                            const float* kv_scales, void* workspace, void* stream) {
  if (int32_t st = check_pass_args(lay, dev_tables, q, kv_pool, kv_scales, workspace)) return st;
  const psdev::AttnParams p = make_params(lay, dev_tables, q, kv_pool, kv_scales, workspace);
  return launch_range(lay, p, lay->suffix_variant, lay->num_prefix_items,
                      int(lay->items.size()) - lay->num_prefix_items, static_cast<hipStream_t>(stream));
}

int32_t ps_merge_states(const ps_layout* lay, const void* dev_tables, const void* workspace, void* out,
                        float* out_lse, void* stream) {
  if (!lay || !dev_tables || !workspace) return PS_ERR_INVALID_ARG;
  if (lay->num_requests && !out) return PS_ERR_INVALID_ARG;
  const psdev::AttnParams p = make_params(lay, dev_tables, nullptr, nullptr, nullptr, const_cast<void*>(workspace));
  if (int32_t rc = psdev::launch_merge(p.slot_base, p.ws_o, p.ws_lse, out, out_lse, lay->num_requests, lay->geo,
                                       static_cast<hipStream_t>(stream)))
    return rc;
  return check_hip(hipGetLastError());
}

int32_t ps_prefix_suffix_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                                   const float* kv_scales, void* workspace, void* stream) {
  if (int32_t st = check_pass_args(lay, dev_tables, q, kv_pool, kv_scales, workspace)) return st;
  const psdev::AttnParams p = make_params(lay, dev_tables, q, kv_pool, kv_scales, workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int n_all = int(lay->items.size());
  if (lay->prefix_variant == lay->suffix_variant)  // same kernel: one launch over the whole work list
    return launch_range(lay, p, lay->prefix_variant, 0, n_all, st);
  if (int32_t rc = launch_range(lay, p, lay->prefix_variant, 0, lay->num_prefix_items, st)) return rc;
  return launch_range(lay, p, lay->suffix_variant, lay->num_prefix_items, n_all - lay->num_prefix_items, st);
}

int32_t ps_decode_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                            const float* kv_scales, void* workspace, void* out, float* out_lse, void* stream) {
  if (lay && lay->num_requests && !out) return PS_ERR_INVALID_ARG;
  if (int32_t rc = ps_prefix_suffix_attention(lay, dev_tables, q, kv_pool, kv_scales, workspace, stream)) return rc;
  return ps_merge_states(lay, dev_tables, workspace, out, out_lse, stream);
}

}  // extern "C"
