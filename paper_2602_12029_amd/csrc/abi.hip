// Device-facing entry points of the C ABI: table upload and the attention passes.
#include <hip/hip_runtime.h>

#include <cmath>

#include "device_common.h"
#include "launch.h"
#include "prefillshare_probe.h"
#include <atomic>
#include <cstring>
#include <new>

// Partial-state workspace for callers that cannot allocate (ps_decode_attention_static): part of the library's device
// image, so every GPU the library runs on holds one copy at its own address until the process ends.  In host code
// this name only stands for the symbol; its device address comes from hipGetSymbolAddress (static_workspace below).
static __device__ __align__(256) unsigned char scratch[PS_STATIC_WORKSPACE_BYTES];

struct ps_layout::upload_staging {
  void* buffer[2] = {nullptr, nullptr};   // pinned host memory
  size_t capacity[2] = {0, 0};
  hipEvent_t done[2] = {nullptr, nullptr};   // recorded behind the copy that reads the buffer
  bool in_use[2] = {false, false};
  int next = 0;
};

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
  p.visible = t + lay->off_visible;
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

void free_upload_staging(ps_layout::upload_staging* s) {
  for (int i = 0; i < 2; ++i) {
    if (s->in_use[i]) (void)hipEventSynchronize(s->done[i]);
    if (s->done[i]) (void)hipEventDestroy(s->done[i]);
    if (s->buffer[i]) (void)hipHostFree(s->buffer[i]);
  }
  delete s;
}

// Compute units of the current device (asked once per device), 0 if there is no device to ask: the planner's
// default for ps_plan_options.num_cus = 0.
constexpr int kMaxDevices = 64;
int32_t current_device_num_cus() {
  static std::atomic<int32_t> cached[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
  if (const int32_t known = cached[dev].load(std::memory_order_relaxed)) return known;
  int count = 0;
  if (hipDeviceGetAttribute(&count, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || count <= 0) return 0;
  cached[dev].store(count, std::memory_order_relaxed);
  return count;
}
const struct HookInstaller {
  HookInstaller() { ps_device_num_cus_hook = current_device_num_cus; }
} g_hook_installer;

// Device address of `scratch` on the current device, resolved once per device with that device current.
int32_t static_workspace(void** out) {
  static std::atomic<void*> resolved[kMaxDevices];
  int dev = -1;
  if (int32_t st = check_hip(hipGetDevice(&dev))) return st;
  if (dev < 0 || dev >= kMaxDevices) return PS_ERR_UNSUPPORTED;
  void* ptr = resolved[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (int32_t st = check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)))) return st;
    if (!ptr) return PS_ERR_DEVICE;
    resolved[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return PS_OK;
}

enum class WorkSet { kPrefix, kSuffix, kAll };

// Launches one set of work items with the kernel family the plan chose for it.
int32_t launch_set(const ps_layout* lay, const psdev::AttnParams& p, const void* dev_tables, WorkSet set,
                   hipStream_t st) {
  const int n_all = int(lay->items.size());
  const int begin = set == WorkSet::kSuffix ? lay->num_prefix_items : 0;
  const int end = set == WorkSet::kPrefix ? lay->num_prefix_items : n_all;
  if (end <= begin) return PS_OK;
  const int variant = set == WorkSet::kSuffix ? lay->suffix_variant : lay->prefix_variant;
  int32_t rc;
  if (variant == PS_VARIANT_MFMA) {
    const ps_layout::schedule& s = set == WorkSet::kPrefix ? lay->sched_prefix
                                   : set == WorkSet::kSuffix ? lay->sched_suffix : lay->sched_all;
    const int32_t* t = static_cast<const int32_t*>(dev_tables);
    rc = PS_OK;
    // the row-split prefix items (partial prefill) lead the item array and run one workgroup each
    if (set != WorkSet::kSuffix && lay->num_rowsplit_items > 0)
      rc = psdev::launch_prefill_attention(p, lay->geo, p.items, lay->num_rowsplit_items, st);
    if (rc == PS_OK)
      rc = psdev::launch_mfma_attention(p, lay->geo, s.max_rows, s.occ, set != WorkSet::kSuffix && lay->any_masked, s.stream,
                                        reinterpret_cast<const ps_item*>(t + s.off_items), t + s.off_indptr, s.num_wg,
                                        st);
  } else {
    rc = psdev::launch_wave_attention(p, lay->geo, begin, end - begin, st);
  }
  if (rc != PS_OK) return rc;
  return check_hip(hipGetLastError());
}

int32_t check_pass_args(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv,
                        const float* scales, const void* workspace) {
  if (!lay || !dev_tables || !workspace || lay->parked) return PS_ERR_INVALID_ARG;
  if (!lay->items.empty() && (!q || !kv)) return PS_ERR_INVALID_ARG;
  if (lay->geo.kv_dtype == PS_FP8_E4M3 && !scales && !lay->items.empty()) return PS_ERR_INVALID_ARG;
  return PS_OK;
}

}  // namespace

extern "C" {

int32_t ps_last_hip_error(void) { return g_last_hip_error; }

int32_t ps_layout_upload(const ps_layout* lay, void* dev_tables, void* stream) {
  if (!lay || !dev_tables) return PS_ERR_INVALID_ARG;
  // The tables go through one of two pinned host buffers the layout owns, so the copy is truly asynchronous: the
  // call returns once it is enqueued, and the next ps_layout_append may rebuild the tables while it is in flight.
  // A buffer is reused two uploads later, after the copy that last read it has finished (an event per buffer).
  if (!lay->staging) {
    lay->staging = new (std::nothrow) ps_layout::upload_staging();
    if (!lay->staging) return PS_ERR_OOM;
    lay->staging_free = free_upload_staging;
  }
  ps_layout::upload_staging* s = lay->staging;
  const int i = s->next;
  s->next ^= 1;
  const size_t bytes = lay->blob.size() * sizeof(int32_t);
  if (s->in_use[i]) {
    if (int32_t st = check_hip(hipEventSynchronize(s->done[i]))) return st;
    s->in_use[i] = false;
  }
  if (s->capacity[i] < bytes) {
    if (s->buffer[i]) (void)hipHostFree(s->buffer[i]);
    s->buffer[i] = nullptr;
    s->capacity[i] = 0;
    const size_t want = bytes + bytes / 4 + 4096;
    if (int32_t st = check_hip(hipHostMalloc(&s->buffer[i], want, hipHostMallocDefault))) return st;
    s->capacity[i] = want;
  }
  if (!s->done[i])
    if (int32_t st = check_hip(hipEventCreateWithFlags(&s->done[i], hipEventDisableTiming))) return st;
  std::memcpy(s->buffer[i], lay->blob.data(), bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (int32_t rc = check_hip(hipMemcpyAsync(dev_tables, s->buffer[i], bytes, hipMemcpyHostToDevice, st))) return rc;
  if (int32_t rc = check_hip(hipEventRecord(s->done[i], st))) return rc;
  s->in_use[i] = true;
  return PS_OK;
}

int32_t ps_prefix_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                            const float* kv_scales, void* workspace, void* stream) {
  if (int32_t st = check_pass_args(lay, dev_tables, q, kv_pool, kv_scales, workspace)) return st;
  const psdev::AttnParams p = make_params(lay, dev_tables, q, kv_pool, kv_scales, workspace);
  return launch_set(lay, p, dev_tables, WorkSet::kPrefix, static_cast<hipStream_t>(stream));
}

int32_t ps_suffix_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                            const float* kv_scales, void* workspace, void* stream) {
  if (int32_t st = check_pass_args(lay, dev_tables, q, kv_pool, kv_scales, workspace)) return st;
  const psdev::AttnParams p = make_params(lay, dev_tables, q, kv_pool, kv_scales, workspace);
  return launch_set(lay, p, dev_tables, WorkSet::kSuffix, static_cast<hipStream_t>(stream));
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
  if (lay->prefix_variant == lay->suffix_variant)  // same kernel: one launch over the whole work list
    return launch_set(lay, p, dev_tables, WorkSet::kAll, st);
  if (int32_t rc = launch_set(lay, p, dev_tables, WorkSet::kPrefix, st)) return rc;
  return launch_set(lay, p, dev_tables, WorkSet::kSuffix, st);
}

int32_t ps_kv_ingest(const ps_layout* lay, const void* dev_tables, int32_t which, const void* src_k, const void* src_v,
                     int64_t src_stride_tok, int64_t src_stride_head, void* kv_pool, float* kv_scales, void* stream) {
  if (!lay || !dev_tables || which < 0 || which > 2 || lay->parked) return PS_ERR_INVALID_ARG;
  const ps_geometry& g = lay->geo;
  const size_t entries = which == 0 ? lay->prefix_blk.size() : (which == 1 ? lay->suffix_blk.size() : lay->root_blk.size());
  if (entries == 0) return PS_OK;
  if (!src_k || !src_v || !kv_pool || (g.kv_dtype == PS_FP8_E4M3 && !kv_scales)) return PS_ERR_INVALID_ARG;
  const int64_t esz = g.kv_dtype == PS_F32 ? 4 : 2;   // source element: float32 for float32 pools, else bf16
  if (src_stride_head < g.head_dim || src_stride_tok < g.head_dim || (src_stride_head * esz) % 16 ||
      (src_stride_tok * esz) % 16 || reinterpret_cast<uintptr_t>(src_k) % 16 || reinterpret_cast<uintptr_t>(src_v) % 16)
    return PS_ERR_SHAPE;
  if (int32_t rc = psdev::launch_kv_ingest(lay, dev_tables, which, src_k, src_v, src_stride_tok, src_stride_head,
                                           kv_pool, kv_scales, static_cast<hipStream_t>(stream)))
    return rc;
  return check_hip(hipGetLastError());
}

int32_t ps_kv_append(const ps_layout* lay, const void* dev_tables, const void* new_k, const void* new_v, void* kv_pool,
                     float* kv_scales, void* stream) {
  if (!lay || !dev_tables || lay->parked) return PS_ERR_INVALID_ARG;
  if (lay->num_requests == 0) return PS_OK;
  if (!new_k || !new_v || !kv_pool || (lay->geo.kv_dtype == PS_FP8_E4M3 && !kv_scales)) return PS_ERR_INVALID_ARG;
  if (int32_t rc = psdev::launch_kv_append(lay, dev_tables, new_k, new_v, kv_pool, kv_scales,
                                           static_cast<hipStream_t>(stream)))
    return rc;
  return check_hip(hipGetLastError());
}

namespace {

int32_t stage(const ps_layout* lay, const void* dev_tables, bool to_image, void* kv_pool, float* kv_scales, void* image,
              void* stream) {
  if (!lay || !dev_tables || lay->parked) return PS_ERR_INVALID_ARG;
  int64_t scales_off = 0, total = 0;
  ps_stage_layout(lay, nullptr, &scales_off, &total);
  if (lay->prefix_blk.empty() && lay->suffix_blk.empty() && lay->root_blk.empty()) return PS_OK;
  if (!kv_pool || !image || (lay->geo.kv_dtype == PS_FP8_E4M3 && !kv_scales)) return PS_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(image) % 16) return PS_ERR_SHAPE;
  if (int32_t rc = psdev::launch_kv_stage(lay, dev_tables, to_image, kv_pool, kv_scales, image, scales_off,
                                          static_cast<hipStream_t>(stream)))
    return rc;
  return check_hip(hipGetLastError());
}

}  // namespace

int32_t ps_kv_stage_out(const ps_layout* lay, const void* dev_tables, const void* kv_pool, const float* kv_scales,
                        void* image, void* stream) {
  return stage(lay, dev_tables, true, const_cast<void*>(kv_pool), const_cast<float*>(kv_scales), image, stream);
}

int32_t ps_kv_stage_in(const ps_layout* lay, const void* dev_tables, const void* image, void* kv_pool, float* kv_scales,
                       void* stream) {
  return stage(lay, dev_tables, false, kv_pool, kv_scales, const_cast<void*>(image), stream);
}

int32_t ps_probe_read(const void* dev_buf, int64_t bytes, int32_t pattern, int32_t num_workgroups, void* stream) {
  if (!dev_buf || bytes < 0 || num_workgroups <= 0 || num_workgroups > 65536 || pattern < 0 || pattern > 6 ||
      reinterpret_cast<uintptr_t>(dev_buf) % 16 != 0)
    return PS_ERR_INVALID_ARG;
  if (int32_t rc = psdev::launch_probe_read(dev_buf, bytes, pattern, num_workgroups, static_cast<hipStream_t>(stream)))
    return rc;
  return check_hip(hipGetLastError());
}

int32_t ps_decode_attention(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                            const float* kv_scales, void* workspace, void* out, float* out_lse, void* stream) {
  if (lay && lay->num_requests && !out) return PS_ERR_INVALID_ARG;
  if (int32_t rc = ps_prefix_suffix_attention(lay, dev_tables, q, kv_pool, kv_scales, workspace, stream)) return rc;
  return ps_merge_states(lay, dev_tables, workspace, out, out_lse, stream);
}

int32_t ps_decode_attention_static(const ps_layout* lay, const void* dev_tables, const void* q, const void* kv_pool,
                                   const float* kv_scales, void* out, float* out_lse, void* stream) {
  if (!lay) return PS_ERR_INVALID_ARG;
  if (ps_workspace_bytes(lay) > PS_STATIC_WORKSPACE_BYTES) return PS_ERR_TOO_LARGE;
  void* workspace = nullptr;
  if (int32_t st = static_workspace(&workspace)) return st;
  // the same launches as ps_decode_attention, with the library's own buffer as the workspace (a kernel argument like
  // any other device pointer); nothing here or below allocates
  return ps_decode_attention(lay, dev_tables, q, kv_pool, kv_scales, workspace, out, out_lse, stream);
}

}  // extern "C"
