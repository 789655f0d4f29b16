// Writing KV into the paged pool: whole-segment ingest (a prefill worker's shared prefix cache, or a private
// segment produced elsewhere, handed over as contiguous [token][kv_head][d] tensors) and the per-step append
// of one new token per request.  bf16 / float32 pools store the source bits; e4m3 pools quantise per
// (block, kv head) tile with one float32 scale for K and one for V.
//
// Quantiser (every decision in float32 so that results are reproducible bit for bit): a = max |x| over the
// tile's valid tokens, scale = a / 448 (1 if a = 0), code = round-to-nearest-even e4m3fn of x / scale.  An
// append whose token raises the tile's scale re-encodes the tokens already stored from their stored values:
// y = (decode(code) * scale_old) / scale_new.
//
// Both kernels are plain streaming code: one wavefront per (block, kv head, K|V) tile (ingest) or per
// (request, kv head, K|V) row (append); HBM-bound, no matrix work.
#include "device_common.h"
#include "launch.h"

namespace psdev {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Bulk K/V passes through these kernels once and is far larger than the caches: loads and stores are non-temporal,
// so the lines neither displace what the caches hold nor wait there for a reader that never comes.
template <typename V>
__device__ __forceinline__ V stream_load(const V* p) { return __builtin_nontemporal_load(p); }
template <typename V>
__device__ __forceinline__ void stream_store(V* p, V v) { __builtin_nontemporal_store(v, p); }

// e4m3fn code -> float32 (exact)
__device__ __forceinline__ float e4m3_to_f32(uint32_t code) {
  const uint32_t e = (code >> 3) & 0xf, m = code & 7;
  const float mag = e ? __uint_as_float(((e + 120u) << 23) | (m << 20)) : float(m) * 0x1p-9f;
  return (code & 0x80) ? -mag : mag;
}

// two float32 -> two e4m3fn codes in the low 16 bits (v_cvt_pk_fp8_f32: nearest even).  Inputs never reach the
// midpoint above 448 here (|x| <= tile maximum), so saturation behaviour is not relied upon.
__device__ __forceinline__ uint32_t f32x2_to_e4m3(float a, float b) {
  return uint32_t(__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false)) & 0xffffu;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) x = fmaxf(x, lane_xor(x, m));
  return x;
}

struct KvWriteParams {
  const int32_t* blk;        // concatenated block array
  const int32_t* ent_tok0;   // per entry: its first token in the ragged source of its kind
  const int32_t* ent_valid;  // per entry: tokens stored in the block
  const int32_t* ent_order;  // per entry position: the entry an ingest or stage-in takes there (shared kinds by physical block)
  const int32_t* dest;       // [R] block * B + slot of the token being appended, -1 = none
  void* kv;
  float* scales;
  int32_t num_kv_heads, head_dim, block_size;
  int64_t s_block, s_head, s_kv, s_tok;  // pool strides, elements
};

// ---- ingest, storage formats that keep the source bits (T = uint16_t for bf16, float) --------------------
// One wavefront per TILES consecutive (entry, head, K|V) tiles (K and V of neighbouring heads: a contiguous run on
// the pool side in the dense layout); all loads of a step -- four 16-byte pieces per lane and tile -- go out
// before the first store.
template <typename T, int TILES>
__global__ __launch_bounds__(256) void ingest_copy_kernel(KvWriteParams p, const T* __restrict__ src_k,
                                                          const T* __restrict__ src_v, int64_t src_s_tok,
                                                          int64_t src_s_head, int entry0, int num_entries) {
  constexpr int kVec = 16 / int(sizeof(T));
  const int lane = threadIdx.x & 63;
  const int64_t num_tiles = int64_t(num_entries) * p.num_kv_heads * 2;
  const int64_t tile0 = (int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6)) * TILES;
  if (tile0 >= num_tiles) return;
  const int cpt = p.head_dim / kVec;   // 16-byte chunks per token
  const T* src[TILES];
  T* dst[TILES];
  int chunks[TILES];
  int most = 0;
#pragma unroll
  for (int i = 0; i < TILES; ++i) {
    const int64_t tile = min(tile0 + i, num_tiles - 1);
    const int which = int(tile & 1);
    const int h = int((tile >> 1) % p.num_kv_heads);
    const int e = p.ent_order[entry0 + int((tile >> 1) / p.num_kv_heads)];
    // a block adopted from another layout has no valid tokens here: its contents are already there
    chunks[i] = tile0 + i < num_tiles ? max(0, p.ent_valid[e]) * cpt : 0;
    most = max(most, chunks[i]);
    src[i] = (which ? src_v : src_k) + int64_t(p.ent_tok0[e]) * src_s_tok + int64_t(h) * src_s_head;
    dst[i] = static_cast<T*>(p.kv) + int64_t(p.blk[e]) * p.s_block + int64_t(h) * p.s_head + int64_t(which) * p.s_kv;
  }
  for (int c0 = 0; c0 < most; c0 += 256) {
    u32x4 v[TILES][4];
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + 64 * u + lane;
        if (c < chunks[i]) {
          const int t = c / cpt, col = (c % cpt) * kVec;
          v[i][u] = stream_load(reinterpret_cast<const u32x4*>(src[i] + int64_t(t) * src_s_tok + col));
        }
      }
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + 64 * u + lane;
        if (c < chunks[i]) {
          const int t = c / cpt, col = (c % cpt) * kVec;
          stream_store(reinterpret_cast<u32x4*>(dst[i] + int64_t(t) * p.s_tok + col), v[i][u]);
        }
      }
  }
}

// ---- ingest, bf16 source -> e4m3 pool.  CH: 16-byte source chunks a lane keeps in registers; SHIFT >= 0:
// head_dim / 8 chunks per token is 2^SHIFT (index math by shifts), -1: any multiple of 8 ------------------------
template <int CH, int SHIFT>
__global__ __launch_bounds__(256) void ingest_e4m3_kernel(KvWriteParams p, const uint16_t* __restrict__ src_k,
                                                          const uint16_t* __restrict__ src_v, int64_t src_s_tok,
                                                          int64_t src_s_head, int entry0, int num_entries) {
  const int lane = threadIdx.x & 63;
  // wave-uniform tile coordinates (the launcher keeps the tile count under 2^31)
  const uint32_t tile = blockIdx.x * 4u + uint32_t(__builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6));
  if (tile >= uint32_t(num_entries) * uint32_t(p.num_kv_heads) * 2u) return;
  const int which = int(tile & 1u);
  const int h = int((tile >> 1) % uint32_t(p.num_kv_heads));
  const int e = p.ent_order[entry0 + int((tile >> 1) / uint32_t(p.num_kv_heads))];
  const int n_valid = p.ent_valid[e];
  if (n_valid <= 0) return;   // a block adopted from another layout: contents and scale are already there
  const uint16_t* src = (which ? src_v : src_k) + int64_t(p.ent_tok0[e]) * src_s_tok + int64_t(h) * src_s_head;
  const int id = p.blk[e];
  uint8_t* dst = static_cast<uint8_t*>(p.kv) + int64_t(id) * p.s_block + int64_t(h) * p.s_head + int64_t(which) * p.s_kv;
  const int cpt = p.head_dim / 8;
  const int total = n_valid * cpt;
  auto token_of = [&](int c) { return SHIFT >= 0 ? c >> SHIFT : c / cpt; };
  auto column_of = [&](int c) { return (SHIFT >= 0 ? c & ((1 << SHIFT) - 1) : c % cpt) * 8; };
  // every load goes out before anything waits: chunks past the tile re-read its last chunk and are zeroed after
  u32x4 raw[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = min(lane + 64 * i, total - 1);
    raw[i] = stream_load(reinterpret_cast<const u32x4*>(src + int64_t(token_of(c)) * src_s_tok + column_of(c)));
  }
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    if (lane + 64 * i >= total) raw[i] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      amax = fmaxf(amax, fabsf(bf16_bits_to_f32(raw[i][j] & 0xffffu)));
      amax = fmaxf(amax, fabsf(bf16_bits_to_f32(raw[i][j] >> 16)));
    }
  }
  amax = wave_max(amax);
  const float scale = amax > 0.f ? amax / 448.f : 1.f;
  if (lane == 0) p.scales[(int64_t(id) * p.num_kv_heads + h) * 2 + which] = scale;
  // x / scale without a division per element.  q0 = x * RN(1 / scale) is within 2 ulp of the exact quotient and
  // the correctly rounded quotient within 0.5 ulp, so both lie on the same side of every rounding boundary of
  // e4m3 -- and get the same code -- unless q0 is within a few ulp of one.  Boundaries (midpoints of neighbouring
  // e4m3 values) have the float32 pattern "3 mantissa bits, then 1000...0" in the normal range; a chunk in which
  // any lane is that close to one, or may fall into the subnormal range of e4m3 (an absolute grid), is redone with
  // the real division.  The stored codes are therefore exactly those of RN(x / scale) everywhere.
  const float rinv = 1.f / scale;
  const float subnormal_below = scale * 0x1.000002p-6f;   // |x| under this: the quotient may be under 2^-6
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = lane + 64 * i;
    float x[8], q[8];
    bool risky = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[2 * j] = bf16_bits_to_f32(raw[i][j] & 0xffffu);
      x[2 * j + 1] = bf16_bits_to_f32(raw[i][j] >> 16);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      q[j] = x[j] * rinv;
      // low 20 mantissa bits within [0x7fffc, 0x80004]: shifted to the top of the word, offset so the window starts at 0
      risky |= (__float_as_uint(q[j]) << 12) + 0x80004000u <= 0x8000u;
      risky |= fabsf(x[j]) < subnormal_below;               // subnormal range of e4m3 (also catches exact zeros)
    }
    risky = risky && c < total;                               // lanes past the tile hold zeros: no say
    if (__builtin_amdgcn_ballot_w64(risky) != 0) {
      // second look: a quotient near a boundary that is exact (zero residual x - q0 * scale; ties of short
      // mantissas are common with bf16 inputs) is the correctly rounded quotient already
      bool divide = false;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool near = (__float_as_uint(q[j]) << 12) + 0x80004000u <= 0x8000u;
        divide |= near && __builtin_fmaf(-q[j], scale, x[j]) != 0.f;
        divide |= fabsf(x[j]) < subnormal_below;
      }
      divide = divide && c < total;
      if (__builtin_amdgcn_ballot_w64(divide) != 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = x[j] / scale;
      }
    }
    if (c < total) {
      u32x2 out;
      out[0] = uint32_t(__builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], 0, false), true));
      out[1] = uint32_t(__builtin_amdgcn_cvt_pk_fp8_f32(q[6], q[7], __builtin_amdgcn_cvt_pk_fp8_f32(q[4], q[5], 0, false), true));
      stream_store(reinterpret_cast<u32x2*>(dst + int64_t(token_of(c)) * p.s_tok + column_of(c)), out);
    }
  }
}

// ---- append: one wavefront per (request, kv head, K|V) ----------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void append_copy_kernel(KvWriteParams p, const T* __restrict__ new_k,
                                                          const T* __restrict__ new_v, int num_requests) {
  const int lane = threadIdx.x & 63;
  const int64_t row = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= int64_t(num_requests) * p.num_kv_heads * 2) return;
  const int which = int(row & 1);
  const int h = int((row >> 1) % p.num_kv_heads);
  const int r = int((row >> 1) / p.num_kv_heads);
  const int dest = p.dest[r];
  if (dest < 0) return;
  const int id = dest / p.block_size, slot = dest % p.block_size;
  const T* src = (which ? new_v : new_k) + (int64_t(r) * p.num_kv_heads + h) * p.head_dim;
  T* dst = static_cast<T*>(p.kv) + int64_t(id) * p.s_block + int64_t(h) * p.s_head + int64_t(which) * p.s_kv +
           int64_t(slot) * p.s_tok;
  for (int c = lane; c < p.head_dim; c += 64) dst[c] = src[c];
}

__global__ __launch_bounds__(256) void append_e4m3_kernel(KvWriteParams p, const uint16_t* __restrict__ new_k,
                                                          const uint16_t* __restrict__ new_v, int num_requests) {
  const int lane = threadIdx.x & 63;
  const int64_t row = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= int64_t(num_requests) * p.num_kv_heads * 2) return;
  const int which = int(row & 1);
  const int h = int((row >> 1) % p.num_kv_heads);
  const int r = int((row >> 1) / p.num_kv_heads);
  const int dest = p.dest[r];
  if (dest < 0) return;
  const int id = dest / p.block_size, slot = dest % p.block_size;
  const uint16_t* src = (which ? new_v : new_k) + (int64_t(r) * p.num_kv_heads + h) * p.head_dim;
  uint8_t* tile = static_cast<uint8_t*>(p.kv) + int64_t(id) * p.s_block + int64_t(h) * p.s_head + int64_t(which) * p.s_kv;
  float* scale_ptr = p.scales + (int64_t(id) * p.num_kv_heads + h) * 2 + which;
  float amax = 0.f;
  for (int c = lane; c < p.head_dim; c += 64) amax = fmaxf(amax, fabsf(bf16_bits_to_f32(src[c])));
  amax = wave_max(amax);
  const float cand = amax / 448.f;
  float scale;
  if (slot == 0) {
    scale = amax > 0.f ? cand : 1.f;
  } else {
    const float old = *scale_ptr;
    scale = fmaxf(old, cand);
    if (scale != old) {   // the tile's scale grew: re-encode what is stored, from the stored values
      for (int c = lane; c < slot * p.head_dim; c += 64) {
        uint8_t* at = tile + int64_t(c / p.head_dim) * p.s_tok + c % p.head_dim;
        *at = uint8_t(f32x2_to_e4m3((e4m3_to_f32(*at) * old) / scale, 0.f) & 0xffu);
      }
    }
  }
  if (lane == 0) *scale_ptr = scale;
  uint8_t* dst = tile + int64_t(slot) * p.s_tok;
  for (int c = lane; c < p.head_dim; c += 64) dst[c] = uint8_t(f32x2_to_e4m3(bf16_bits_to_f32(src[c]) / scale, 0.f) & 0xffu);
}

// ---- staging of whole blocks (cold KV parked in host memory and reloaded, Appendix B.2) -------------------
// One wavefront per TILES consecutive (entry, KV head, K|V) tiles of B x d elements; the image is dense,
// [entry][head][K|V][slot][d] in table order, followed by the e4m3 scales [entry][head][K|V].  TO_IMAGE: pool ->
// image, else image -> pool.  Bits are copied, 16 bytes per lane and step, four loads per tile in flight before the
// first store.
template <bool TO_IMAGE, int TILES>
__global__ __launch_bounds__(256) void stage_copy_kernel(KvWriteParams p, uint8_t* __restrict__ image,
                                                         float* __restrict__ image_scales, int num_entries,
                                                         int elem_bytes) {
  const int lane = threadIdx.x & 63;
  const int64_t num_tiles = int64_t(num_entries) * p.num_kv_heads * 2;
  const int64_t tile0 = (int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6)) * TILES;   // (entry, head, which), TILES in a row
  if (tile0 >= num_tiles) return;
  const int row_bytes = p.head_dim * elem_bytes;
  const int row_chunks = row_bytes >> 4;
  const int chunks = p.block_size * row_chunks;
  const int64_t tok_bytes = p.s_tok * elem_bytes;
  uint8_t* pool_tile[TILES];
  uint8_t* image_tile[TILES];
  int live[TILES];
#pragma unroll
  for (int i = 0; i < TILES; ++i) {
    const int64_t tile = min(tile0 + i, num_tiles - 1);
    live[i] = tile0 + i < num_tiles;
    const int which = int(tile & 1);
    const int h = int((tile >> 1) % p.num_kv_heads);
    // Into the pool the shared blocks are walked in the order of their addresses there, so that the scattered side of
    // the copy is the read of the image (scattered writes cost more); out of it in table order, for the same reason.
    const int pos = int((tile >> 1) / p.num_kv_heads);
    const int e = TO_IMAGE ? pos : p.ent_order[pos];
    const int64_t image_tile_index = (int64_t(e) * p.num_kv_heads + h) * 2 + which;
    const int id = p.blk[e];
    pool_tile[i] = static_cast<uint8_t*>(p.kv) +
                   (int64_t(id) * p.s_block + int64_t(h) * p.s_head + int64_t(which) * p.s_kv) * elem_bytes;
    image_tile[i] = image + image_tile_index * int64_t(p.block_size) * row_bytes;
    if (image_scales && lane == 0 && live[i]) {
      float* pool_scale = p.scales + (int64_t(id) * p.num_kv_heads + h) * 2 + which;
      if (TO_IMAGE) image_scales[image_tile_index] = *pool_scale;
      else *pool_scale = image_scales[image_tile_index];
    }
  }
  // every load of a step (four 16-byte pieces per lane and tile) goes out before the first store
  for (int c0 = 0; c0 < chunks; c0 += 256) {
    u32x4 v[TILES][4];
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + 64 * u + lane;
        if (c < chunks && live[i]) {
          const int slot = c / row_chunks, col = c % row_chunks;
          const uint8_t* src = TO_IMAGE ? pool_tile[i] + slot * tok_bytes + 16 * col : image_tile[i] + 16 * int64_t(c);
          v[i][u] = stream_load(reinterpret_cast<const u32x4*>(src));
        }
      }
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + 64 * u + lane;
        if (c < chunks && live[i]) {
          const int slot = c / row_chunks, col = c % row_chunks;
          uint8_t* dst = TO_IMAGE ? image_tile[i] + 16 * int64_t(c) : pool_tile[i] + slot * tok_bytes + 16 * col;
          stream_store(reinterpret_cast<u32x4*>(dst), v[i][u]);
        }
      }
  }
}

KvWriteParams make_write_params(const ps_layout* lay, const void* dev_tables, void* kv, float* scales) {
  const int32_t* t = static_cast<const int32_t*>(dev_tables);
  const ps_geometry& g = lay->geo;
  KvWriteParams p{};
  p.blk = t + lay->off_blk;
  p.ent_tok0 = t + lay->off_ent_tok0;
  p.ent_valid = t + lay->off_ent_valid;
  p.ent_order = t + lay->off_ent_order;
  p.dest = t + lay->off_dest;
  p.kv = kv;
  p.scales = scales;
  p.num_kv_heads = g.num_kv_heads;
  p.head_dim = g.head_dim;
  p.block_size = g.block_size;
  p.s_block = g.kv_stride_block;
  p.s_head = g.kv_stride_head;
  p.s_kv = g.kv_stride_kv;
  p.s_tok = g.kv_stride_tok;
  return p;
}

}  // namespace

int32_t launch_kv_ingest(const ps_layout* lay, const void* dev_tables, int which, const void* src_k, const void* src_v,
                         int64_t src_s_tok, int64_t src_s_head, void* kv, float* scales, hipStream_t st) {
  const ps_geometry& g = lay->geo;
  const int n_prefix = int(lay->prefix_blk.size());
  const int n_suffix = int(lay->suffix_blk.size());
  // entries follow the concatenated block array: prefixes, suffixes, roots
  const int entry0 = which == 0 ? 0 : (which == 1 ? n_prefix : n_prefix + n_suffix);
  const int num_entries = which == 0 ? n_prefix : (which == 1 ? n_suffix : int(lay->root_blk.size()));
  if (num_entries == 0) return PS_OK;
  const int64_t tiles = int64_t(num_entries) * g.num_kv_heads * 2;
  const int64_t grid64 = (tiles + 3) / 4;
  if (tiles > INT32_MAX) return PS_ERR_INVALID_ARG;
  const dim3 grid{unsigned(grid64)}, block{256};
  const KvWriteParams p = make_write_params(lay, dev_tables, kv, scales);
  if (g.kv_dtype == PS_F32) {
    if (g.head_dim % 4) return PS_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((ingest_copy_kernel<float, 1>), grid, block, 0, st, p, static_cast<const float*>(src_k),
                       static_cast<const float*>(src_v), src_s_tok, src_s_head, entry0, num_entries);
  } else if (g.kv_dtype == PS_BF16) {
    if (g.head_dim % 8) return PS_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((ingest_copy_kernel<uint16_t, 1>), grid, block, 0, st, p, static_cast<const uint16_t*>(src_k),
                       static_cast<const uint16_t*>(src_v), src_s_tok, src_s_head, entry0, num_entries);
  } else {
    if (g.head_dim % 8) return PS_ERR_UNSUPPORTED;
    const int64_t chunks = (int64_t(g.block_size) * (g.head_dim / 8) + 63) / 64;   // per lane, whole tile in registers
#define PS_INGEST(CH, SHIFT)                                                                                     \
  hipLaunchKernelGGL((ingest_e4m3_kernel<CH, SHIFT>), grid, block, 0, st, p, static_cast<const uint16_t*>(src_k), \
                     static_cast<const uint16_t*>(src_v), src_s_tok, src_s_head, entry0, num_entries)
    if (g.head_dim == 128) {   // 16 chunks per token
      if (chunks <= 4) PS_INGEST(4, 4);
      else if (chunks <= 8) PS_INGEST(8, 4);
      else if (chunks <= 16) PS_INGEST(16, 4);
      else if (chunks <= 32) PS_INGEST(32, 4);
      else return PS_ERR_UNSUPPORTED;
    } else {
      if (chunks <= 4) PS_INGEST(4, -1);
      else if (chunks <= 8) PS_INGEST(8, -1);
      else if (chunks <= 16) PS_INGEST(16, -1);
      else if (chunks <= 32) PS_INGEST(32, -1);
      else return PS_ERR_UNSUPPORTED;
    }
#undef PS_INGEST
  }
  return PS_OK;
}

int32_t launch_kv_append(const ps_layout* lay, const void* dev_tables, const void* new_k, const void* new_v, void* kv,
                         float* scales, hipStream_t st) {
  const ps_geometry& g = lay->geo;
  if (lay->num_requests == 0) return PS_OK;
  const int64_t rows = int64_t(lay->num_requests) * g.num_kv_heads * 2;
  const dim3 grid{unsigned((rows + 3) / 4)}, block{256};
  const KvWriteParams p = make_write_params(lay, dev_tables, kv, scales);
  if (g.kv_dtype == PS_F32)
    hipLaunchKernelGGL(append_copy_kernel<float>, grid, block, 0, st, p, static_cast<const float*>(new_k),
                       static_cast<const float*>(new_v), lay->num_requests);
  else if (g.kv_dtype == PS_BF16)
    hipLaunchKernelGGL(append_copy_kernel<uint16_t>, grid, block, 0, st, p, static_cast<const uint16_t*>(new_k),
                       static_cast<const uint16_t*>(new_v), lay->num_requests);
  else
    hipLaunchKernelGGL(append_e4m3_kernel, grid, block, 0, st, p, static_cast<const uint16_t*>(new_k),
                       static_cast<const uint16_t*>(new_v), lay->num_requests);
  return PS_OK;
}

int32_t launch_kv_stage(const ps_layout* lay, const void* dev_tables, bool to_image, void* kv, float* scales,
                        void* image, int64_t scales_offset_bytes, hipStream_t st) {
  const ps_geometry& g = lay->geo;
  const int64_t entries = int64_t(lay->prefix_blk.size() + lay->suffix_blk.size() + lay->root_blk.size());
  if (entries == 0) return PS_OK;
  const int esz = g.kv_dtype == PS_F32 ? 4 : (g.kv_dtype == PS_BF16 ? 2 : 1);
  if ((g.head_dim * esz) % 16) return PS_ERR_UNSUPPORTED;
  const int64_t tiles = entries * g.num_kv_heads * 2;
  if (tiles > INT32_MAX) return PS_ERR_INVALID_ARG;
  const KvWriteParams p = make_write_params(lay, dev_tables, kv, scales);
  uint8_t* img = static_cast<uint8_t*>(image);
  float* img_scales = g.kv_dtype == PS_FP8_E4M3 ? reinterpret_cast<float*>(img + scales_offset_bytes) : nullptr;
  // Tiles per wave: four consecutive tiles are K and V of two neighbouring heads, 16 KiB in a row on the pool side
  // for bf16 -- measured on scattered blocks, stage_in (dense reads, scattered writes) gains 9 % from the longer
  // runs (5.16 -> 5.65 TB/s), stage_out is unchanged; with the 2 KiB tiles of e4m3 more tiles per wave only lose.
  const int per_wave = esz >= 2 ? 4 : 1;
#define PS_STAGE(TO, N)                                                                                             \
  hipLaunchKernelGGL((stage_copy_kernel<TO, N>), dim3{unsigned((tiles + 4 * N - 1) / (4 * N))}, dim3{256}, 0, st, p, img, \
                     img_scales, int(entries), esz)
  if (to_image) {
    if (per_wave == 4) PS_STAGE(true, 4); else PS_STAGE(true, 1);
  } else {
    if (per_wave == 4) PS_STAGE(false, 4); else PS_STAGE(false, 1);
  }
#undef PS_STAGE
  return PS_OK;
}

}  // namespace psdev
