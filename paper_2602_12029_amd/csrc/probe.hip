// Read-bandwidth probe: what the footprint of one load instruction costs on this chip.
//
// A measurement aid, not part of the attention path: it reads a buffer once, in the launch shape of the attention
// kernel (4-wave workgroups, 8 KiB in flight per wave, non-temporal loads), and throws the data away.  The patterns
// are the footprints the attention kernel's tile loads have or used to have, so that the ceiling each one allows can
// be measured next to the kernel itself.
#include "device_common.h"
#include "launch.h"
#include "mfma_common.h"

namespace psdev {

namespace {

// One unit = 8 KiB, taken by one wave in one turn.
//   0: 8 x 16-byte loads, each instruction 1 KiB contiguous (8 whole 128-byte lines)
//   1: 8 x 16-byte loads over 64 rows of 128 B: an instruction takes 16 rows x 64 B (half a line per row, every line
//      asked for twice) -- lane (n, kg): row 16 r + n, byte 64 s + 16 kg
//   2: the same over 32 rows of 256 B (an instruction takes 16 rows x 64 B, four instructions per 16 rows)
//   3: 16 x 8-byte loads, each instruction 512 B contiguous
//   4, 5, 6: the loads of pattern 0, but the buffer is taken in chunks of 2, 4 or 8 KiB in a scrambled order (chunk
//      index times an odd constant, modulo the power-of-two chunk count): what block-granular scatter of the KV pool
//      costs by itself, at the chunk sizes a (block, head) record of K or V has
template <int PATTERN>
__global__ __launch_bounds__(256) void probe_read_kernel(const char* __restrict__ buf, int64_t n_units) {
  const int lane = threadIdx.x & 63, n = lane & 15, kg = lane >> 4;
  const int64_t wave = (int64_t(blockIdx.x) * 256 + threadIdx.x) >> 6, n_waves = (int64_t(gridDim.x) * 256) >> 6;
  u32x4 acc = {0, 0, 0, 0};
  for (int64_t u = wave; u < n_units; u += n_waves) {
    const char* base = buf + u * 8192;
    if constexpr (PATTERN >= 4) {
      constexpr int kChunk = 2048 << (PATTERN - 4), kPerUnit = 8192 / kChunk;
      const int64_t mask = n_units * kPerUnit - 1;   // the launcher checks that the chunk count is a power of two
      u32x4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int64_t chunk = ((u * kPerUnit + i * 1024 / kChunk) * 0x9E3779B1ll) & mask;
        v[i] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(buf + chunk * kChunk + (i * 1024) % kChunk + lane * 16));
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) acc ^= v[i];
    } else if constexpr (PATTERN == 3) {
      u32x2 v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i)
        v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(base + i * 512 + lane * 8));
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc.x ^= v[i].x;
        acc.y ^= v[i].y;
      }
    } else {
      u32x4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int off;
        if (PATTERN == 0) off = i * 1024 + lane * 16;
        else if (PATTERN == 1) off = ((i >> 1) * 16 + n) * 128 + (i & 1) * 64 + kg * 16;
        else off = ((i >> 2) * 16 + n) * 256 + (i & 3) * 64 + kg * 16;
        v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) acc ^= v[i];
    }
  }
  // the data goes nowhere; the empty statement keeps the loads from being dropped
  asm volatile("" ::"v"(acc.x), "v"(acc.y), "v"(acc.z), "v"(acc.w));
}

}  // namespace

int32_t launch_probe_read(const void* buf, int64_t bytes, int pattern, int num_workgroups, hipStream_t st) {
  const int64_t n_units = bytes / 8192;
  if (n_units <= 0) return PS_OK;
  const dim3 grid(num_workgroups), block(256);
  const char* b = static_cast<const char*>(buf);
  switch (pattern) {
    case 0: hipLaunchKernelGGL(probe_read_kernel<0>, grid, block, 0, st, b, n_units); break;
    case 1: hipLaunchKernelGGL(probe_read_kernel<1>, grid, block, 0, st, b, n_units); break;
    case 2: hipLaunchKernelGGL(probe_read_kernel<2>, grid, block, 0, st, b, n_units); break;
    case 3: hipLaunchKernelGGL(probe_read_kernel<3>, grid, block, 0, st, b, n_units); break;
    case 4: case 5: case 6:
      if (n_units & (n_units - 1)) return PS_ERR_INVALID_ARG;
      if (pattern == 4) hipLaunchKernelGGL(probe_read_kernel<4>, grid, block, 0, st, b, n_units);
      else if (pattern == 5) hipLaunchKernelGGL(probe_read_kernel<5>, grid, block, 0, st, b, n_units);
      else hipLaunchKernelGGL(probe_read_kernel<6>, grid, block, 0, st, b, n_units);
      break;
    default: return PS_ERR_INVALID_ARG;
  }
  return PS_OK;
}

}  // namespace psdev
