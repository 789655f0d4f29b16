/*
 * prefillshare_probe.h -- measurement aid of the shared-prefix decode attention library; no part of the method's ABI
 * (prefillshare.h does not include this file, and nothing in the attention path calls it).
 */
#ifndef PREFILLSHARE_PROBE_H
#define PREFILLSHARE_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ps_probe_read (device, asynchronous on `stream`): no part of the method.  Reads the first
 * floor(bytes / 8192) * 8192 bytes of dev_buf (device memory, 16-byte aligned, caller-owned, not written) once and
 * discards them, with `num_workgroups` workgroups of four wavefronts, 8 KiB in flight per wavefront and
 * non-temporal loads -- the launch shape of the attention kernel -- and the per-instruction footprint `pattern`
 * names: 0 = 16 bytes per lane, 1 KiB contiguous per instruction; 1 = 16 rows x 64 bytes of 128-byte rows (half a
 * cache line per row and instruction); 2 = 16 rows x 64 bytes of 256-byte rows; 3 = 8 bytes per lane, 512 bytes
 * contiguous per instruction; 4, 5, 6 = the loads of pattern 0 with the buffer taken in chunks of 2, 4, 8 KiB in a
 * scrambled order (the number of such chunks in the bytes read must be a power of two): the cost of block-granular
 * scatter alone.  Timed by the caller (`bench.py --path probe`), it gives the read ceiling each
 * footprint allows, next to which the attention kernel's own rate is to be read.
 * PS_ERR_INVALID_ARG: null or misaligned buffer, negative size, pattern outside 0..6 (or 4..6 with a chunk count that is no power of two), num_workgroups outside
 * 1..65536. */
int32_t ps_probe_read(const void* dev_buf, int64_t bytes, int32_t pattern, int32_t num_workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PREFILLSHARE_PROBE_H */
