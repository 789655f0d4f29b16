#!/usr/bin/env python3
"""Benchmark: one decode-attention step over shared prefix KV + private suffix KV on one MI355X.

A step is one ps_decode_attention call (prefix pass, suffix pass, merge) over one synthetic batch
with all inputs resident in HBM.  Steps rotate over several copies of the KV pool so that no step
finds its KV in the last-level cache.  The default workload is `mixed`, the largest of the benchmark
configurations.  Prints one JSON line:
  value     ideal-byte GB/s of the whole step (shared KV counted once + private KV + Q + O), wall clock over
            exactly --steps steps; ms_per_step_median / value_at_median come from an event-bracketed loop after it
  roofline  the attention launch alone, timed with HIP events on its stream (at least 20 brackets)
  cpu_baseline  the fp64 numpy oracle on a bounded sample of the same workload, on this host
  per_config    the same step on b8, long, mixed and fp8_70b (short runs, no oracle leg)
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mixed",
                    help="tiny | b8 | long | mixed | fp8_70b; tree_tiny | tree_b8 (a context common to all sessions, stored "
                         "once as a third sharing level); sessions<S> (S concurrent four-agent sessions, e.g. sessions80: "
                         "the shape of a sweep over the cap on concurrent sessions)")
    ap.add_argument("--stage-image", default="device", choices=["device", "host"],
                    help="--path stage: where the staging image lives (device memory: the kernels' own rate; pinned "
                         "host memory: the rate across PCIe)")
    ap.add_argument("--path", default="decode", choices=["decode", "ingest", "prefill", "stage", "loop", "probe"],
                    help="decode: the attention step (the headline metric); ingest: hand-off of the batch's KV into "
                         "the paged pool (ps_kv_ingest over every prefix and suffix), a step = one whole hand-off; "
                         "prefill: attention of newly appended context tokens against the cached context "
                         "(workloads prefill_b8 | prefill_fp8 | prefill_tiny); stage: a step copies every KV block of "
                         "the batch to a staging image and back (ps_kv_stage_out + ps_kv_stage_in); loop: a multi-step decode "
                         "loop, a step = one token appended to every private segment (ps_layout_append, upload, "
                         "ps_kv_append) + the attention step; probe: no part of the method -- a read-only kernel in "
                         "the attention kernel's launch shape over 2 GiB, one rate per load-instruction footprint "
                         "(ps_probe_read), the ceilings the attention kernel's rate is read against")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--models", type=int, default=0, help="override the number of decode models M (b8, long, fp8_70b)")
    ap.add_argument("--copies", type=int, default=3, help="distinct KV pool copies rotated between steps")
    ap.add_argument("--prefix-chunk", type=int, default=0)
    ap.add_argument("--suffix-chunk", type=int, default=0)
    ap.add_argument("--prefix-variant", default="auto")
    ap.add_argument("--suffix-variant", default="auto")
    ap.add_argument("--kv-policy", default="auto", choices=["auto", "stream", "cacheable"],
                    help="K/V loads of the matrix-core decode kernel: non-temporal, ordinary, or chosen per launch")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target wall time of the oracle sample; 0 = skip")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events in the timed loop")
    ap.add_argument("--event-steps", type=int, default=100,
                    help="decode path: steps of the event-bracketed loop that follows the timed region (attention "
                         "launches and whole step one by one: mean, median; at least 20)")
    ap.add_argument("--no-per-config", dest="per_config", action="store_false",
                    help="decode path: only the headline workload, not the per_config map over b8 / long / mixed / fp8_70b")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket the attention kernel with HIP events on every n-th timed step (each bracket costs "
                         "a few microseconds of stream time)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB read + 1 GiB write elementwise kernel (reference for HBM byte counters)")
    return ap.parse_args()


class HipEvents:
    """hipEvent pairs on a raw stream (torch.cuda.Event only sees torch's current stream object)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.events = []
        for _ in range(n):
            pair = (ctypes.c_void_p(), ctypes.c_void_p())
            for e in pair:
                assert self.hip.hipEventCreate(ctypes.byref(e)) == 0
            self.events.append(pair)

    def record(self, i, which, stream):
        assert self.hip.hipEventRecord(self.events[i][which], ctypes.c_void_p(stream)) == 0

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(ms), self.events[i][0], self.events[i][1]) == 0
        return ms.value


def cpu_baseline(w, lay_tables, data, seconds):
    """The oracle on the host: with the threads its BLAS takes by itself, and (a shorter sample) on one thread."""
    line = _cpu_baseline_leg(w, data, seconds)
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            one = _cpu_baseline_leg(w, data, seconds / 3)
        line["single_thread"] = {"value": one["value"], "unit": "GB/s", "queries_per_s": one["queries_per_s"],
                                 "sample": one["sample"]}
    except ImportError:
        pass
    return line


def _cpu_baseline_leg(w, data, seconds):
    """Time the oracle on whole prompts (all their requests) until about `seconds` have passed."""
    from oracle import attention as oa
    from oracle import layout as ol
    import workloads as wl
    g = w.geometry
    opool = ol.BlockPool(w.num_blocks, w.free_order)
    if w.num_roots:
        olay = ol.build_layout_tree(opool, g.block_size, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt,
                                    w.req_model, w.suffix_len)
    else:
        olay = ol.build_layout(opool, g.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    q_bits = w.q_bits()
    done_req, done_bytes = 0, 0
    wall0, cpu0 = time.perf_counter(), time.process_time()
    prompts = 0
    for p in list(range(w.num_prompts)) * 64:        # whole prompts, cycling, until the time target
        reqs = olay.group_req[olay.group_indptr[p]:olay.group_indptr[p + 1]].tolist()
        oa.decode_attention(q_bits, g.q_dtype, data.kv, data.scales, g.kv_dtype, olay, reqs)
        done_req += len(reqs)
        nblk = -(-int(w.prefix_len[p]) // g.block_size) + sum(-(-int(w.suffix_len[r]) // g.block_size) for r in reqs)
        done_bytes += (int(w.prefix_len[p]) + int(w.suffix_len[reqs].sum())) * g.token_bytes
        if w.num_roots and w.prompt_root[p] >= 0 and prompts < w.num_prompts:      # a root counts once per pass
            done_bytes += int(w.root_len[w.prompt_root[p]]) * g.token_bytes // max(1, int((w.prompt_root == w.prompt_root[p]).sum()))
        done_bytes += 2 * len(reqs) * g.num_q_heads * g.head_dim * wl.generate.ELEM_BYTES[g.q_dtype]
        if g.kv_dtype == "fp8_e4m3":
            done_bytes += nblk * g.num_kv_heads * 8
        prompts += 1
        if time.perf_counter() - wall0 >= seconds:
            break
    wall = time.perf_counter() - wall0
    cpu = time.process_time() - cpu0
    return {"value": done_bytes / wall / 1e9, "unit": "GB/s", "cores": max(1, int(round(cpu / wall))),
            "kind": "oracle", "queries_per_s": done_req / wall,
            "sample": f"fp64 numpy oracle over {prompts} prompt groups ({done_req} requests, all q heads; the "
                      f"workload has {w.num_prompts} prompts / {w.num_requests} requests, cycled), {wall:.1f} s wall"}


def calibrate_copy(dev):
    """A plain elementwise kernel of known traffic (reads 2^30 bytes, writes 2^30 bytes per launch): the
    reference the HBM byte counters of a profiler run are scaled by."""
    import torch
    src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1, out=dst)
    torch.cuda.synchronize()
    del src, dst


def cpu_ingest_baseline(w, olay, sources, seconds):
    """Time the oracle's ingest on whole prompts until about `seconds` have passed."""
    from oracle import kv_update as ku
    import workloads as wl
    g = w.geometry
    shape = (w.num_blocks, g.num_kv_heads, 2, g.block_size, g.head_dim)
    kv = np.zeros(shape, wl.generate.STORAGE[g.kv_dtype])
    scales = np.ones((w.num_blocks, g.num_kv_heads, 2), np.float32) if g.kv_dtype == "fp8_e4m3" else None
    esz_src = 4 if g.kv_dtype == "f32" else 2
    esz_dst = wl.generate.ELEM_BYTES[g.kv_dtype]
    done, prompts = 0, 0
    wall0, cpu0 = time.perf_counter(), time.process_time()
    for p in list(range(w.num_prompts)) * 64:
        ids = olay.prefix_blk[olay.prefix_blk_indptr[p]:olay.prefix_blk_indptr[p + 1]]
        ku.ingest_segment(kv, scales, g.kv_dtype, ids, sources[p][0], sources[p][1])
        done += int(w.prefix_len[p]) * g.num_kv_heads * g.head_dim * 2 * (esz_src + esz_dst)
        prompts += 1
        if time.perf_counter() - wall0 >= seconds:
            break
    wall = time.perf_counter() - wall0
    cpu = time.process_time() - cpu0
    return {"value": done / wall / 1e9, "unit": "GB/s", "cores": max(1, int(round(cpu / wall))), "kind": "oracle",
            "sample": f"numpy oracle ingest of {prompts} prompt prefixes (the workload has {w.num_prompts}, cycled), "
                      f"{wall:.1f} s wall"}


def main_ingest(args):
    """--path ingest: one step stores every prefix and every suffix of the batch from contiguous sources."""
    import torch
    import workloads as wl
    from oracle import layout as ol
    from paper_2602_12029_amd import binding as B
    from paper_2602_12029_amd.runtime import DecodeBatch, to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    w = wl.named_workload(args.workload, args.seed, args.models or None)
    g = w.geometry
    geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    pool = B.ps_pool_create(w.num_blocks, w.free_order)
    layout = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    src_dtype = "f32" if g.kv_dtype == "f32" else "bf16"
    pre = [w.prefix_source(p) for p in range(w.num_prompts)]
    suf = [w.suffix_source(r) for r in range(w.num_requests)]

    def ragged(parts, which):
        parts = [x[which] for x in parts if x[which].shape[0]]
        return to_device(np.concatenate(parts, axis=0), src_dtype, dev) if parts else None

    # two copies of the sources, alternated, so that a step does not find its input in the last-level cache
    srcs = [[(ragged(pre, 0), ragged(pre, 1)), (ragged(suf, 0), ragged(suf, 1))]]
    srcs.append([tuple(None if t is None else t.clone() for t in pair) for pair in srcs[0]])
    nelem = w.num_blocks * g.num_kv_heads * 2 * g.block_size * g.head_dim
    torch_dtype = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.uint8}[g.kv_dtype]
    kv = torch.zeros(nelem, dtype=torch_dtype, device=dev)
    scales = torch.ones((w.num_blocks, g.num_kv_heads, 2), dtype=torch.float32, device=dev) if g.kv_dtype == "fp8_e4m3" else None
    q = to_device(w.q_bits(), g.q_dtype, dev)
    batch = DecodeBatch(layout, geo, w.num_requests, q, kv, scales)
    stream = int(torch.cuda.current_stream().cuda_stream)

    def step(i, ev=None, slot=0):
        (pk, pv), (sk, sv) = srcs[i % 2]
        if ev is not None:
            ev.record(slot, 0, stream)
        if pk is not None:
            batch.kv_ingest(0, pk, pv)
        if ev is not None:
            ev.record(slot, 1, stream)
        if sk is not None:
            batch.kv_ingest(1, sk, sv)

    if args.calibrate_copy:
        calibrate_copy(dev)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev = None if args.no_events else HipEvents(args.steps)
    every = max(1, args.event_every)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, ev if (ev is not None and i % every == 0) else None, i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    esz_src = 4 if g.kv_dtype == "f32" else 2
    esz_dst = wl.generate.ELEM_BYTES[g.kv_dtype]
    per_tok = g.num_kv_heads * g.head_dim * 2 * (esz_src + esz_dst)
    t_pre, t_suf = int(w.prefix_len.astype(np.int64).sum()), int(w.suffix_len.astype(np.int64).sum())
    scale_bytes = w.blocks_needed() * g.num_kv_heads * 8 if g.kv_dtype == "fp8_e4m3" else 0
    moved = (t_pre + t_suf) * per_tok + scale_bytes
    pre_blocks = int(((w.prefix_len.astype(np.int64) + g.block_size - 1) // g.block_size).sum())
    pre_bytes = t_pre * per_tok + (pre_blocks * g.num_kv_heads * 8 if g.kv_dtype == "fp8_e4m3" else 0)
    roofline = {"bound": "hbm", "kernel": "ingest (shared prefixes)", "achieved": None, "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": None, "traffic": None}
    if ev is not None:
        k_ms = float(np.mean([ev.elapsed_ms(i) for i in range(0, args.steps, every)]))
        roofline.update(achieved=pre_bytes / (k_ms * 1e-3) / 1e9, kernel_ms=k_ms, algorithmic_bytes=pre_bytes)
        roofline["frac"] = roofline["achieved"] / PEAK_HBM_GBS
    summary = os.path.join(ROOT, "profiles", f"ingest_kernel_{args.workload}.md")
    if os.path.exists(summary):
        for text in open(summary):
            if text.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(text.split(":")[1])
                roofline["traffic_source"] = os.path.relpath(summary, ROOT) + " (rocprofv3 --pmc runs of this command, not this run)"
    value = moved / (ms_per_step * 1e-3) / 1e9
    line = {
        "metric": "KV hand-off ingest into the paged pool: bytes read + written, GB/s",
        "value": value, "unit": "GB/s", "pct_of_peak_hbm": 100.0 * value / PEAK_HBM_GBS,
        "tokens_per_s": (t_pre + t_suf) / (ms_per_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp8_e4m3": "bf16 -> fp8_e4m3", "f32": "f32"}[g.kv_dtype], "data": "synthetic",
        "config": {"workload": args.workload, "path": "ingest", "prompts": w.num_prompts, "requests": w.num_requests,
                   "prefix_tokens": t_pre, "suffix_tokens": t_suf, "kv_heads": g.num_kv_heads, "head_dim": g.head_dim,
                   "block_size": g.block_size, "moved_bytes": moved},
        "roofline": roofline,
    }
    if args.cpu_seconds > 0:
        opool = ol.BlockPool(w.num_blocks, w.free_order)
        olay = ol.build_layout(opool, g.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        line["cpu_baseline"] = cpu_ingest_baseline(w, olay, pre, args.cpu_seconds)
    return line


PEAK_MFMA_BF16_TFLOPS = 2500.0


def main_stage(args):
    """--path stage: one step = ps_kv_stage_out of the whole batch followed by ps_kv_stage_in."""
    import torch
    import workloads as wl
    from oracle import layout as ol
    from oracle import staging as ost
    from paper_2602_12029_amd import binding as B
    from paper_2602_12029_amd.runtime import DecodeBatch, to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    w = wl.named_workload(args.workload, args.seed, args.models or None)
    g = w.geometry
    geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    pool = B.ps_pool_create(w.num_blocks, w.free_order)
    layout = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    nelem = w.num_blocks * g.num_kv_heads * 2 * g.block_size * g.head_dim
    torch_dtype = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.uint8}[g.kv_dtype]
    kv = torch.zeros(nelem, dtype=torch_dtype, device=dev)
    scales = torch.ones((w.num_blocks, g.num_kv_heads, 2), dtype=torch.float32, device=dev) if g.kv_dtype == "fp8_e4m3" else None
    q = to_device(w.q_bits(), g.q_dtype, dev)
    batch = DecodeBatch(layout, geo, w.num_requests, q, kv, scales)
    block_bytes, _, total = B.ps_stage_layout(layout)
    host = args.stage_image == "host"
    images = [torch.zeros(total, dtype=torch.uint8, pin_memory=True) if host else torch.zeros(total, dtype=torch.uint8, device=dev)
              for _ in range(2)]
    stream = int(torch.cuda.current_stream().cuda_stream)

    def step(i, ev=None, slot=0):
        if ev is not None:
            ev.record(slot, 0, stream)
        batch.stage_out(images[i % 2])
        if ev is not None:
            ev.record(slot, 1, stream)
        batch.stage_in(images[(i + 1) % 2])

    if args.calibrate_copy:
        calibrate_copy(dev)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev = None if args.no_events else HipEvents(args.steps)
    every = max(1, args.event_every)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, ev if (ev is not None and i % every == 0) else None, i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    nblk = w.blocks_needed()
    image_bytes = nblk * block_bytes + (nblk * g.num_kv_heads * 8 if g.kv_dtype == "fp8_e4m3" else 0)
    moved = 4 * image_bytes                                     # out: read + write, in: read + write
    roofline = {"bound": "hbm", "kernel": "stage_out (pool -> image)", "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": None, "traffic": None}
    if ev is not None:
        k_ms = float(np.mean([ev.elapsed_ms(i) for i in range(0, args.steps, every)]))
        roofline.update(achieved=2 * image_bytes / (k_ms * 1e-3) / 1e9, kernel_ms=k_ms, algorithmic_bytes=2 * image_bytes)
        roofline["frac"] = roofline["achieved"] / PEAK_HBM_GBS
    summary = os.path.join(ROOT, "profiles", f"stage_kernel_{args.workload}.md")
    if not host and os.path.exists(summary):
        for text in open(summary):
            if text.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(text.split(":")[1])
                roofline["traffic_source"] = os.path.relpath(summary, ROOT) + " (rocprofv3 --pmc runs of this command, not this run)"
    value = moved / (ms_per_step * 1e-3) / 1e9
    line = {
        "metric": "staging of a batch's KV blocks to an image and back: bytes read + written, GB/s",
        "value": value, "unit": "GB/s", "pct_of_peak_hbm": 100.0 * value / PEAK_HBM_GBS,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp8_e4m3": "u8", "f32": "f32"}[g.kv_dtype], "data": "synthetic",
        "config": {"workload": args.workload, "path": "stage", "image": args.stage_image, "blocks": nblk,
                   "image_bytes": image_bytes, "moved_bytes": moved,
                   "note": "pinned host image: both copies cross PCIe, the HBM roofline does not apply" if host else
                           "device image: an HBM-to-HBM copy each way"},
        "roofline": roofline,
    }
    if args.cpu_seconds > 0:                                    # the oracle's stage_out + stage_in, cycled
        opool = ol.BlockPool(w.num_blocks, w.free_order)
        olay = ol.build_layout(opool, g.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        shape = (w.num_blocks, g.num_kv_heads, 2, g.block_size, g.head_dim)
        okv = np.zeros(shape, wl.generate.STORAGE[g.kv_dtype])
        osc = np.ones((w.num_blocks, g.num_kv_heads, 2), np.float32) if g.kv_dtype == "fp8_e4m3" else None
        wall0, cpu0, reps = time.perf_counter(), time.process_time(), 0
        while time.perf_counter() - wall0 < args.cpu_seconds:
            img, img_sc = ost.stage_out(okv, osc, olay)
            ost.stage_in(okv, osc, olay, img, img_sc)
            reps += 1
        wall = time.perf_counter() - wall0
        line["cpu_baseline"] = {"value": reps * moved / wall / 1e9, "unit": "GB/s",
                                "cores": max(1, int(round((time.process_time() - cpu0) / wall))), "kind": "oracle",
                                "sample": f"numpy oracle, {reps} round trips of the whole batch, {wall:.1f} s wall"}
    return line


def cpu_prefill_baseline(w, visible, data, seconds):
    """Time the oracle on query rows of the chunk workload, one by one, until about `seconds` have passed."""
    from oracle import attention as oa
    from oracle import layout as ol
    g = w.geometry
    opool = ol.BlockPool(w.num_blocks, w.free_order)
    olay = ol.build_layout(opool, g.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    q_bits = w.q_bits()
    rows = np.random.default_rng(0).permutation(w.num_requests).tolist()
    done, flops = 0, 0
    wall0, cpu0 = time.perf_counter(), time.process_time()
    for r in rows:
        oa.decode_attention(q_bits, g.q_dtype, data.kv, data.scales, g.kv_dtype, olay, [r], visible)
        done += 1
        flops += 4 * g.head_dim * g.num_q_heads * int(visible[r])
        if time.perf_counter() - wall0 >= seconds:
            break
    wall = time.perf_counter() - wall0
    cpu = time.process_time() - cpu0
    return {"value": flops / wall / 1e12, "unit": "TFLOP/s", "cores": max(1, int(round(cpu / wall))), "kind": "oracle",
            "tokens_per_s": done / wall,
            "sample": f"fp64 numpy oracle over {done} of the {w.num_requests} new tokens (all q heads, seeded order), "
                      f"{wall:.1f} s wall"}


def main_prefill(args):
    """--path prefill: one step = the attention of every newly appended context token against its context's cached
    KV and the new tokens before it (ps_layout_set_visible + ps_decode_attention)."""
    import torch
    import workloads as wl
    from paper_2602_12029_amd import binding as B
    from paper_2602_12029_amd.runtime import DecodeBatch, to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    variant = {"auto": B.PS_VARIANT_AUTO, "wave": B.PS_VARIANT_WAVE, "mfma": B.PS_VARIANT_MFMA}
    name = args.workload if args.workload.startswith("prefill") else "prefill_" + args.workload
    w, visible = wl.named_chunk_prefill(name, args.seed)
    g = w.geometry
    geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    pool = B.ps_pool_create(w.num_blocks, w.free_order)
    layout = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    tables = B.ps_layout_tables(layout, w.num_prompts, w.num_requests)
    data = wl.fill_pool(w, tables["prefix_blk_indptr"], tables["prefix_blk"], tables["suffix_blk_indptr"],
                        tables["suffix_blk"])
    q = to_device(w.q_bits(), g.q_dtype, dev)
    kv0 = to_device(data.kv, g.kv_dtype, dev)
    copies = [kv0] + [kv0.clone() for _ in range(max(0, args.copies - 1))]
    scales = None if data.scales is None else torch.from_numpy(data.scales).to(dev)
    batch = DecodeBatch(layout, geo, w.num_requests, q, kv0, scales)
    t_lay0 = time.perf_counter()
    policy = {"auto": B.PS_KV_POLICY_AUTO, "stream": B.PS_KV_POLICY_STREAM, "cacheable": B.PS_KV_POLICY_CACHEABLE}
    B.ps_layout_replan(layout, B.plan_options(args.prefix_chunk, args.suffix_chunk, variant[args.prefix_variant],
                                              variant[args.suffix_variant], 0, policy[args.kv_policy]))
    batch.set_visible(visible)
    t_plan_ms = (time.perf_counter() - t_lay0) * 1e3
    plan = B.ps_layout_plan(layout, w.num_requests)
    stream = int(torch.cuda.current_stream().cuda_stream)
    sc = scales.data_ptr() if scales is not None else 0
    tp, qp, wp, op = batch.tables.data_ptr(), q.data_ptr(), batch.workspace.data_ptr(), batch.out.data_ptr()

    if args.calibrate_copy:
        calibrate_copy(dev)
    for i in range(args.warmup):
        batch.decode_attention(with_lse=False, kv=copies[i % len(copies)])
    torch.cuda.synchronize()
    ev = None if args.no_events else HipEvents(args.steps)
    every = max(1, args.event_every)
    t0 = time.perf_counter()
    for i in range(args.steps):
        kv = copies[i % len(copies)]
        if ev is None or i % every:
            batch.decode_attention(with_lse=False, kv=kv)
        else:
            ev.record(i, 0, stream)
            B.ps_prefix_suffix_attention(layout, tp, qp, kv.data_ptr(), sc, wp, stream)
            ev.record(i, 1, stream)
            B.ps_merge_states(layout, tp, wp, op, 0, stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # algorithmic work: 2 d multiply-adds for the score and 2 d for the weighted value, per (q head, visible token)
    flops = 4 * g.head_dim * g.num_q_heads * int(visible.astype(np.int64).sum())
    ideal = wl.ideal_bytes(w)
    roofline = {"bound": "mfma", "kernel": "attention (masked prefix work list)", "achieved": None,
                "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s", "frac": None, "traffic": None}
    if ev is not None:
        k_ms = float(np.mean([ev.elapsed_ms(i) for i in range(0, args.steps, every)]))
        roofline.update(achieved=flops / (k_ms * 1e-3) / 1e12, kernel_ms=k_ms, algorithmic_flops=flops)
        roofline["frac"] = roofline["achieved"] / PEAK_MFMA_BF16_TFLOPS
    summary = os.path.join(ROOT, "profiles", f"attention_kernel_{name}.md")
    if os.path.exists(summary):
        for text in open(summary):
            if text.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(text.split(":")[1])
                roofline["traffic_source"] = os.path.relpath(summary, ROOT) + " (rocprofv3 --pmc runs of this command, not this run)"
    value = flops / (ms_per_step * 1e-3) / 1e12
    line = {
        "metric": "partial-prefill attention over the shared cache: algorithmic TFLOP/s + new tokens/sec",
        "value": value, "unit": "TFLOP/s", "pct_of_peak_mfma": 100.0 * value / PEAK_MFMA_BF16_TFLOPS,
        "tokens_per_s": w.num_requests / (ms_per_step * 1e-3),
        "ideal_byte_gbs": ideal / (ms_per_step * 1e-3) / 1e9,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if g.kv_dtype == "bf16" else ("fp8_e4m3 KV / bf16 Q" if g.kv_dtype == "fp8_e4m3" else "f32"),
        "data": "synthetic",
        "config": {"workload": name, "path": "prefill", "contexts": w.num_prompts, "new_tokens": w.num_requests,
                   "cached_tokens": int((w.prefix_len.astype(np.int64)).sum()) - w.num_requests,
                   "q_heads": g.num_q_heads, "kv_heads": g.num_kv_heads, "head_dim": g.head_dim,
                   "block_size": g.block_size, "ideal_bytes": ideal, "pool_copies": len(copies),
                   "plan_items": int(plan["items"].shape[0]), "plan_ms": t_plan_ms},
        "roofline": roofline,
    }
    if args.cpu_seconds > 0:
        line["cpu_baseline"] = cpu_prefill_baseline(w, visible, data, args.cpu_seconds)
    return line


def measure_loop(args, name, steps, warmup, random_kv=False):
    """A multi-step decode loop: per step one token is appended to every private segment (host tables, upload, the
    store of the new K/V) and one decode-attention call follows, all on one stream, the host never waiting for the GPU.
    random_kv: fill the pool on the device with random bits instead of the workload's generated K/V (the step's time
    does not depend on the values; used for the per_config map, where generating `mixed` a second time would cost a
    minute of host time)."""
    import torch
    import workloads as wl
    from paper_2602_12029_amd import binding as B
    from paper_2602_12029_amd.runtime import to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    w = wl.named_workload(name, args.seed, args.models or None)
    g = w.geometry
    R = w.num_requests
    total_steps = warmup + steps
    extra = R * (total_steps // g.block_size + 2)                       # blocks the appends may take
    geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    order = np.concatenate([np.asarray(w.free_order, np.int32), np.arange(w.num_blocks, w.num_blocks + extra, dtype=np.int32)])
    pool = B.ps_pool_create(w.num_blocks + extra, order)
    layout = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    tables = B.ps_layout_tables(layout, w.num_prompts, R)
    per_block = g.num_kv_heads * 2 * g.block_size * g.head_dim
    scales = None
    if random_kv:
        n_el = (w.num_blocks + extra) * per_block
        if g.kv_dtype == "fp8_e4m3":
            kv = torch.randint(0, 120, (n_el,), dtype=torch.uint8, device=dev)          # finite e4m3 codes
            scales = torch.ones((w.num_blocks + extra, g.num_kv_heads, 2), dtype=torch.float32, device=dev)
        else:
            kv = torch.randn(n_el, device=dev).to(torch.bfloat16 if g.kv_dtype == "bf16" else torch.float32)
    else:
        data = wl.fill_pool(w, tables["prefix_blk_indptr"], tables["prefix_blk"], tables["suffix_blk_indptr"], tables["suffix_blk"])
        kv_filled = to_device(data.kv, g.kv_dtype, dev)
        kv = torch.zeros((w.num_blocks + extra) * per_block, dtype=kv_filled.dtype, device=dev)
        kv[:kv_filled.numel()] = kv_filled.reshape(-1)
        if data.scales is not None:
            scales = torch.ones((w.num_blocks + extra, g.num_kv_heads, 2), dtype=torch.float32, device=dev)
            scales[:w.num_blocks] = torch.from_numpy(data.scales).to(dev)
    q = to_device(w.q_bits(), g.q_dtype, dev)
    out = torch.empty_like(q)
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    new_k = torch.randn((R, g.num_kv_heads, g.head_dim), device=dev, generator=gen).to(torch.bfloat16 if g.kv_dtype != "f32" else torch.float32)
    new_v = torch.randn((R, g.num_kv_heads, g.head_dim), device=dev, generator=gen).to(new_k.dtype)
    # device buffers with room for the growth of the tables and of the partial-state workspace; two table buffers,
    # filled alternately on a copy stream, so that the upload of step i + 1 overlaps with the kernels of step i
    tab_bytes = int(B.ps_layout_device_bytes(layout) * 1.5) + (1 << 20)
    tabs = [torch.empty(tab_bytes, dtype=torch.uint8, device=dev) for _ in range(2)]
    wsp = torch.empty(int(B.ps_workspace_bytes(layout) * 2) + (1 << 20), dtype=torch.uint8, device=dev)
    compute = torch.cuda.current_stream()
    copy = torch.cuda.Stream()                                    # default priority
    uploaded = [torch.cuda.Event() for _ in range(2)]             # tables i are on the device
    consumed = [torch.cuda.Event() for _ in range(2)]             # the kernels that read tables i are done
    stream, copy_stream = int(compute.cuda_stream), int(copy.cuda_stream)
    sc = scales.data_ptr() if scales is not None else 0
    host_s = 0.0
    host_all = [0.0]
    count = 0

    def step():
        nonlocal host_s, count
        i = count & 1
        count += 1
        h0 = time.perf_counter()
        B.ps_layout_append(pool, layout, R)
        if B.ps_layout_device_bytes(layout) > tab_bytes or B.ps_workspace_bytes(layout) > wsp.numel():
            sys.exit("bench.py: tables or workspace outgrew their buffers")
        host_s += time.perf_counter() - h0
        if count > 2:
            copy.wait_event(consumed[i])
        B.ps_layout_upload(layout, tabs[i].data_ptr(), copy_stream)
        uploaded[i].record(copy)
        uploaded[i].synchronize()     # on the host (it runs ahead of the GPU): no wait packet in the compute stream
        tp = tabs[i].data_ptr()
        B.ps_kv_append(layout, tp, new_k.data_ptr(), new_v.data_ptr(), kv.data_ptr(), sc, stream)
        B.ps_decode_attention(layout, tp, q.data_ptr(), kv.data_ptr(), sc, wsp.data_ptr(), out.data_ptr(), 0, stream)
        consumed[i].record(compute)
        host_all[0] += time.perf_counter() - h0

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    host_s = 0.0
    host_all[0] = 0.0
    bytes0 = wl.ideal_bytes(w) + R * warmup * g.token_bytes
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    ideal = bytes0 + R * g.token_bytes * (steps + 1) / 2            # mean over the timed steps: one more token per request and step
    value = ideal / (ms_per_step * 1e-3) / 1e9
    line = {
        "metric": "decode loop (append + decode attention per step): ideal-byte HBM GB/s + queries/sec",
        "value": value, "unit": "GB/s", "pct_of_peak_hbm": 100.0 * value / PEAK_HBM_GBS,
        "queries_per_s": R / (ms_per_step * 1e-3), "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "host_ms_per_step": host_s * 1e3 / steps,
        "host_enqueue_ms_per_step": host_all[0] * 1e3 / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp8_e4m3": "u8", "f32": "f32"}[g.kv_dtype], "data": "synthetic",
        "config": {"workload": name, "path": "loop", "requests": R, "mean_ideal_bytes": ideal,
                   "note": "host_ms_per_step = ps_layout_append; the tables go up on a copy stream into two device buffers "
                           "used alternately, so the upload of a step overlaps with the kernels of the step before"},
        "roofline": {"bound": "hbm", "achieved": value, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": value / PEAK_HBM_GBS,
                     "traffic": None, "kernel": "whole step (append store + attention + merge), wall clock"},
    }
    torch.cuda.synchronize()
    B.ps_layout_release(pool, layout)
    B.ps_pool_destroy(pool)
    del kv, tabs, wsp
    torch.cuda.empty_cache()
    return line


def main_loop(args):
    print(json.dumps(measure_loop(args, args.workload, args.steps, args.warmup)))


def read_ceiling_gbs(stream, nbytes=1 << 30):
    """Rate of the read probe with whole-line loads: the ceiling this GPU gives a kernel shaped like the attention kernel."""
    import torch
    from paper_2602_12029_amd import binding as B
    buf = torch.ones(nbytes, dtype=torch.uint8, device="cuda:0")
    ev = HipEvents(5)
    B.ps_probe_read(buf.data_ptr(), nbytes, 0, 512, stream)
    for i in range(5):
        ev.record(i, 0, stream)
        B.ps_probe_read(buf.data_ptr(), nbytes, 0, 512, stream)
        ev.record(i, 1, stream)
    torch.cuda.synchronize()
    return nbytes / (min(ev.elapsed_ms(i) for i in range(5)) * 1e-3) / 1e9


def main_probe(args):
    """--path probe: read ceilings of this GPU for the load footprints of the attention kernel (ps_probe_read)."""
    import torch
    from paper_2602_12029_amd import binding as B

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    nbytes = 2 << 30                                   # well past the 256 MB last-level cache
    buf = torch.ones(nbytes, dtype=torch.uint8, device="cuda:0")
    stream = int(torch.cuda.current_stream().cuda_stream)
    patterns = {0: "16 B per lane, 1 KiB contiguous per instruction",
                1: "16 B per lane, 16 rows x 64 B of 128-byte rows (half lines)",
                2: "16 B per lane, 16 rows x 64 B of 256-byte rows (half lines)",
                3: "8 B per lane, 512 B contiguous per instruction",
                4: "16 B per lane, 1 KiB per instruction, 2 KiB chunks in scrambled order",
                5: "16 B per lane, 1 KiB per instruction, 4 KiB chunks in scrambled order",
                6: "16 B per lane, 1 KiB per instruction, 8 KiB chunks in scrambled order"}
    steps = max(1, min(args.steps, 20))
    ev = HipEvents(steps)
    rates = {}
    t0 = time.perf_counter()
    for pat, what in patterns.items():
        for _ in range(2):
            B.ps_probe_read(buf.data_ptr(), nbytes, pat, 512, stream)
        for i in range(steps):
            ev.record(i, 0, stream)
            B.ps_probe_read(buf.data_ptr(), nbytes, pat, 512, stream)
            ev.record(i, 1, stream)
        torch.cuda.synchronize()
        ms = min(ev.elapsed_ms(i) for i in range(steps))
        rates[what] = {"GB/s": nbytes / (ms * 1e-3) / 1e9, "ms": ms}
    wall_ms = (time.perf_counter() - t0) * 1e3 / (len(patterns) * steps)
    best = max(r["GB/s"] for r in rates.values())
    print(json.dumps({
        "metric": "read probe: GB/s of a read-only kernel by load-instruction footprint (not the method's metric)",
        "value": best, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": 2, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "probe", "bytes": nbytes, "workgroups": 512, "in_flight_per_wave": 8192,
                   "loads": "non-temporal", "timing": "fastest of the timed launches, HIP events"},
        "patterns": rates,
        "roofline": {"bound": "hbm", "achieved": best, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": best / PEAK_HBM_GBS,
                     "traffic": None},
    }))


def _stats(samples):
    x = np.asarray(samples, np.float64)
    return {"mean": float(x.mean()), "median": float(np.median(x)), "min": float(x.min()), "n": int(x.size)}


def measure_decode(args, name, steps, warmup, cpu_seconds, ceiling):
    """One workload through ps_decode_attention: wall clock over exactly `steps` steps, then an event-bracketed loop
    (at least 20 steps, whatever `steps` is) that gives the attention launch(es) and the whole step one by one."""
    import torch
    import workloads as wl
    from paper_2602_12029_amd import binding as B
    from paper_2602_12029_amd.runtime import DecodeBatch, to_device

    dev = "cuda:0"
    variant = {"auto": B.PS_VARIANT_AUTO, "wave": B.PS_VARIANT_WAVE, "mfma": B.PS_VARIANT_MFMA}
    tree = name.startswith("tree")
    w = wl.named_tree_workload(name, args.seed) if tree else wl.named_workload(name, args.seed, args.models or None)
    g = w.geometry
    geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    pool = B.ps_pool_create(w.num_blocks, w.free_order)
    t_lay0 = time.perf_counter()
    if tree:
        layout = B.ps_kv_layout_tree(pool, geo, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt, w.req_model,
                                     w.suffix_len)
    else:
        layout = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    policy = {"auto": B.PS_KV_POLICY_AUTO, "stream": B.PS_KV_POLICY_STREAM, "cacheable": B.PS_KV_POLICY_CACHEABLE}
    B.ps_layout_replan(layout, B.plan_options(args.prefix_chunk, args.suffix_chunk, variant[args.prefix_variant],
                                              variant[args.suffix_variant], 0, policy[args.kv_policy]))
    t_layout_ms = (time.perf_counter() - t_lay0) * 1e3
    tables = B.ps_layout_tables(layout, w.num_prompts, w.num_requests)
    roots = B.ps_layout_root_tables(layout)
    data = wl.fill_pool(w, tables["prefix_blk_indptr"], tables["prefix_blk"], tables["suffix_blk_indptr"],
                        tables["suffix_blk"], roots["root_blk_indptr"], roots["root_blk"])
    q = to_device(w.q_bits(), g.q_dtype, dev)
    kv0 = to_device(data.kv, g.kv_dtype, dev)
    copies = [kv0] + [kv0.clone() for _ in range(max(0, args.copies - 1))]
    scales = None if data.scales is None else torch.from_numpy(data.scales).to(dev)
    batch = DecodeBatch(layout, geo, w.num_requests, q, kv0, scales)
    plan = B.ps_layout_plan(layout, w.num_requests)
    stream = int(torch.cuda.current_stream().cuda_stream)
    sc = scales.data_ptr() if scales is not None else 0
    tp, qp, wp, op = batch.tables.data_ptr(), q.data_ptr(), batch.workspace.data_ptr(), batch.out.data_ptr()

    if args.calibrate_copy:
        calibrate_copy(dev)

    for i in range(warmup):
        batch.decode_attention(with_lse=False, kv=copies[i % len(copies)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        batch.decode_attention(with_lse=False, kv=copies[i % len(copies)])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    ideal = wl.ideal_bytes(w)
    esz_q = wl.generate.ELEM_BYTES[g.q_dtype]
    attn_bytes = ideal - w.num_requests * g.num_q_heads * g.head_dim * esz_q        # O is written by the merge
    roofline = {"bound": "hbm", "kernel": "attention (prefix + suffix work list)", "achieved": None,
                "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None, "traffic": None}
    step_stats = None
    if not args.no_events:
        # the same step, one by one: event, attention launch(es), event, merge, event
        n = max(20, args.event_steps)
        ev_a, ev_b = HipEvents(n), HipEvents(n)
        for i in range(n):
            kv = copies[(steps + i) % len(copies)]
            ev_a.record(i, 0, stream)
            B.ps_prefix_suffix_attention(layout, tp, qp, kv.data_ptr(), sc, wp, stream)
            ev_a.record(i, 1, stream)
            B.ps_merge_states(layout, tp, wp, op, 0, stream)
            ev_b.record(i, 1, stream)
        torch.cuda.synchronize()
        ev_b.events = [(ev_a.events[i][0], ev_b.events[i][1]) for i in range(n)]
        k = _stats([ev_a.elapsed_ms(i) for i in range(n)])
        step_stats = _stats([ev_b.elapsed_ms(i) for i in range(n)])
        roofline.update(achieved=attn_bytes / (k["mean"] * 1e-3) / 1e9, kernel_ms=k["mean"], kernel_ms_median=k["median"],
                        kernel_ms_min=k["min"], kernel_samples=k["n"], algorithmic_bytes=attn_bytes)
        roofline["frac"] = roofline["achieved"] / PEAK_HBM_GBS
        if ceiling:
            roofline["read_ceiling"] = {"value": ceiling, "unit": "GB/s", "frac_of_it": roofline["achieved"] / ceiling,
                                        "how": "ps_probe_read, 16 B per lane and 1 KiB per instruction, fastest of 5 launches"}

    # HBM bytes per launch: not measured by this run -- read from the committed rocprofv3 counter summary of this
    # workload (two --pmc runs of this command, FETCH_SIZE and WRITE_SIZE), if there is one
    summary = os.path.join(ROOT, "profiles", f"attention_kernel_{name}.md")
    if os.path.exists(summary):
        for text in open(summary):
            if text.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(text.split(":")[1])
                roofline["traffic_source"] = f"profiles/attention_kernel_{name}.md (rocprofv3 --pmc runs of this command, not this run)"

    value = ideal / (ms_per_step * 1e-3) / 1e9
    res = {
        "value": value, "pct_of_peak_hbm": 100.0 * value / PEAK_HBM_GBS,
        "queries_per_s": w.num_requests / (ms_per_step * 1e-3), "ms_per_step": ms_per_step,
        "dtype": "bf16" if g.kv_dtype == "bf16" else ("fp8_e4m3 KV / bf16 Q" if g.kv_dtype == "fp8_e4m3" else "f32"),
        "config": {"workload": name, "roots": w.num_roots, "models": w.num_models, "prompts": w.num_prompts,
                   "requests": w.num_requests, "q_heads": g.num_q_heads, "kv_heads": g.num_kv_heads,
                   "head_dim": g.head_dim, "block_size": g.block_size, "ideal_bytes": ideal,
                   "pool_copies": len(copies), "plan_items": int(plan["items"].shape[0]),
                   "prefix_variant": plan["prefix_variant"], "suffix_variant": plan["suffix_variant"],
                   "layout_plan_ms": t_layout_ms},
        "roofline": roofline,
    }
    if not tree:
        # KV footprint with the prompts' contexts stored once against once per decode model (Efficiency Analysis, Eq. 9)
        blk_bytes = g.num_kv_heads * 2 * g.block_size * g.head_dim * wl.generate.ELEM_BYTES[g.kv_dtype]
        shared = B.ps_blocks_needed(g.block_size, w.prefix_len, w.suffix_len)
        unshared = B.ps_blocks_needed(g.block_size, [], w.prefix_len[w.req_prompt] + w.suffix_len)
        res["config"].update(kv_bytes_shared=shared * blk_bytes, kv_bytes_unshared=unshared * blk_bytes,
                             kv_footprint_ratio=unshared / max(shared, 1))
    if step_stats:
        res["ms_per_step_median"] = step_stats["median"]
        res["ms_per_step_events_mean"] = step_stats["mean"]
        res["value_at_median"] = ideal / (step_stats["median"] * 1e-3) / 1e9
    if cpu_seconds > 0:
        res["cpu_baseline"] = cpu_baseline(w, tables, data, cpu_seconds)
    torch.cuda.synchronize()
    B.ps_layout_release(pool, layout)
    B.ps_pool_destroy(pool)
    del batch, copies, kv0, q, scales, data
    torch.cuda.empty_cache()
    return res


PER_CONFIG = ("b8", "long", "mixed", "fp8_70b")


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the decode attention of ONE GPU (no collectives, no sharding); "
                 "use --gpus 1")
    if args.path == "ingest":
        return print(json.dumps(main_ingest(args)))
    if args.path == "prefill":
        return print(json.dumps(main_prefill(args)))
    if args.path == "stage":
        return print(json.dumps(main_stage(args)))
    if args.path == "loop":
        return main_loop(args)
    if args.path == "probe":
        return main_probe(args)
    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    stream = int(torch.cuda.current_stream().cuda_stream)
    # what a read-only kernel of the attention kernel's launch shape reaches on this GPU right now (1 GiB)
    ceiling = None if args.no_events else read_ceiling_gbs(stream)
    head = measure_decode(args, args.workload, args.steps, args.warmup, args.cpu_seconds, ceiling)
    line = {
        "metric": "shared-prefix decode attention: ideal-byte HBM GB/s (% peak) + queries/sec",
        "value": head["value"], "unit": "GB/s", "pct_of_peak_hbm": head["pct_of_peak_hbm"],
        "queries_per_s": head["queries_per_s"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "ms_per_step_median": head.get("ms_per_step_median"), "value_at_median": head.get("value_at_median"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"], "roofline": head["roofline"],
    }
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
    if args.per_config:
        # the other benchmark configurations, each its own short run of the same step (no oracle leg)
        per = {}
        for name in PER_CONFIG:
            r = head if name == args.workload else measure_decode(args, name, max(args.steps, 50), max(args.warmup, 10), 0.0, ceiling)
            rf = r["roofline"]
            per[name] = {"ms_per_step": r["ms_per_step"], "ms_per_step_median": r.get("ms_per_step_median"),
                         "value": r["value"], "unit": "GB/s", "pct_of_peak_hbm": r["pct_of_peak_hbm"],
                         "queries_per_s": r["queries_per_s"], "ideal_bytes": r["config"]["ideal_bytes"],
                         "roofline_frac": rf["frac"], "kernel_ms": rf.get("kernel_ms"),
                         "kernel_ms_median": rf.get("kernel_ms_median"),
                         "read_ceiling_frac": (rf.get("read_ceiling") or {}).get("frac_of_it")}
            # the multi-step decode loop on the same batch (append on the host, table upload, ps_kv_append, the step)
            lp = measure_loop(args, name, max(args.steps, 50), max(args.warmup, 10), random_kv=True)
            per[name]["loop"] = {"ms_per_step": lp["ms_per_step"], "value": lp["value"], "unit": "GB/s",
                                 "host_append_ms_per_step": lp["host_ms_per_step"]}
        line["per_config"] = per
        # the paths around the decode step, each a short run of its own `--path` line (no oracle leg): hand-off of
        # the batch's KV into the pool, partial prefill of newly appended context tokens, staging out and back
        import copy
        other = {}
        for key, fn, over in (("ingest_b8", main_ingest, {"workload": "b8"}),
                              ("ingest_fp8_70b", main_ingest, {"workload": "fp8_70b"}),
                              ("prefill_b8", main_prefill, {"workload": "prefill_b8"}),
                              ("prefill_fp8", main_prefill, {"workload": "prefill_fp8"}),
                              ("stage_b8", main_stage, {"workload": "b8"})):
            a = copy.copy(args)
            a.cpu_seconds, a.steps, a.warmup, a.models, a.no_events = 0.0, 30, 5, 0, False
            for k, v in over.items():
                setattr(a, k, v)
            r = fn(a)
            rf = r.get("roofline") or {}
            other[key] = {"metric": r["metric"], "ms_per_step": r["ms_per_step"], "value": r["value"], "unit": r["unit"],
                          "roofline_bound": rf.get("bound"), "roofline_kernel": rf.get("kernel"),
                          "roofline_frac": rf.get("frac"), "kernel_ms": rf.get("kernel_ms")}
            torch.cuda.empty_cache()
        line["other_paths"] = other
    print(json.dumps(line))


if __name__ == "__main__":
    main()
