#!/usr/bin/env python3
"""Benchmark: one decode-attention step over shared prefix KV + private suffix KV on one MI355X.

A step is one ps_decode_attention call (prefix pass, suffix pass, merge) over one synthetic batch
with all inputs resident in HBM.  Steps rotate over several copies of the KV pool so that no step
finds its KV in the last-level cache.  Prints one JSON line:
  value     ideal-byte GB/s of the whole step (shared KV counted once + private KV + Q + O)
  roofline  the attention kernel alone, timed with HIP events on its stream inside the timed loop
  cpu_baseline  the fp64 numpy oracle on a bounded sample of the same workload, on this host
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
    ap.add_argument("--workload", default="b8", help="tiny | b8 | long | mixed | fp8_70b")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--models", type=int, default=0, help="override the number of decode models M (b8, long, fp8_70b)")
    ap.add_argument("--copies", type=int, default=3, help="distinct KV pool copies rotated between steps")
    ap.add_argument("--prefix-chunk", type=int, default=0)
    ap.add_argument("--suffix-chunk", type=int, default=0)
    ap.add_argument("--prefix-variant", default="auto")
    ap.add_argument("--suffix-variant", default="auto")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target wall time of the oracle sample; 0 = skip")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events in the timed loop")
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
    """Time the oracle on whole prompts (all their requests) until about `seconds` have passed."""
    from oracle import attention as oa
    from oracle import layout as ol
    import workloads as wl
    g = w.geometry
    opool = ol.BlockPool(w.num_blocks, w.free_order)
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


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the decode attention of ONE GPU (no collectives, no sharding); "
                 "use --gpus 1")
    import torch
    import workloads as wl
    from paper_2602_12029_amd import binding as B
    from paper_2602_12029_amd.runtime import DecodeBatch, to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    variant = {"auto": B.PS_VARIANT_AUTO, "wave": B.PS_VARIANT_WAVE, "mfma": B.PS_VARIANT_MFMA}
    w = wl.named_workload(args.workload, args.seed, args.models or None)
    g = w.geometry
    geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    pool = B.ps_pool_create(w.num_blocks, w.free_order)
    t_lay0 = time.perf_counter()
    layout = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    B.ps_layout_replan(layout, B.plan_options(args.prefix_chunk, args.suffix_chunk, variant[args.prefix_variant],
                                              variant[args.suffix_variant]))
    t_layout_ms = (time.perf_counter() - t_lay0) * 1e3
    tables = B.ps_layout_tables(layout, w.num_prompts, w.num_requests)
    data = wl.fill_pool(w, tables["prefix_blk_indptr"], tables["prefix_blk"], tables["suffix_blk_indptr"],
                        tables["suffix_blk"])
    q = to_device(w.q_bits(), g.q_dtype, dev)
    kv0 = to_device(data.kv, g.kv_dtype, dev)
    copies = [kv0] + [kv0.clone() for _ in range(max(0, args.copies - 1))]
    scales = None if data.scales is None else torch.from_numpy(data.scales).to(dev)
    batch = DecodeBatch(layout, geo, w.num_requests, q, kv0, scales)
    plan = B.ps_layout_plan(layout, w.num_requests)
    stream = int(torch.cuda.current_stream().cuda_stream)
    sc = scales.data_ptr() if scales is not None else 0
    tp, qp, wp, op = batch.tables.data_ptr(), q.data_ptr(), batch.workspace.data_ptr(), batch.out.data_ptr()

    def attention(kv):      # the dominant kernel(s): prefix + suffix work list
        B.ps_prefix_suffix_attention(layout, tp, qp, kv.data_ptr(), sc, wp, stream)

    if args.calibrate_copy:      # known traffic: reads 2^30 bytes, writes 2^30 bytes per launch
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        batch.decode_attention(with_lse=False, kv=copies[i % len(copies)])
    torch.cuda.synchronize()

    ev = None if args.no_events else HipEvents(args.steps)
    every = max(1, args.event_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        kv = copies[i % len(copies)]
        if ev is None or i % every:
            batch.decode_attention(with_lse=False, kv=kv)
        else:
            ev.record(i, 0, stream)
            attention(kv)
            ev.record(i, 1, stream)
            B.ps_merge_states(layout, tp, wp, op, 0, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    ideal = wl.ideal_bytes(w)
    esz_q = wl.generate.ELEM_BYTES[g.q_dtype]
    attn_bytes = ideal - w.num_requests * g.num_q_heads * g.head_dim * esz_q        # O is written by the merge
    roofline = {"bound": "hbm", "kernel": "attention (prefix + suffix work list)", "achieved": None,
                "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None, "traffic": None}
    if ev is not None:
        k_ms = float(np.mean([ev.elapsed_ms(i) for i in range(0, args.steps, every)]))
        roofline.update(achieved=attn_bytes / (k_ms * 1e-3) / 1e9, kernel_ms=k_ms, algorithmic_bytes=attn_bytes)
        roofline["frac"] = roofline["achieved"] / PEAK_HBM_GBS

    # HBM bytes per launch from the committed rocprofv3 counter summary of this workload, if there is one
    summary = os.path.join(ROOT, "profiles", f"attention_kernel_{args.workload}.md")
    if os.path.exists(summary):
        for text in open(summary):
            if text.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(text.split(":")[1])

    value = ideal / (ms_per_step * 1e-3) / 1e9
    line = {
        "metric": "shared-prefix decode attention: ideal-byte HBM GB/s (% peak) + queries/sec",
        "value": value, "unit": "GB/s", "pct_of_peak_hbm": 100.0 * value / PEAK_HBM_GBS,
        "queries_per_s": w.num_requests / (ms_per_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if g.kv_dtype == "bf16" else ("fp8_e4m3 KV / bf16 Q" if g.kv_dtype == "fp8_e4m3" else "f32"),
        "data": "synthetic",
        "config": {"workload": args.workload, "models": w.num_models, "prompts": w.num_prompts,
                   "requests": w.num_requests, "q_heads": g.num_q_heads, "kv_heads": g.num_kv_heads,
                   "head_dim": g.head_dim, "block_size": g.block_size, "ideal_bytes": ideal,
                   "pool_copies": len(copies), "plan_items": int(plan["items"].shape[0]),
                   "prefix_variant": plan["prefix_variant"], "suffix_variant": plan["suffix_variant"],
                   "layout_plan_ms": t_layout_ms},
        "roofline": roofline,
    }
    if args.cpu_seconds > 0:
        line["cpu_baseline"] = cpu_baseline(w, tables, data, args.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
