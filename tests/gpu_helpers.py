"""Plumbing for the GPU parity tests: build the library-side layout, check it against the oracle's, upload."""
import numpy as np
import torch

import workloads as wl
from helpers import oracle_setup
from paper_2602_12029_amd import binding as B
from paper_2602_12029_amd.runtime import DecodeBatch, to_device

VARIANT = {"auto": B.PS_VARIANT_AUTO, "wave": B.PS_VARIANT_WAVE, "mfma": B.PS_VARIANT_MFMA}


class GpuCase:
    """One workload on the GPU next to its oracle-side layout and pool."""

    def __init__(self, w: wl.Workload, device="cuda:0"):
        self.w = w
        g = w.geometry
        self.geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
        self.pool = B.ps_pool_create(w.num_blocks, w.free_order)
        self.layout = B.ps_kv_layout(self.pool, self.geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        self.opool, self.olay, self.data = oracle_setup(w)
        t = B.ps_layout_tables(self.layout, w.num_prompts, w.num_requests)
        for key in t:                                      # index work is bit-exact, so one pool serves both sides
            assert np.array_equal(t[key], getattr(self.olay, key)), key
        self.q_bits = w.q_bits()
        q = to_device(self.q_bits, g.q_dtype, device)
        kv = to_device(self.data.kv, g.kv_dtype, device)
        scales = None if self.data.scales is None else torch.from_numpy(self.data.scales).to(device)
        self.batch = DecodeBatch(self.layout, self.geo, w.num_requests, q, kv, scales)

    def replan(self, prefix_chunk=0, suffix_chunk=0, prefix_variant="auto", suffix_variant="auto", num_cus=0):
        self.batch.replan(B.plan_options(prefix_chunk, suffix_chunk, VARIANT[prefix_variant], VARIANT[suffix_variant],
                                         num_cus))

    def poison_workspace(self):
        self.batch.workspace.view(torch.float32).fill_(float("nan"))
        self.batch.out.view(torch.int16 if self.w.geometry.q_dtype == "bf16" else torch.int32).fill_(-1)
        self.batch.lse.fill_(float("nan"))

    def close(self):
        torch.cuda.synchronize()
        B.ps_layout_release(self.pool, self.layout)
        B.ps_pool_destroy(self.pool)
