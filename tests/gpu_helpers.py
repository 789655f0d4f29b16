"""Plumbing for the GPU parity tests: build the library-side layout, check it against the oracle's, upload."""
import numpy as np
import torch

import workloads as wl
from helpers import errors, oracle_setup
from oracle import attention as oa
from paper_2602_12029_amd import binding as B
from paper_2602_12029_amd.runtime import DecodeBatch, to_device

VARIANT = {"auto": B.PS_VARIANT_AUTO, "wave": B.PS_VARIANT_WAVE, "mfma": B.PS_VARIANT_MFMA}


TOL = {"f32": (1e-5, 1e-5), "bf16": (1e-2, 5e-3), "fp8_e4m3": (1e-2, 5e-3)}   # (max-abs, relative RMS) by KV dtype


def check_against_oracle(case, requests=None, label="", visible=None, scaled_bar=False):
    """Output and LSE of the last step on the GPU against the fp64 oracle, element by element.

    The bars are the stated ones: max-abs and relative RMS by KV dtype (TOL).  scaled_bar=True is for cases whose rows
    see only a handful of tokens (or whose softmax is peaked on a few), so that |O| reaches 2-4: an element with
    |O_ref| > 1 is then held to tol x |O_ref| instead, because half the spacing of bf16 -- the output format -- is
    already 7.8e-3 on [2, 4); elements with |O_ref| <= 1 keep the literal bar.  The number of elements that used the
    scaled bar is printed.  Without the flag every element is held to the literal bar."""
    from paper_2602_12029_amd.runtime import from_device
    w = case.w
    g = w.geometry
    ref_o, ref_lse = oa.decode_attention(case.q_bits, g.q_dtype, case.data.kv, case.data.scales, g.kv_dtype, case.olay,
                                         requests, visible)
    torch.cuda.synchronize()
    got_o = from_device(case.batch.out)
    got_lse = from_device(case.batch.lse)
    if requests is not None:
        got_o, got_lse = got_o[list(requests)], got_lse[list(requests)]
    max_abs, rel_rms, worst = errors(got_o, ref_o)
    tol_abs, tol_rms = TOL[g.kv_dtype]
    assert np.isfinite(got_o).all()
    err = np.abs(got_o - ref_o)
    big = np.abs(ref_o) > 1.0
    n_scaled = int(big.sum()) if (scaled_bar and g.q_dtype != "f32") else 0
    print(f"[{label or w.name}] max_abs={max_abs:.3e} rel_rms={rel_rms:.3e} worst_req_rel_rms={worst:.3e} "
          f"scaled_bar_elements={n_scaled}/{err.size}", flush=True)
    if n_scaled:
        assert err[~big].max(initial=0.0) <= tol_abs
        assert (err[big] / np.abs(ref_o[big])).max(initial=0.0) <= tol_abs
    else:
        assert max_abs <= tol_abs
    assert rel_rms <= tol_rms
    finite = np.isfinite(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(ref_lse))
    assert np.abs(got_lse[finite] - ref_lse[finite]).max(initial=0.0) <= (1e-4 if g.kv_dtype == "f32" else 2e-3)
    return max_abs, rel_rms


def pool_strides(g, num_blocks, pool_layout):
    """(block, head, kv, tok) strides in elements of a physical pool layout, and the axis order that turns the dense
    [blk][Hkv][2][B][d] array into it.

    dense        [blk][Hkv][K|V][B][d]   a (block, head) tile is one contiguous piece
    token_major  [blk][K|V][B][Hkv][d]   all heads of a token side by side, as a model's projection writes them
    planes       [K|V][blk][Hkv][B][d]   one K cache and one V cache, a whole pool apart
    """
    h, b, d = g.num_kv_heads, g.block_size, g.head_dim
    if pool_layout == "dense":
        return None, (0, 1, 2, 3, 4)
    if pool_layout == "token_major":
        return (2 * b * h * d, d, b * h * d, h * d), (0, 2, 3, 1, 4)
    if pool_layout == "planes":
        return (h * b * d, b * d, num_blocks * h * b * d, d), (2, 0, 1, 3, 4)
    raise ValueError(pool_layout)


class GpuCase:
    """One workload on the GPU next to its oracle-side layout and pool."""

    def __init__(self, w: wl.Workload, device="cuda:0", pool_layout="dense"):
        self.w = w
        g = w.geometry
        strides, axes = pool_strides(g, w.num_blocks, pool_layout)
        self.pool_axes = axes
        self.geo = B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype, strides)
        self.pool = B.ps_pool_create(w.num_blocks, w.free_order)
        if w.num_roots:
            self.layout = B.ps_kv_layout_tree(self.pool, self.geo, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt,
                                              w.req_model, w.suffix_len)
        else:
            self.layout = B.ps_kv_layout(self.pool, self.geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        self.opool, self.olay, self.data = oracle_setup(w)
        t = B.ps_layout_tables(self.layout, w.num_prompts, w.num_requests)
        if w.num_roots:
            t.update(B.ps_layout_root_tables(self.layout))
        for key in t:                                      # index work is bit-exact, so one pool serves both sides
            assert np.array_equal(t[key], getattr(self.olay, key)), key
        self.q_bits = w.q_bits()
        q = to_device(self.q_bits, g.q_dtype, device)
        # the oracle keeps its dense pool; the device gets the same bits in the layout the strides describe
        kv = to_device(np.ascontiguousarray(self.data.kv.transpose(axes)), g.kv_dtype, device)
        scales = None if self.data.scales is None else torch.from_numpy(self.data.scales).to(device)
        self.batch = DecodeBatch(self.layout, self.geo, w.num_requests, q, kv, scales)

    def replan(self, prefix_chunk=0, suffix_chunk=0, prefix_variant="auto", suffix_variant="auto", num_cus=0,
               kv_cache_policy=0):
        self.batch.replan(B.plan_options(prefix_chunk, suffix_chunk, VARIANT[prefix_variant], VARIANT[suffix_variant],
                                         num_cus, kv_cache_policy))

    def set_visible(self, visible=None):
        self.batch.set_visible(visible)

    def poison_workspace(self):
        self.batch.workspace.view(torch.float32).fill_(float("nan"))
        self.batch.out.view(torch.int16 if self.w.geometry.q_dtype == "bf16" else torch.int32).fill_(-1)
        self.batch.lse.fill_(float("nan"))

    def close(self):
        torch.cuda.synchronize()
        B.ps_layout_release(self.pool, self.layout)
        B.ps_pool_destroy(self.pool)
