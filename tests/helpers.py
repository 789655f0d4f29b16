"""Shared test plumbing (no arithmetic of the method)."""
import numpy as np

import workloads as wl
from oracle import attention as oa
from oracle import layout as ol


def oracle_setup(w: wl.Workload, free_order=None):
    """Oracle-side block tables and a pool filled through them."""
    pool = ol.BlockPool(w.num_blocks, w.free_order if free_order is None else free_order)
    if w.num_roots:
        lay = ol.build_layout_tree(pool, w.geometry.block_size, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt,
                                   w.req_model, w.suffix_len)
        data = wl.fill_pool(w, lay.prefix_blk_indptr, lay.prefix_blk, lay.suffix_blk_indptr, lay.suffix_blk,
                            lay.root_blk_indptr, lay.root_blk)
    else:
        lay = ol.build_layout(pool, w.geometry.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        data = wl.fill_pool(w, lay.prefix_blk_indptr, lay.prefix_blk, lay.suffix_blk_indptr, lay.suffix_blk)
    return pool, lay, data


def oracle_decode(w: wl.Workload, lay, data, requests=None):
    g = w.geometry
    return oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay, requests)


def errors(got: np.ndarray, ref: np.ndarray):
    """(max-abs, relative RMS over the whole tensor, worst per-request relative RMS)."""
    got = np.asarray(got, np.float64)
    diff = got - ref
    max_abs = float(np.abs(diff).max()) if diff.size else 0.0
    rel_rms = float(np.sqrt((diff ** 2).sum() / max((ref ** 2).sum(), 1e-300)))
    per_req = np.sqrt((diff ** 2).reshape(diff.shape[0], -1).sum(1) / np.maximum((ref ** 2).reshape(ref.shape[0], -1).sum(1), 1e-300))
    return max_abs, rel_rms, float(per_req.max()) if per_req.size else 0.0
