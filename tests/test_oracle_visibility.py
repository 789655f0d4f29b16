"""Pins for per-request visible prefix lengths (causal chunk prefill against the shared cache)."""
import numpy as np
import torch

import workloads as wl
from oracle import attention as oa
from oracle import layout as ol
from helpers import oracle_setup


def _chunk_workload(cached, chunk, kv_dtype="f32", seed=0, hq=4, hkv=2, d=16, bsz=16):
    """One prompt whose prefix holds `cached` old tokens followed by `chunk` new ones; every new token is a
    query row on that prompt (model index = position in the chunk), no private suffix."""
    geo = wl.Geometry(hq, hkv, d, bsz, "f32" if kv_dtype == "f32" else "bf16", kv_dtype)
    w = wl.make_workload("chunk", geo, chunk, [cached + chunk], [list(range(chunk))], [0] * chunk, seed=seed)
    visible = np.array([cached + i + 1 for i in range(chunk)], np.int32)
    return w, visible


def test_full_visibility_is_the_unmasked_result_and_zero_sees_nothing():
    w = wl.named_workload("tiny")
    pool, lay, data = oracle_setup(w)
    g = w.geometry
    a = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay)
    b = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay, None, lay.prefix_len[lay.req_prompt])
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # nothing visible, no suffix -> the empty state
    w2, _ = _chunk_workload(5, 3)
    _, lay2, data2 = oracle_setup(w2)
    o, lse = oa.decode_attention(w2.q_bits(), "f32", data2.kv, None, "f32", lay2, None, np.zeros(3, np.int32))
    assert not o.any() and np.isneginf(lse).all()


def test_causal_chunk_equals_library_sdpa_with_a_mask():
    cached, chunk = 21, 19
    w, visible = _chunk_workload(cached, chunk)
    g = w.geometry
    _, lay, data = oracle_setup(w)
    o, _ = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay, None, visible)
    seg = w.prefix_kv(0)
    q = torch.from_numpy(w.q_bits().astype(np.float64)).permute(1, 0, 2)                 # [Hq, chunk, d]
    k = torch.from_numpy(seg.k.astype(np.float64)).permute(1, 0, 2).repeat_interleave(g.group, 0)   # [Hq, L, d]
    v = torch.from_numpy(seg.v.astype(np.float64)).permute(1, 0, 2).repeat_interleave(g.group, 0)
    cols = torch.arange(cached + chunk)[None, :]
    mask = cols < torch.from_numpy(visible.astype(np.int64))[:, None]                    # row i sees columns < visible_i
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask).permute(1, 0, 2).numpy()
    assert np.abs(o - ref).max() < 1e-10


def test_causal_chunk_equals_token_by_token_decoding():
    """Prefilling a chunk at once must give each token what it would get if the tokens were appended one at a
    time: token i alone against a cache of cached + i + 1 tokens, built as a layout of its own."""
    cached, chunk = 13, 9
    w, visible = _chunk_workload(cached, chunk, kv_dtype="bf16", seed=3)
    g = w.geometry
    _, lay, data = oracle_setup(w)
    o, lse = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay, None, visible)
    seg = w.prefix_kv(0)
    q = oa.widen(w.q_bits(), g.q_dtype)
    for i in range(chunk):
        n = cached + i + 1
        pool = ol.BlockPool(8, [3, 1, 7, 0, 2, 6, 5, 4])
        lay_i = ol.build_layout(pool, g.block_size, [n], [0], [0], [0])
        kv = np.zeros((8, g.num_kv_heads, 2, g.block_size, g.head_dim), np.uint16)
        for j in range(n):
            blk = lay_i.prefix_blk[j // g.block_size]
            kv[blk, :, 0, j % g.block_size] = seg.k[j]
            kv[blk, :, 1, j % g.block_size] = seg.v[j]
        k_i, v_i = oa.request_kv(kv, None, g.kv_dtype, lay_i, 0)
        o_i, lse_i = oa.attention_state(q[i], k_i, v_i)
        assert np.allclose(o[i], o_i, atol=1e-13) and np.allclose(lse[i], lse_i, atol=1e-13)


def test_rows_are_independent_of_each_other():
    """Changing what one row may see leaves every other row bitwise unchanged."""
    w, visible = _chunk_workload(8, 6)
    g = w.geometry
    _, lay, data = oracle_setup(w)
    a, _ = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, None, g.kv_dtype, lay, None, visible)
    other = visible.copy()
    other[2] = 3
    b, _ = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, None, g.kv_dtype, lay, None, other)
    keep = [0, 1, 3, 4, 5]
    assert np.array_equal(a[keep], b[keep]) and not np.array_equal(a[2], b[2])
