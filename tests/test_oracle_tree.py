"""Pins for the oracle's third sharing level (a context several prompts begin with): a hand-worked table, block-count
and refcount invariants, brute-force dense attention, and identity with the two-level oracle on the flattened batch."""
import json
import os

import numpy as np
import pytest

import workloads as wl
from oracle import attention as oa
from oracle import layout as ol
from helpers import oracle_setup

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layout_tree_small.json")
TREE_KEYS = ("root_blk_indptr", "root_blk", "root_group_indptr", "root_group_req", "prefix_blk_indptr", "prefix_blk",
             "group_indptr", "group_req", "suffix_blk_indptr", "suffix_blk")


def _build(g):
    pool = ol.BlockPool(g["num_blocks"], g["free_order"])
    lay = ol.build_layout_tree(pool, g["block_size"], g["root_len"], g["prompt_root"], g["prefix_len"], g["req_prompt"],
                               g["req_model"], g["suffix_len"])
    return pool, lay


def test_hand_worked_instance():
    g = json.load(open(GOLDEN))
    pool, lay = _build(g)
    e = g["expect"]
    for name in TREE_KEYS:
        assert getattr(lay, name).tolist() == e[name], name
    assert pool.refcount.tolist() == e["refcount"] and list(pool.free) == e["free_after_build"]
    assert int((pool.refcount > 0).sum()) == e["blocks_used"]
    ol.release_layout(pool, lay)
    assert not pool.refcount.any() and list(pool.free) == e["free_after_release"]
    with pytest.raises(ol.RefcountError):
        ol.release_layout(pool, lay)


@pytest.mark.parametrize("name", ["tree_tiny", "tree_b8"])
def test_block_count_and_refcounts(name):
    """Blocks in use = sum over roots + prompts + requests of ceil(len / B): neither shared term grows with the number
    of sessions or models below it."""
    w = wl.named_tree_workload(name)
    b = w.geometry.block_size
    pool = ol.BlockPool(w.num_blocks, w.free_order)
    lay = ol.build_layout_tree(pool, b, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    nb = [-(-x.astype(np.int64) // b) for x in (w.root_len, w.prefix_len, w.suffix_len)]
    assert int((pool.refcount > 0).sum()) == int(sum(x.sum() for x in nb))
    assert np.array_equal(np.diff(lay.root_blk_indptr), nb[0])
    for t in range(w.num_roots):
        below = [r for r in range(w.num_requests) if w.prompt_root[w.req_prompt[r]] == t]
        assert lay.root_group_req[lay.root_group_indptr[t]:lay.root_group_indptr[t + 1]].tolist() == below
        assert np.all(pool.refcount[lay.root_blk[lay.root_blk_indptr[t]:lay.root_blk_indptr[t + 1]]] == len(below))
    everything = np.concatenate([lay.root_blk, lay.prefix_blk, lay.suffix_blk])
    assert len(np.unique(everything)) == len(everything)
    assert np.array_equal(everything, w.free_order[:len(everything)])        # roots first, in free-list order
    ol.release_layout(pool, lay)
    assert not pool.refcount.any() and sorted(pool.free) == list(range(w.num_blocks))


def test_no_roots_is_the_two_level_table_and_bad_input_is_rejected():
    w = wl.named_workload("tiny")
    b = w.geometry.block_size
    p1, p2 = ol.BlockPool(w.num_blocks, w.free_order), ol.BlockPool(w.num_blocks, w.free_order)
    flat = ol.build_layout(p1, b, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    tree = ol.build_layout_tree(p2, b, [], [-1] * w.num_prompts, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    for name in TREE_KEYS[4:]:
        assert np.array_equal(getattr(flat, name), getattr(tree, name))
    assert np.array_equal(p1.refcount, p2.refcount) and len(tree.root_blk) == 0
    pool = ol.BlockPool(4, [3, 1, 0, 2])
    with pytest.raises(ol.OutOfBlocks):
        ol.build_layout_tree(pool, 4, [9], [0], [4], [0], [0], [1])          # needs 3 + 1 + 1
    with pytest.raises(ol.LayoutError):
        ol.build_layout_tree(pool, 4, [4], [1], [4], [0], [0], [1])          # unknown root
    with pytest.raises(ol.LayoutError):
        ol.build_layout_tree(pool, 4, [4, 4], [0], [4], [0], [0], [1])       # root nobody begins with
    with pytest.raises(ol.LayoutError):
        ol.build_layout_tree(pool, 4, [4], [0], [4], [0, 0], [1, 1], [1, 1])  # duplicate request: root blocks go back
    assert list(pool.free) == [3, 1, 0, 2] and not pool.refcount.any()


def _dense(q, k, v, group):
    """Attention of one request written out in loops: q [Hq, d], k / v [L, Hkv, d] -> o [Hq, d], lse [Hq]."""
    hq, d = q.shape
    o, lse = np.zeros((hq, d)), np.zeros(hq)
    for h in range(hq):
        s = [sum(q[h, c] * k[j, h // group, c] for c in range(d)) / np.sqrt(d) for j in range(k.shape[0])]
        m = max(s)
        den = sum(np.exp(x - m) for x in s)
        lse[h] = m + np.log(den)
        for j, x in enumerate(s):
            o[h] += np.exp(x - m) / den * v[j, h // group]
    return o, lse


def test_brute_force_dense_attention_over_root_prefix_suffix():
    geo = wl.Geometry(4, 2, 8, 4, "f32", "f32")
    w = wl.make_tree_workload("t", geo, 2, [6, 3], [0, -1, 1, 0], [5, 7, 0, 2], [[0, 1], [1], [0], [0, 1]],
                              [1, 0, 4, 6, 0, 3], pool_factor=1.4, seed=11)
    _, lay, data = oracle_setup(w)
    o, lse = oa.decode_attention(w.q_bits(), "f32", data.kv, None, "f32", lay)
    q = w.q_bits().astype(np.float64)
    for r in range(w.num_requests):
        p = int(w.req_prompt[r])
        segs = ([w.root_kv(int(w.prompt_root[p]))] if w.prompt_root[p] >= 0 else []) + [w.prefix_kv(p), w.suffix_kv(r)]
        k = np.concatenate([s.k for s in segs]).astype(np.float64)
        v = np.concatenate([s.v for s in segs]).astype(np.float64)
        ro, rl = _dense(q[r], k, v, geo.group)
        assert np.abs(o[r] - ro).max() < 1e-12 and np.abs(lse[r] - rl).max() < 1e-12


def test_same_result_as_the_two_level_oracle_on_the_flattened_batch():
    """Storing the common context once must not change what is computed: a two-level batch in which every prompt's
    prefix is the concatenation root ++ own part, filled with the same values, gives bitwise the same outputs."""
    w = wl.named_tree_workload("tree_tiny", seed=5)
    g = w.geometry
    _, lay, data = oracle_setup(w)
    o, lse = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, None, g.kv_dtype, lay)
    flat_len = [int(w.prefix_len[p]) + (int(w.root_len[w.prompt_root[p]]) if w.prompt_root[p] >= 0 else 0)
                for p in range(w.num_prompts)]
    b = g.block_size
    need = sum(-(-x // b) for x in flat_len) + int((-(-w.suffix_len.astype(np.int64) // b)).sum())
    pool = ol.BlockPool(need)
    flat = ol.build_layout(pool, b, flat_len, w.req_prompt, w.req_model, w.suffix_len)
    kv = np.full((need, g.num_kv_heads, 2, b, g.head_dim), np.nan, np.float32)

    def put(ids, k, v):
        for j in range(k.shape[0]):
            kv[ids[j // b], :, 0, j % b] = k[j]
            kv[ids[j // b], :, 1, j % b] = v[j]
    for p in range(w.num_prompts):
        segs = ([w.root_kv(int(w.prompt_root[p]))] if w.prompt_root[p] >= 0 else []) + [w.prefix_kv(p)]
        put(flat.prefix_blk[flat.prefix_blk_indptr[p]:flat.prefix_blk_indptr[p + 1]],
            np.concatenate([s.k for s in segs]), np.concatenate([s.v for s in segs]))
    for r in range(w.num_requests):
        seg = w.suffix_kv(r)
        put(flat.suffix_blk[flat.suffix_blk_indptr[r]:flat.suffix_blk_indptr[r + 1]], seg.k, seg.v)
    fo, flse = oa.decode_attention(w.q_bits(), g.q_dtype, kv, None, g.kv_dtype, flat)
    assert np.array_equal(o, fo) and np.array_equal(lse, flse)


def test_root_is_shared_only_by_the_prompts_below_it():
    w = wl.named_tree_workload("tree_tiny", seed=2)
    g = w.geometry
    _, lay, data = oracle_setup(w)
    a, _ = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, None, g.kv_dtype, lay)
    kv = data.kv.copy()
    kv[lay.root_blk[0], :, 1, 0] += 1.0                       # touch one stored root token
    c, _ = oa.decode_attention(w.q_bits(), g.q_dtype, kv, None, g.kv_dtype, lay)
    below = [r for r in range(w.num_requests) if w.prompt_root[w.req_prompt[r]] == 0]
    others = [r for r in range(w.num_requests) if r not in below]
    assert others and np.array_equal(a[others], c[others])
    assert all(not np.array_equal(a[r], c[r]) for r in below)
