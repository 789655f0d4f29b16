"""Pins for the oracle's block-table policy: a hand-worked instance and the Eq. 8 / Eq. 9 invariants."""
import json
import os

import numpy as np
import pytest

import workloads as wl
from oracle import layout as ol

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layout_small.json")


def test_hand_worked_instance():
    g = json.load(open(GOLDEN))
    pool = ol.BlockPool(g["num_blocks"], g["free_order"])
    lay = ol.build_layout(pool, g["block_size"], g["prefix_len"], g["req_prompt"], g["req_model"], g["suffix_len"])
    e = g["expect"]
    for name in ("prefix_blk_indptr", "prefix_blk", "group_indptr", "group_req", "suffix_blk_indptr", "suffix_blk"):
        assert getattr(lay, name).tolist() == e[name], name
    assert pool.refcount.tolist() == e["refcount"]
    assert list(pool.free) == e["free_after_build"]
    used = int((pool.refcount > 0).sum())
    assert used == e["blocks_used_eq9"]
    # an unshared layout (Eq. 8) would hold every request's full sequence
    b = g["block_size"]
    unshared = sum(-(-g["prefix_len"][p] // b) + -(-s // b) for p, s in zip(g["req_prompt"], g["suffix_len"]))
    assert unshared == e["blocks_used_unshared_eq8"]
    ol.release_layout(pool, lay)
    assert pool.refcount.tolist() == [0] * 8 and list(pool.free) == e["free_after_release"]
    with pytest.raises(ol.RefcountError):
        ol.release_layout(pool, lay)


@pytest.mark.parametrize("name", ["tiny", "b8", "mixed"])
def test_eq9_invariants(name):
    w = wl.named_workload(name)
    b = w.geometry.block_size
    pool = ol.BlockPool(w.num_blocks, w.free_order)
    lay = ol.build_layout(pool, b, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    nb_p = -(-w.prefix_len.astype(np.int64) // b)
    nb_s = -(-w.suffix_len.astype(np.int64) // b)
    # blocks in use = sum ceil(Lp/B) + sum ceil(Ls/B): the shared term does not grow with the number of models
    assert int((pool.refcount > 0).sum()) == int(nb_p.sum() + nb_s.sum())
    assert np.array_equal(np.diff(lay.prefix_blk_indptr), nb_p) and np.array_equal(np.diff(lay.suffix_blk_indptr), nb_s)
    k = np.bincount(w.req_prompt, minlength=w.num_prompts)
    for p in range(w.num_prompts):
        ids = lay.prefix_blk[lay.prefix_blk_indptr[p]:lay.prefix_blk_indptr[p + 1]]
        assert np.all(pool.refcount[ids] == k[p])
        reqs = lay.group_req[lay.group_indptr[p]:lay.group_indptr[p + 1]]
        assert np.all(w.req_prompt[reqs] == p) and np.all(np.diff(reqs) > 0)
    assert np.all(pool.refcount[lay.suffix_blk] == 1)
    everything = np.concatenate([lay.prefix_blk, lay.suffix_blk])
    assert len(np.unique(everything)) == len(everything)          # no block serves two owners
    # allocation follows the free order
    assert np.array_equal(everything, w.free_order[:len(everything)])
    ol.release_layout(pool, lay)
    assert not pool.refcount.any() and sorted(pool.free) == list(range(w.num_blocks))


def test_two_batches_share_one_pool_and_release_independently():
    pool = ol.BlockPool(10)
    a = ol.build_layout(pool, 4, [8], [0, 0], [0, 1], [4, 4])      # 2 + 1 + 1
    bb = ol.build_layout(pool, 4, [4], [0], [0], [2])              # 1 + 1
    assert a.prefix_blk.tolist() == [0, 1] and bb.prefix_blk.tolist() == [4] and bb.suffix_blk.tolist() == [5]
    ol.release_layout(pool, a)
    assert pool.refcount.tolist() == [0, 0, 0, 0, 1, 1, 0, 0, 0, 0]
    assert list(pool.free) == [6, 7, 8, 9, 0, 1, 2, 3]
    ol.release_layout(pool, bb)
    assert not pool.refcount.any()


def test_exhaustion_leaves_pool_untouched_and_bad_input_is_rejected():
    pool = ol.BlockPool(3, [2, 0, 1])
    with pytest.raises(ol.OutOfBlocks):
        ol.build_layout(pool, 16, [33], [0], [0], [1])
    assert list(pool.free) == [2, 0, 1] and not pool.refcount.any()
    with pytest.raises(ol.LayoutError):
        ol.build_layout(pool, 16, [16], [0, 0], [1, 1], [1, 1])    # duplicate (prompt, model)
    with pytest.raises(ol.LayoutError):
        ol.build_layout(pool, 16, [16, 16], [0], [0], [1])         # prompt nobody decodes on
    with pytest.raises(ol.LayoutError):
        ol.build_layout(pool, 16, [16], [1], [0], [1])             # unknown prompt
    with pytest.raises(ol.LayoutError):
        ol.BlockPool(3, [0, 0, 1])


def test_adopted_blocks_hand_worked():
    """Pool of 10 (B = 4, ascending).  Layout A: prompt of 10 tokens (blocks 0 1 2) for two models with suffixes 2 and 5
    (blocks 3 and 4 5).  Layout C continues the context to 14 tokens for three requests: it adopts A's two full blocks
    0 1 (tokens 0..7), takes 6 7 for tokens 8..13 and 8 for its one non-empty suffix.  Blocks 0 1 are then referenced
    2 + 3 times; releasing A frees 2 3 4 5 only; releasing C frees the rest."""
    pool = ol.BlockPool(10)
    a = ol.build_layout(pool, 4, [10], [0, 0], [0, 1], [2, 5])
    assert a.prefix_blk.tolist() == [0, 1, 2] and a.suffix_blk.tolist() == [3, 4, 5]
    c = ol.build_layout(pool, 4, [14], [0, 0, 0], [0, 1, 2], [0, 3, 0], adopt=[[0, 1]])
    assert c.prefix_blk.tolist() == [0, 1, 6, 7] and c.suffix_blk.tolist() == [8]
    assert pool.refcount.tolist() == [5, 5, 2, 1, 1, 1, 3, 3, 1, 0] and list(pool.free) == [9]
    ol.release_layout(pool, a)
    assert pool.refcount.tolist() == [3, 3, 0, 0, 0, 0, 3, 3, 1, 0] and list(pool.free) == [9, 2, 3, 4, 5]
    ol.release_layout(pool, c)
    assert not pool.refcount.any() and list(pool.free) == [9, 2, 3, 4, 5, 0, 1, 6, 7, 8]


def test_adoption_rules():
    pool = ol.BlockPool(6)
    a = ol.build_layout(pool, 4, [9], [0], [0], [0])                       # blocks 0 1 2, the last one partial
    with pytest.raises(ol.LayoutError):
        ol.build_layout(pool, 4, [11], [0], [0], [0], adopt=[[0, 1, 2]])   # only full blocks: 3 * 4 > 11
    with pytest.raises(ol.LayoutError):
        ol.build_layout(pool, 4, [12], [0], [0], [0], adopt=[[0, 5]])      # block 5 is not alive
    with pytest.raises(ol.LayoutError):
        ol.build_layout(pool, 4, [12, 12], [0, 1], [0, 0], [0, 0], adopt=[[0], [0]])   # named twice
    with pytest.raises(ol.OutOfBlocks):
        ol.build_layout(pool, 4, [24], [0], [0], [0], adopt=[[0, 1]])      # needs 4 more, 3 free
    assert pool.refcount.tolist() == [1, 1, 1, 0, 0, 0] and list(pool.free) == [3, 4, 5]
    # adopting nothing is the ordinary layout
    b = ol.build_layout(pool, 4, [4], [0], [0], [0], adopt=[[]])
    assert b.prefix_blk.tolist() == [3]
    ol.release_layout(pool, a)
    ol.release_layout(pool, b)
    assert not pool.refcount.any()


def test_adopting_layout_reads_the_same_context():
    """A continued context gives the old tokens the same K/V: attention of the continuing layout over [old ; new]
    equals the oracle on a fresh layout holding the concatenated context."""
    from oracle import attention as oa
    from helpers import oracle_setup
    geo = wl.Geometry(4, 2, 8, 4, "f32", "f32")
    old = wl.make_workload("old", geo, 2, [10], [[0, 1]], [2, 5], pool_factor=3.0, seed=13)
    pool, a, data = oracle_setup(old)
    n_full = 10 // 4
    new = wl.make_workload("new", geo, 3, [14], [[0, 1, 2]], [0, 3, 0], seed=14)
    c = ol.build_layout(pool, 4, new.prefix_len, new.req_prompt, new.req_model, new.suffix_len,
                        adopt=[a.prefix_blk[:n_full].tolist()])
    assert c.prefix_blk[:n_full].tolist() == a.prefix_blk[:n_full].tolist()
    # context of the new layout: the old prompt's first 8 tokens (already in the pool), then 6 new ones
    old_seg, new_seg = old.prefix_kv(0), new.prefix_kv(0)
    k_ctx = np.concatenate([old_seg.k[:8], new_seg.k[8:14]])
    v_ctx = np.concatenate([old_seg.v[:8], new_seg.v[8:14]])
    for j in range(8, 14):
        blk = c.prefix_blk[j // 4]
        data.kv[blk, :, 0, j % 4] = k_ctx[j]
        data.kv[blk, :, 1, j % 4] = v_ctx[j]
    for r in range(new.num_requests):
        seg = new.suffix_kv(r)
        ids = c.suffix_blk[c.suffix_blk_indptr[r]:c.suffix_blk_indptr[r + 1]]
        for j in range(seg.k.shape[0]):
            data.kv[ids[j // 4], :, 0, j % 4] = seg.k[j]
            data.kv[ids[j // 4], :, 1, j % 4] = seg.v[j]
    o, lse = oa.decode_attention(new.q_bits(), "f32", data.kv, None, "f32", c)
    q = oa.widen(new.q_bits(), "f32")
    for r in range(new.num_requests):
        seg = new.suffix_kv(r)
        ro, rl = oa.attention_state(q[r], np.concatenate([k_ctx, seg.k]).astype(np.float64),
                                    np.concatenate([v_ctx, seg.v]).astype(np.float64))
        assert np.abs(o[r] - ro).max() < 1e-13 and np.abs(lse[r] - rl).max() < 1e-13
    # the old layout still reads its own context, untouched
    o_old, _ = oa.decode_attention(old.q_bits(), "f32", data.kv, None, "f32", a)
    fresh_pool, fresh, fresh_data = oracle_setup(old)
    o_ref, _ = oa.decode_attention(old.q_bits(), "f32", fresh_data.kv, None, "f32", fresh)
    assert np.array_equal(o_old, o_ref)
