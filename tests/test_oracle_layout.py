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
