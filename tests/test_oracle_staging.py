"""Pins for the oracle's staging of cold KV blocks: a hand-worked park / resume sequence, the block count used for
admission, and bit-for-bit read-back after the freed blocks were reused and overwritten."""
import numpy as np
import pytest

import workloads as wl
from oracle import attention as oa
from oracle import layout as ol
from oracle import staging as st
from helpers import oracle_setup


def test_hand_worked_park_and_resume():
    """Pool of 8 blocks (B = 4), free order 3 1 7 0 2 6 5 4.  Batch A: prefix 6 tokens shared by two models, suffixes 1
    and 5 -> prefix blocks [3, 1], suffix blocks [7] and [0, 2]; free: 6 5 4.  Parking A returns 0 1 2 3 7 (ascending)
    to the tail: free 6 5 4 0 1 2 3 7.  Batch B (prefix 4, one model, suffix 9) then takes [6] and [5, 4, 0]; free
    1 2 3 7.  Resuming A would need 5 blocks: it does not fit and nothing changes.  After B is released (free
    1 2 3 7 0 4 5 6), A resumes into prefix [1, 2], suffixes [3] and [7, 0]; free 4 5 6."""
    pool = ol.BlockPool(8, [3, 1, 7, 0, 2, 6, 5, 4])
    a = ol.build_layout(pool, 4, [6], [0, 0], [0, 1], [1, 5])
    assert a.prefix_blk.tolist() == [3, 1] and a.suffix_blk.tolist() == [7, 0, 2] and list(pool.free) == [6, 5, 4]
    assert st.table_order(a).tolist() == [3, 1, 7, 0, 2]
    st.park_layout(pool, a)
    assert list(pool.free) == [6, 5, 4, 0, 1, 2, 3, 7] and not pool.refcount.any()
    with pytest.raises(ol.LayoutError):
        st.park_layout(pool, a)
    b = ol.build_layout(pool, 4, [4], [0], [0], [9])
    assert b.prefix_blk.tolist() == [6] and b.suffix_blk.tolist() == [5, 4, 0] and list(pool.free) == [1, 2, 3, 7]
    with pytest.raises(ol.OutOfBlocks):
        st.resume_layout(pool, a)
    assert list(pool.free) == [1, 2, 3, 7] and a.parked
    ol.release_layout(pool, b)
    assert list(pool.free) == [1, 2, 3, 7, 0, 4, 5, 6]
    st.resume_layout(pool, a)
    assert a.prefix_blk.tolist() == [1, 2] and a.suffix_blk.tolist() == [3, 7, 0] and list(pool.free) == [4, 5, 6]
    assert pool.refcount.tolist() == [1, 2, 2, 1, 0, 0, 0, 1]
    with pytest.raises(ol.LayoutError):
        st.resume_layout(pool, a)
    ol.release_layout(pool, a)
    assert not pool.refcount.any()


@pytest.mark.parametrize("name", ["tiny", "b8", "tree_tiny"])
def test_blocks_needed_is_the_number_of_blocks_a_layout_takes(name):
    w = wl.named_tree_workload(name) if name.startswith("tree") else wl.named_workload(name)
    pool, lay, _ = oracle_setup(w)
    used = int((pool.refcount > 0).sum())
    assert st.blocks_needed(w.geometry.block_size, w.prefix_len, w.suffix_len, w.root_len) == used == len(st.table_order(lay))
    assert used == w.blocks_needed()


@pytest.mark.parametrize("spec", [("f32", False), ("bf16", True), ("fp8_e4m3", False), ("fp8_e4m3", True)])
def test_parked_batch_reads_back_bit_for_bit_after_its_blocks_were_reused(spec):
    kv_dtype, tree = spec
    geo = wl.Geometry(4, 2, 16, 4, "f32" if kv_dtype == "f32" else "bf16", kv_dtype)
    if tree:
        w = wl.make_tree_workload("s", geo, 2, [6], [0, -1, 0], [5, 3, 0], [[0, 1], [0], [1]], [1, 0, 4, 6],
                                  pool_factor=1.5, seed=7)
    else:
        w = wl.make_workload("s", geo, 2, [9, 3], [[0, 1], [1]], [2, 0, 7], pool_factor=1.5, seed=7)
    pool, lay, data = oracle_setup(w)
    g = w.geometry
    before = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay)
    image, image_scales = st.stage_out(data.kv, data.scales, lay)
    assert image.shape[0] == st.blocks_needed(g.block_size, w.prefix_len, w.suffix_len, w.root_len)
    old_ids = st.table_order(lay).copy()
    st.park_layout(pool, lay)
    # somebody else uses the pool meanwhile: every block is overwritten, and the free list is rotated
    data.kv[:] = wl.generate.POISON[kv_dtype]
    if data.scales is not None:
        data.scales[:] = np.nan
    pool.free.rotate(3)
    st.resume_layout(pool, lay)
    assert not np.array_equal(st.table_order(lay), old_ids)              # other physical blocks this time
    st.stage_in(data.kv, data.scales, lay, image, image_scales)
    after = oa.decode_attention(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay)
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    with pytest.raises(ol.LayoutError):
        st.stage_in(data.kv, data.scales, lay, image[:-1], image_scales)
