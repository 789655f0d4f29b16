"""Staging of cold KV blocks in host memory and their reload (oracle side, test infrastructure).

What is modelled (Appendix B.2, "KV transfer and staging at high concurrency"): when the decode side's resident KV
footprint exceeds the GPU's capacity, the caches of sessions that are not scheduled are staged in CPU memory and
reloaded when their sessions are scheduled again; the alternatives the paper names are admission control and
per-session reservation of KV blocks.  The paper describes the mechanism of its serving stack only in these words;
the readings taken here:

  * the unit is a batch layout (the sessions that were admitted together): *parking* it copies every block it holds
    to a staging area and drops its references, so the blocks return to the pool; *resuming* it takes blocks again
    (by the ordinary policy, from whatever the free list holds then -- in general other physical blocks) and copies
    the staged contents back;
  * a staged image is the layout's blocks in table order -- prefix blocks, suffix blocks, root blocks, the order of
    the concatenated block array -- each block whole (every KV head, K and V, all slots, used or not), followed for
    e4m3 pools by the blocks' scales in the same order; bits are copied, nothing is converted;
  * admission: a batch fits if the number of blocks it needs (the Eq. 9 count) does not exceed the free list.
"""
from __future__ import annotations

import numpy as np

from . import layout as ol


def table_order(lay) -> np.ndarray:
    """The layout's physical block ids in staging order."""
    parts = [lay.prefix_blk, lay.suffix_blk]
    if lay.root_blk is not None:
        parts.append(lay.root_blk)
    return np.concatenate(parts).astype(np.int64)


def stage_out(kv: np.ndarray, scales, lay):
    """(staged blocks [E, Hkv, 2, B, d], staged scales [E, Hkv, 2] or None): copies, in table order."""
    ids = table_order(lay)
    return kv[ids].copy(), (None if scales is None else scales[ids].copy())


def stage_in(kv: np.ndarray, scales, lay, staged_kv: np.ndarray, staged_scales) -> None:
    """Writes a staged image into the blocks the (resumed) layout holds now."""
    ids = table_order(lay)
    if staged_kv.shape[0] != len(ids):
        raise ol.LayoutError("staged image does not match the layout")
    kv[ids] = staged_kv
    if scales is not None:
        scales[ids] = staged_scales


def blocks_needed(block_size: int, prefix_len, suffix_len, root_len=()) -> int:
    """Blocks a batch occupies: every shared segment once, every private segment once (Efficiency Analysis, Eq. 9)."""
    total = 0
    for lens in (root_len, prefix_len, suffix_len):
        total += int(sum(-(-int(x) // block_size) for x in lens))
    return total


def park_layout(pool: ol.BlockPool, lay) -> None:
    """Drop the layout's references (its blocks rejoin the free list as in a release: those that reach zero are
    appended in ascending id) but keep its logical structure, so that it can be resumed."""
    if getattr(lay, "parked", False):
        raise ol.LayoutError("layout is already parked")
    ol.release_layout(pool, lay)
    lay.released = False
    lay.parked = True


def resume_layout(pool: ol.BlockPool, lay) -> None:
    """Take blocks again for a parked layout, by the ordinary policy (roots, prompts, requests, from the head of the
    free list as it is now).  Raises OutOfBlocks, leaving pool and layout as they were, if the batch does not fit."""
    if not getattr(lay, "parked", False):
        raise ol.LayoutError("layout is not parked")
    if lay.root_len is not None:
        fresh = ol.build_layout_tree(pool, lay.block_size, lay.root_len, lay.prompt_root, lay.prefix_len, lay.req_prompt,
                                     lay.req_model, lay.suffix_len)
    else:
        fresh = ol.build_layout(pool, lay.block_size, lay.prefix_len, lay.req_prompt, lay.req_model, lay.suffix_len)
    for name in ("prefix_blk_indptr", "prefix_blk", "suffix_blk_indptr", "suffix_blk", "root_blk_indptr", "root_blk"):
        setattr(lay, name, getattr(fresh, name))
    lay.parked = False
