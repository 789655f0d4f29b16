"""Refcounted block table (two segments, optionally a third shared level above), reference policy (oracle side,
test infrastructure).

Problem statement followed: a pool of fixed-size cached KV blocks (Background,
"Multi-Model Inference and Prefix Caching"); every decode module starts from
the *same* base cache, C <- C_base (Method, Eq. 6), so a prompt's prefix blocks
are stored once and referenced by all its requests, while each request owns
the blocks of its model-specific segment (Efficiency Analysis, Eq. 9:
Mem = O(L_shared + N * L_unique)).

Canonical policy (fixed so that two builders can be compared bit for bit):
  * the pool's free list starts in the caller-given order;
  * prompts are served in ascending index, each taking ceil(Lp/B) blocks from the
    head of the free list in logical order; then requests in ascending index,
    each taking ceil(Ls/B) private blocks (a private segment always starts in a
    fresh block; a partially filled last prefix block stays shared, read-only);
  * a prefix block's refcount is the number of requests on that prompt, a
    private block's is 1;
  * release drops those references; blocks that reach zero are appended to the
    free list in ascending block id;
  * a batch that does not fit leaves the pool untouched.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass

import numpy as np


class LayoutError(Exception):
    pass


class OutOfBlocks(LayoutError):
    pass


class RefcountError(LayoutError):
    pass


class BlockPool:
    def __init__(self, num_blocks: int, free_order=None):
        order = list(range(num_blocks)) if free_order is None else [int(x) for x in free_order]
        if sorted(order) != list(range(num_blocks)):
            raise LayoutError("free_order must be a permutation of the pool")
        self.num_blocks = num_blocks
        self.free = deque(order)
        self.refcount = np.zeros(num_blocks, dtype=np.int32)


@dataclass
class Layout:
    block_size: int
    prefix_len: np.ndarray          # [P]
    suffix_len: np.ndarray          # [R]
    req_prompt: np.ndarray          # [R]
    req_model: np.ndarray           # [R]
    prefix_blk_indptr: np.ndarray   # [P+1]
    prefix_blk: np.ndarray
    group_indptr: np.ndarray        # [P+1]  prompt -> its requests
    group_req: np.ndarray           # [R]
    suffix_blk_indptr: np.ndarray   # [R+1]
    suffix_blk: np.ndarray
    released: bool = False
    # third level (build_layout_tree): contexts several prompts have in common
    root_len: np.ndarray = None            # [T]
    prompt_root: np.ndarray = None         # [P], -1 = the prompt has no root
    root_blk_indptr: np.ndarray = None     # [T+1]
    root_blk: np.ndarray = None
    root_group_indptr: np.ndarray = None   # [T+1]  root -> the requests of all its prompts, ascending
    root_group_req: np.ndarray = None


def build_layout(pool: BlockPool, block_size: int, prefix_len, req_prompt, req_model, suffix_len, adopt=None) -> Layout:
    """adopt (optional): per prompt, the physical ids of blocks another layout already holds that contain the
    beginning of this prompt's prefix -- the cached context a later step continues from (System Design: prefix-aware
    routing keeps a context's cache where it is, "enabling incremental cache extension instead of recomputing the
    prefix from scratch"; execution pipeline: X(i) = [X(i-1); Y(i)]).  Only full blocks are adopted: the n adopted
    blocks of prompt p are the prompt's tokens [0, n * B), n * B <= Lp; each gains one reference per request on the
    prompt, exactly like a block taken from the free list, so it stays alive until the last layout that references
    it is released.  The remaining ceil(Lp/B) - n blocks come from the free list as usual."""
    prefix_len = np.asarray(prefix_len, dtype=np.int64)
    suffix_len = np.asarray(suffix_len, dtype=np.int64)
    req_prompt = np.asarray(req_prompt, dtype=np.int64)
    req_model = np.asarray(req_model, dtype=np.int64)
    num_p, num_r = len(prefix_len), len(req_prompt)
    if block_size <= 0 or (prefix_len < 0).any() or (suffix_len < 0).any():
        raise LayoutError("negative length or bad block size")
    if len(req_model) != num_r or len(suffix_len) != num_r:
        raise LayoutError("request arrays differ in length")
    if num_r and (req_prompt.min() < 0 or req_prompt.max() >= num_p or req_model.min() < 0):
        raise LayoutError("request names an unknown prompt or model")
    if len({(int(p), int(m)) for p, m in zip(req_prompt, req_model)}) != num_r:
        raise LayoutError("duplicate (prompt, model) request")
    members = [[] for _ in range(num_p)]
    for r in range(num_r):
        members[int(req_prompt[r])].append(r)
    if any(len(m) == 0 for m in members):
        raise LayoutError("prompt without a request")

    nb_prefix = (prefix_len + block_size - 1) // block_size
    nb_suffix = (suffix_len + block_size - 1) // block_size
    adopted = [[] for _ in range(num_p)] if adopt is None else [[int(b) for b in a] for a in adopt]
    if len(adopted) != num_p:
        raise LayoutError("one list of adopted blocks per prompt")
    seen = set()
    for p in range(num_p):
        if len(adopted[p]) * block_size > prefix_len[p]:
            raise LayoutError("adopted blocks must be full blocks of the prompt's prefix")
        for blk in adopted[p]:
            if not 0 <= blk < pool.num_blocks or pool.refcount[blk] <= 0 or blk in seen:
                raise LayoutError("an adopted block must be alive and named once")
            seen.add(blk)
    needed = int(nb_prefix.sum() + nb_suffix.sum()) - sum(len(a) for a in adopted)
    if needed > len(pool.free):
        raise OutOfBlocks(f"need {needed} blocks, {len(pool.free)} free")

    prefix_indptr = np.zeros(num_p + 1, np.int32)
    prefix_blk = []
    for p in range(num_p):
        for i in range(int(nb_prefix[p])):
            blk = adopted[p][i] if i < len(adopted[p]) else pool.free.popleft()
            pool.refcount[blk] += len(members[p])
            prefix_blk.append(blk)
        prefix_indptr[p + 1] = len(prefix_blk)
    suffix_indptr = np.zeros(num_r + 1, np.int32)
    suffix_blk = []
    for r in range(num_r):
        for _ in range(int(nb_suffix[r])):
            blk = pool.free.popleft()
            pool.refcount[blk] += 1
            suffix_blk.append(blk)
        suffix_indptr[r + 1] = len(suffix_blk)
    group_indptr = np.zeros(num_p + 1, np.int32)
    group_req = []
    for p in range(num_p):
        group_req.extend(members[p])
        group_indptr[p + 1] = len(group_req)
    return Layout(block_size, prefix_len.astype(np.int32), suffix_len.astype(np.int32),
                  req_prompt.astype(np.int32), req_model.astype(np.int32),
                  prefix_indptr, np.asarray(prefix_blk, np.int32), group_indptr,
                  np.asarray(group_req, np.int32), suffix_indptr, np.asarray(suffix_blk, np.int32))


def build_layout_tree(pool: BlockPool, block_size: int, root_len, prompt_root, prefix_len, req_prompt, req_model,
                      suffix_len) -> Layout:
    """Three-level table: root -> prompt -> request.

    Several prompts may begin with the same context (Background, "Multi-Model Inference and Prefix Caching": a common
    system prompt or a shared document in front of each session's own history); that common part -- a *root* -- is
    stored once, like a prompt's prefix is stored once for its models (Eq. 9 applied one level up).  The cache of
    request r on prompt p with root t = prompt_root[p] is [root t ; prefix p ; suffix r]; prompt_root[p] = -1 means
    the prompt has no root.

    Policy: roots in ascending index take ceil(L/B) blocks each from the head of the free list, then prompts and
    requests exactly as build_layout does.  A root block's refcount is the number of requests below the root; a
    root's last block may be partially filled and stays shared and read-only; a prompt's own prefix starts in a
    fresh block.  A root no prompt names is an error; a batch that does not fit leaves the pool untouched.
    """
    root_len = np.asarray(root_len, dtype=np.int64)
    prompt_root = np.asarray(prompt_root, dtype=np.int64)
    prefix_arr = np.asarray(prefix_len, dtype=np.int64)
    suffix_arr = np.asarray(suffix_len, dtype=np.int64)
    req_prompt_arr = np.asarray(req_prompt, dtype=np.int64)
    num_t = len(root_len)
    if len(prompt_root) != len(prefix_arr) or (root_len < 0).any():
        raise LayoutError("one root index per prompt, root lengths >= 0")
    if len(prompt_root) and (prompt_root.min() < -1 or prompt_root.max() >= num_t):
        raise LayoutError("prompt names an unknown root")
    if len(req_prompt_arr) and (req_prompt_arr.min() < 0 or req_prompt_arr.max() >= len(prefix_arr)):
        raise LayoutError("request names an unknown prompt")
    below = [[] for _ in range(num_t)]
    for r, p in enumerate(req_prompt_arr):
        if prompt_root[p] >= 0:
            below[int(prompt_root[p])].append(r)
    for t in range(num_t):
        if not (prompt_root == t).any():
            raise LayoutError("root without a prompt")
    nb_root = (root_len + block_size - 1) // block_size
    needed = int(nb_root.sum() + ((prefix_arr + block_size - 1) // block_size).sum()
                 + ((suffix_arr + block_size - 1) // block_size).sum())
    if needed > len(pool.free):
        raise OutOfBlocks(f"need {needed} blocks, {len(pool.free)} free")
    taken = []
    root_indptr = np.zeros(num_t + 1, np.int32)
    for t in range(num_t):
        for _ in range(int(nb_root[t])):
            taken.append(pool.free.popleft())
        root_indptr[t + 1] = len(taken)
    try:
        lay = build_layout(pool, block_size, prefix_len, req_prompt, req_model, suffix_len)
    except LayoutError:
        pool.free.extendleft(reversed(taken))           # bad lower levels: hand the root blocks back, in order
        raise
    for t in range(num_t):
        pool.refcount[taken[root_indptr[t]:root_indptr[t + 1]]] += len(below[t])
    group_indptr = np.zeros(num_t + 1, np.int32)
    group = []
    for t in range(num_t):
        group.extend(below[t])
        group_indptr[t + 1] = len(group)
    lay.root_len = root_len.astype(np.int32)
    lay.prompt_root = prompt_root.astype(np.int32)
    lay.root_blk_indptr = root_indptr
    lay.root_blk = np.asarray(taken, np.int32)
    lay.root_group_indptr = group_indptr
    lay.root_group_req = np.asarray(group, np.int32)
    return lay


def release_layout(pool: BlockPool, lay: Layout) -> None:
    if lay.released:
        raise RefcountError("layout released twice")
    drop = np.zeros(pool.num_blocks, dtype=np.int64)
    if lay.root_len is not None:
        for t in range(len(lay.root_len)):
            k = int(lay.root_group_indptr[t + 1] - lay.root_group_indptr[t])
            for blk in lay.root_blk[lay.root_blk_indptr[t]:lay.root_blk_indptr[t + 1]]:
                drop[blk] += k
    for p in range(len(lay.prefix_len)):
        k = int(lay.group_indptr[p + 1] - lay.group_indptr[p])
        for blk in lay.prefix_blk[lay.prefix_blk_indptr[p]:lay.prefix_blk_indptr[p + 1]]:
            drop[blk] += k
    for blk in lay.suffix_blk:
        drop[blk] += 1
    if (pool.refcount < drop).any():
        raise RefcountError("refcount underflow")
    pool.refcount -= drop.astype(np.int32)
    for blk in np.nonzero((drop > 0) & (pool.refcount == 0))[0]:
        pool.free.append(int(blk))
    lay.released = True


def append_step(pool: BlockPool, lay: Layout, active=None) -> np.ndarray:
    """One decode step of cache growth (Method, Eq. 6: every step returns the new entries dC_t that are
    appended to the module's own cache; Background, Eq. 4: the concatenation).

    Each active request gains one token at logical position Ls_r of its private segment.  Requests are
    served in ascending index; a request whose Ls_r is a multiple of the block size (no private block yet,
    or the last one is full) first takes one block from the head of the free list, refcount 1, appended to
    its private list.  Shared prefix blocks are never written (they stay read-only, Eq. 9).  A step that
    does not fit leaves pool and layout untouched.

    Returns dest[R] int64: global slot index block * B + slot where the new token of request r is stored,
    -1 for inactive requests.
    """
    if lay.released:
        raise LayoutError("layout already released")
    num_r = len(lay.req_prompt)
    act = np.ones(num_r, bool) if active is None else np.asarray(active).astype(bool)
    if len(act) != num_r:
        raise LayoutError("active mask has the wrong length")
    bsz = lay.block_size
    need = [r for r in range(num_r) if act[r] and int(lay.suffix_len[r]) % bsz == 0]
    if len(need) > len(pool.free):
        raise OutOfBlocks(f"need {len(need)} blocks, {len(pool.free)} free")
    lists = [list(lay.suffix_blk[lay.suffix_blk_indptr[r]:lay.suffix_blk_indptr[r + 1]]) for r in range(num_r)]
    dest = np.full(num_r, -1, np.int64)
    for r in range(num_r):
        if not act[r]:
            continue
        pos = int(lay.suffix_len[r])
        if pos % bsz == 0:
            blk = pool.free.popleft()
            pool.refcount[blk] += 1
            lists[r].append(blk)
        dest[r] = int(lists[r][pos // bsz]) * bsz + pos % bsz
        lay.suffix_len[r] = pos + 1
    indptr = np.zeros(num_r + 1, np.int32)
    for r in range(num_r):
        indptr[r + 1] = indptr[r] + len(lists[r])
    lay.suffix_blk_indptr = indptr
    lay.suffix_blk = np.asarray([b for l in lists for b in l], np.int32)
    return dest
