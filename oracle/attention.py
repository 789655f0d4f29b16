"""fp64 decode attention over [shared prefix ; private suffix] (oracle side, test infrastructure).

What is computed (Background Eq. 2 and Eq. 4; Method Eq. 6): a decode module's
single query token attends to its whole cache, which is the base module's
prefix cache followed by the tokens the decode module appended itself.  For
request r on prompt p, q head h, KV head g = h // (Hq / Hkv):

    T_r  = prefix tokens of p  ++  suffix tokens of r
    s_j  = <Q[r,h], K_j[g]> / sqrt(d)                      j in T_r
    LSE  = log sum_j exp(s_j)        (natural log)
    O    = sum_j exp(s_j - LSE) V_j[g]

The paper leaves the attention operator itself implicit (its forward pass is a
black-box F_theta); ordinary scaled dot-product softmax attention with grouped
query heads is the reading taken.  All stored inputs are widened exactly to
fp64 first (fp8: code value times the fp32 scale of its tile).

A *partial state* of a subset of tokens is (o normalised over the subset, lse
over the subset); an empty subset is (0, -inf).  States merge by
lse = log sum_i exp(lse_i), o = sum_i exp(lse_i - lse) o_i, which is exact by
softmax algebra over the concatenation.
"""
from __future__ import annotations

import numpy as np

from . import fp8


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Stored bits -> float64, exactly."""
    if dtype == "f32":
        return np.asarray(bits, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype == "fp8_e4m3":
        return fp8.decode(bits)
    raise ValueError(dtype)


def gather_segment(kv: np.ndarray, scales, kv_dtype: str, block_ids, length: int):
    """Walk a block list and return (K, V) as float64 [length, Hkv, d].

    kv is indexed [block, kv_head, 0=K|1=V, slot, :]; token j of the segment sits in
    slot j % B of block_ids[j // B].  Slots past `length` are never read.
    """
    nblk, hkv, _, bsz, dim = kv.shape
    k = np.empty((length, hkv, dim), np.float64)
    v = np.empty((length, hkv, dim), np.float64)
    for i, blk in enumerate(block_ids):
        lo = i * bsz
        n = min(bsz, length - lo)
        if n <= 0:
            break
        kt = widen(kv[blk, :, 0, :n], kv_dtype)            # [Hkv, n, d]
        vt = widen(kv[blk, :, 1, :n], kv_dtype)
        if kv_dtype == "fp8_e4m3":
            kt = kt * scales[blk, :, 0].astype(np.float64)[:, None, None]
            vt = vt * scales[blk, :, 1].astype(np.float64)[:, None, None]
        k[lo:lo + n] = kt.transpose(1, 0, 2)
        v[lo:lo + n] = vt.transpose(1, 0, 2)
    return k, v


def attention_state(q: np.ndarray, k: np.ndarray, v: np.ndarray):
    """q [Hq, d], k/v [L, Hkv, d] (float64) -> (o [Hq, d], lse [Hq]); L = 0 gives (0, -inf)."""
    hq, dim = q.shape
    length, hkv, _ = k.shape
    group = hq // hkv
    o = np.zeros((hq, dim), np.float64)
    lse = np.full(hq, -np.inf, np.float64)
    if length == 0:
        return o, lse
    for h in range(hq):
        g = h // group
        s = (k[:, g, :] @ q[h]) / np.sqrt(float(dim))
        m = s.max()
        e = np.exp(s - m)
        lse[h] = m + np.log(e.sum())
        o[h] = np.exp(s - lse[h]) @ v[:, g, :]
    return o, lse


def merge_states(o_parts: np.ndarray, lse_parts: np.ndarray):
    """o_parts [n, ..., d], lse_parts [n, ...] -> merged (o [..., d], lse [...])."""
    o_parts = np.asarray(o_parts, np.float64)
    lse_parts = np.asarray(lse_parts, np.float64)
    if o_parts.shape[0] == 0:
        return np.zeros(o_parts.shape[1:]), np.full(lse_parts.shape[1:], -np.inf)
    m = lse_parts.max(axis=0)
    safe_m = np.where(np.isfinite(m), m, 0.0)
    w = np.exp(lse_parts - safe_m)                           # exp(-inf) = 0 for empty parts
    total = w.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(total > 0, safe_m + np.log(total), -np.inf)
        coef = np.where(total > 0, w / np.where(total > 0, total, 1.0), 0.0)
    o = (coef[..., None] * o_parts).sum(axis=0)
    return o, lse


def request_kv(kv, scales, kv_dtype, lay, r: int, prefix_visible=None):
    """Concatenated (K, V) of request r: its prompt's root if there is one, the prefix of its prompt, then its
    own suffix.

    prefix_visible[r] (optional) cuts the prefix to its first prefix_visible[r] tokens.  This is how a
    chunk of new prompt tokens is prefilled against the cache (System Design, execution pipeline step 1:
    later steps extend the cache only for the newly appended tokens): the chunk's tokens are stored as
    the continuation of the shared prefix, every one of them is a query row on that prompt, and row i
    sees the old cache plus the chunk's tokens 0..i -- ordinary causal attention written as a length.
    """
    p = int(lay.req_prompt[r])
    seen = int(lay.prefix_len[p]) if prefix_visible is None else int(prefix_visible[r])
    if not 0 <= seen <= int(lay.prefix_len[p]):
        raise ValueError("visible prefix length out of range")
    parts = []
    # a context several prompts have in common (a root, layout.build_layout_tree) comes first, whole
    t = -1 if getattr(lay, "prompt_root", None) is None else int(lay.prompt_root[p])
    if t >= 0:
        parts.append(gather_segment(kv, scales, kv_dtype, lay.root_blk[lay.root_blk_indptr[t]:lay.root_blk_indptr[t + 1]],
                                    int(lay.root_len[t])))
    parts.append(gather_segment(kv, scales, kv_dtype,
                                lay.prefix_blk[lay.prefix_blk_indptr[p]:lay.prefix_blk_indptr[p + 1]], seen))
    parts.append(gather_segment(kv, scales, kv_dtype,
                                lay.suffix_blk[lay.suffix_blk_indptr[r]:lay.suffix_blk_indptr[r + 1]],
                                int(lay.suffix_len[r])))
    return np.concatenate([k for k, _ in parts], axis=0), np.concatenate([v for _, v in parts], axis=0)


def decode_attention(q_bits, q_dtype: str, kv, scales, kv_dtype: str, lay, requests=None, prefix_visible=None):
    """Whole-step oracle: (O [n, Hq, d], LSE [n, Hq]) for `requests` (default: all, in order).

    prefix_visible: optional int [R], see request_kv."""
    q = widen(q_bits, q_dtype)
    reqs = range(q.shape[0]) if requests is None else list(requests)
    out = np.zeros((len(reqs),) + q.shape[1:], np.float64)
    lse = np.zeros((len(reqs), q.shape[1]), np.float64)
    for i, r in enumerate(reqs):
        k, v = request_kv(kv, scales, kv_dtype, lay, r, prefix_visible)
        out[i], lse[i] = attention_state(q[r], k, v)
    return out, lse


def segment_states(q_bits, q_dtype: str, kv, scales, kv_dtype: str, lay, requests=None):
    """Per-request partial states of the two segments: ((o_pre, lse_pre), (o_suf, lse_suf))."""
    q = widen(q_bits, q_dtype)
    reqs = range(q.shape[0]) if requests is None else list(requests)
    shape_o = (len(reqs),) + q.shape[1:]
    o_pre, o_suf = np.zeros(shape_o), np.zeros(shape_o)
    l_pre, l_suf = np.zeros(shape_o[:2]), np.zeros(shape_o[:2])
    for i, r in enumerate(reqs):
        p = int(lay.req_prompt[r])
        kp, vp = gather_segment(kv, scales, kv_dtype,
                                lay.prefix_blk[lay.prefix_blk_indptr[p]:lay.prefix_blk_indptr[p + 1]],
                                int(lay.prefix_len[p]))
        ks, vs = gather_segment(kv, scales, kv_dtype,
                                lay.suffix_blk[lay.suffix_blk_indptr[r]:lay.suffix_blk_indptr[r + 1]],
                                int(lay.suffix_len[r]))
        o_pre[i], l_pre[i] = attention_state(q[r], kp, vp)
        o_suf[i], l_suf[i] = attention_state(q[r], ks, vs)
    return (o_pre, l_pre), (o_suf, l_suf)
