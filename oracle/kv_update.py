"""Writing KV into the paged pool: prefix hand-off ingest and per-step append (oracle side, test infrastructure).

What is modelled.  The base module prefills a prompt once and its cache C_base is handed to the decode
workers (Method Eq. 5; System Design, execution pipeline steps 1 and 3: shared prefill, cache hand-off);
there it is stored once in shared blocks.  Every decode step then returns new cache entries dC_t that are
appended to the decode module's own cache (Method Eq. 6; Background Eq. 2 and Eq. 4).  The paper fixes
neither a storage format nor a quantiser; the readings taken are:

  * Source tensors are contiguous per segment: k_src, v_src [L, Hkv, d] in bf16 bits (uint16) for bf16 and
    e4m3 pools, float32 for float32 pools.  Token j of a segment goes to slot j % B of its block j // B.
    Only valid tokens are written; slots past the segment length keep whatever they held.
  * bf16 / float32 pools store the source bits unchanged.
  * e4m3 pools keep one float32 scale per (block, KV head) for K and one for V.  With a = max |x| over the
    valid tokens of the tile (exact in float32), scale = a / 448 rounded to float32 (1 if a = 0), and every
    value is stored as encode(x / scale): float32 division, then round-to-nearest-even to e4m3fn.
  * Appending one token to a partly filled e4m3 tile: cand = a_new / 448 in float32; the tile's scale
    becomes max(scale_old, cand) (a fresh block, slot 0, takes cand, or 1 if a_new = 0).  If the scale grew,
    every token already in the tile is re-encoded from what is stored: y = (decode(code) * scale_old) /
    scale_new with both operations rounded to float32, code' = encode(y).  The new token is encoded with
    the new scale.  Every decision is taken in float32, so an implementation can match bit for bit.

Pool arrays are indexed kv[block, kv_head, 0=K|1=V, slot, :] and scales[block, kv_head, 0=K|1=V], as
everywhere in this package; they are modified in place.
"""
from __future__ import annotations

import numpy as np

from . import fp8

_F448 = np.float32(448.0)


def _as_f32(src: np.ndarray) -> np.ndarray:
    """bf16 bits (uint16) or float32 -> float32, exactly."""
    src = np.asarray(src)
    if src.dtype == np.uint16:
        return (src.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return src.astype(np.float32)


def _tile_scale(x: np.ndarray) -> np.float32:
    a = np.float32(np.max(np.abs(x))) if x.size else np.float32(0)
    return np.float32(a / _F448) if a > 0 else np.float32(1.0)


def _quantise(x: np.ndarray, scale: np.float32) -> np.ndarray:
    return fp8.encode((x.astype(np.float32) / np.float32(scale)).astype(np.float32))


def ingest_segment(kv: np.ndarray, scales, kv_dtype: str, block_ids, k_src: np.ndarray, v_src: np.ndarray) -> None:
    """Store a whole segment (k_src, v_src: [L, Hkv, d]) into the blocks `block_ids` names."""
    bsz = kv.shape[3]
    length, hkv, _ = k_src.shape
    for which, src in ((0, k_src), (1, v_src)):
        for i in range((length + bsz - 1) // bsz):
            blk = int(block_ids[i])
            n = min(bsz, length - i * bsz)
            for h in range(hkv):
                tile = src[i * bsz:i * bsz + n, h, :]
                if kv_dtype == "fp8_e4m3":
                    x = _as_f32(tile)
                    s = _tile_scale(x)
                    scales[blk, h, which] = s
                    kv[blk, h, which, :n, :] = _quantise(x, s)
                else:
                    kv[blk, h, which, :n, :] = tile


def append_token(kv: np.ndarray, scales, kv_dtype: str, dest: int, k_new: np.ndarray, v_new: np.ndarray) -> None:
    """Store one token (k_new, v_new: [Hkv, d]) at global slot index dest = block * B + slot."""
    bsz = kv.shape[3]
    blk, slot = divmod(int(dest), bsz)
    hkv = k_new.shape[0]
    for which, src in ((0, k_new), (1, v_new)):
        for h in range(hkv):
            if kv_dtype != "fp8_e4m3":
                kv[blk, h, which, slot, :] = src[h]
                continue
            x = _as_f32(src[h])
            a = np.float32(np.max(np.abs(x)))
            cand = np.float32(a / _F448)
            if slot == 0:
                new = cand if a > 0 else np.float32(1.0)
            else:
                old = np.float32(scales[blk, h, which])
                new = max(old, cand)
                if new != old:
                    stored = (fp8.decode(kv[blk, h, which, :slot, :]).astype(np.float32) * old).astype(np.float32)
                    kv[blk, h, which, :slot, :] = _quantise(stored, new)
            scales[blk, h, which] = new
            kv[blk, h, which, slot, :] = _quantise(x, new)
