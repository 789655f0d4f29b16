"""Seeded generators for multi-model shared-prefix decode batches.

A *workload* is one decode step of M task-specific decode modules over P
prompts: every (prompt, model) request holds one query token, reads the
prompt's prefix KV (produced once by the frozen prefill module, Method
"Definitions and Formulation", Eq. 5-6) and its own private suffix KV (the
model-specific segment of the Efficiency Analysis, Eq. 9).

Nothing here computes attention or decides where blocks live: lengths, sharing
structure, the pool's free order and the *stored bits* of Q/K/V are drawn from
PCG64 streams keyed by (seed, tag, index), so every item can be regenerated on
its own and in any order.  Draw tags: 1 lengths, 2 membership, 3 free order,
4 Q, 5 prefix K/V (index = prompt), 6 suffix K/V (index = request), 7 / 8 unquantised
prefix / suffix K/V as a worker hands them over, 9 the K/V of the token each request
appends in a decode step (index = step), 10 root K/V (index = root), 11 unquantised root K/V.

Storage formats: 'f32' -> float32, 'bf16' -> uint16 bit patterns (fp32 draws
rounded to nearest-even), 'fp8_e4m3' -> uint8 OCP e4m3fn codes plus one fp32
scale per (16-token block, KV head) for K and one for V, scale = absmax of the
valid tokens of the tile / 448 (1 if the tile is all zero).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

STORAGE = {"f32": np.float32, "bf16": np.uint16, "fp8_e4m3": np.uint8}
ELEM_BYTES = {"f32": 4, "bf16": 2, "fp8_e4m3": 1}
# Values written into every slot no request may read (NaN in each format).
POISON = {"f32": np.float32("nan"), "bf16": np.uint16(0x7FC0), "fp8_e4m3": np.uint8(0x7F)}

CONFIG_NAMES = ("tiny", "b8", "long", "mixed", "fp8_70b")


def _rng(seed: int, tag: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(tag), int(index)])))


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round finite float32 values to bfloat16 (nearest, ties to even); return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Quantise finite float32 values to OCP e4m3fn codes: nearest-even, saturating at +-448.

    e4m3fn: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent
    field 0 is subnormal (multiples of 2^-9); no infinities.
    """
    x = np.asarray(x, dtype=np.float32)
    sign = (np.signbit(x).astype(np.uint8) << np.uint8(7)).astype(np.uint8)
    a = np.minimum(np.abs(x).astype(np.float64), 448.0)
    sub = a < 2.0 ** -6
    code_sub = np.rint(a * 512.0)                      # 0..8 ; 8 is the smallest normal
    _, e = np.frexp(np.where(sub, 1.0, a))
    big_e = e.astype(np.int64) - 1                     # a = (1.f) * 2^big_e
    frac = np.rint((np.where(sub, 1.0, a) / np.exp2(big_e.astype(np.float64)) - 1.0) * 8.0).astype(np.int64)
    carry = frac == 8
    big_e = big_e + carry
    frac = np.where(carry, 0, frac)
    code_norm = ((big_e + 7) << 3) | frac
    code = np.where(sub, code_sub.astype(np.int64), code_norm).astype(np.uint8)
    return (code | sign).astype(np.uint8)


@dataclass(frozen=True)
class Geometry:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    q_dtype: str          # 'f32' | 'bf16'
    kv_dtype: str         # 'f32' | 'bf16' | 'fp8_e4m3'

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def token_bytes(self) -> int:
        """Bytes of K plus V for one token over all KV heads (b_tok)."""
        return 2 * self.num_kv_heads * self.head_dim * ELEM_BYTES[self.kv_dtype]


@dataclass
class Segment:
    """Stored bits of one KV segment: k, v are [L, Hkv, d]; scales [ceil(L/B), Hkv] or None."""
    k: np.ndarray
    v: np.ndarray
    k_scale: Optional[np.ndarray] = None
    v_scale: Optional[np.ndarray] = None


@dataclass(frozen=True)
class ScoreShape:
    """Deterministic structure laid over the N(0,1) draws, so that attention scores are not unit-spread.

    Decode attention in practice sees sink tokens, late dominant keys and scores that drift over a context; i.i.d.
    N(0,1) queries and keys give none of that (their scores spread a few units and the largest one sits anywhere).
    Everything here acts on the float32 draws before they are rounded / quantised, so the stored bits are still
    what both sides read.

    q_gain, k_gain   factors on the query / key draws (score spread = q_gain * k_gain)
    q_bias           added to every component of every query row
    k_profile        per-token offset c_j added to every component of key j of a segment of L tokens; with
                     q_bias = b the score of token j moves by about b * c_j * sqrt(d):
                       'none'            c_j = 0
                       'ramp_up'         c_j = k_amp * j / max(1, L - 1)        (scores climb through the segment)
                       'ramp_down'       c_j = k_amp * (1 - j / max(1, L - 1))
                       'dominant_first'  c_j = k_amp at j = min(3, L - 1), else 0
                       'dominant_mid'    c_j = k_amp at j = L // 2, else 0
                       'dominant_last'   c_j = k_amp at j = L - 1, else 0
                       'equal'           every key of the segment is replaced by one and the same vector (the
                                         segment's first draw): all its scores are equal
    segments         which KV segments get the profile: 'all', 'prefix' (shared prefixes and roots) or 'suffix'
    """
    q_gain: float = 1.0
    k_gain: float = 1.0
    q_bias: float = 0.0
    k_profile: str = "none"
    k_amp: float = 0.0
    segments: str = "all"

    def shape_q(self, q: np.ndarray) -> np.ndarray:
        return (q * np.float32(self.q_gain) + np.float32(self.q_bias)).astype(np.float32)

    def shape_k(self, k: np.ndarray, shared: bool) -> np.ndarray:
        """k [L, Hkv, d] float32 draws of one segment -> shaped float32."""
        k = (k * np.float32(self.k_gain)).astype(np.float32)
        length = k.shape[0]
        if length == 0 or self.k_profile == "none" or self.segments == ("suffix" if shared else "prefix"):
            return k
        j = np.arange(length, dtype=np.float64)
        if self.k_profile == "ramp_up":
            c = self.k_amp * j / max(1, length - 1)
        elif self.k_profile == "ramp_down":
            c = self.k_amp * (1.0 - j / max(1, length - 1))
        elif self.k_profile in ("dominant_first", "dominant_mid", "dominant_last"):
            at = {"dominant_first": min(3, length - 1), "dominant_mid": length // 2, "dominant_last": length - 1}
            c = np.where(j == at[self.k_profile], self.k_amp, 0.0)
        elif self.k_profile == "equal":
            return np.broadcast_to(k[:1], k.shape).copy()
        else:
            raise ValueError(self.k_profile)
        return (k + c.astype(np.float32)[:, None, None]).astype(np.float32)


@dataclass
class Workload:
    name: str
    seed: int
    geometry: Geometry
    num_models: int
    prefix_len: np.ndarray            # int32 [P]
    req_prompt: np.ndarray            # int32 [R]
    req_model: np.ndarray             # int32 [R]
    suffix_len: np.ndarray            # int32 [R]
    num_blocks: int                   # size of the physical pool
    free_order: np.ndarray            # int32 [num_blocks], a permutation
    _cache: Dict = field(default_factory=dict, repr=False)
    # optional third level: contexts that several prompts begin with (make_tree_workload)
    root_len: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))   # int32 [T]
    prompt_root: Optional[np.ndarray] = None                                      # int32 [P], -1 = no root
    # optional structure on top of the N(0,1) draws (scores that drift, dominate or tie; see ScoreShape)
    score_shape: Optional[ScoreShape] = None

    @property
    def num_roots(self) -> int:
        return int(self.root_len.shape[0])

    @property
    def num_prompts(self) -> int:
        return int(self.prefix_len.shape[0])

    @property
    def num_requests(self) -> int:
        return int(self.req_prompt.shape[0])

    def blocks_needed(self) -> int:
        b = self.geometry.block_size
        return int(((self.prefix_len.astype(np.int64) + b - 1) // b).sum()
                   + ((self.suffix_len.astype(np.int64) + b - 1) // b).sum()
                   + ((self.root_len.astype(np.int64) + b - 1) // b).sum())

    # ---- stored bits -----------------------------------------------------
    def _normal(self, tag: int, index: int, shape) -> np.ndarray:
        return _rng(self.seed, tag, index).standard_normal(shape, dtype=np.float32)

    def q_bits(self) -> np.ndarray:
        g = self.geometry
        x = self._normal(4, 0, (self.num_requests, g.num_q_heads, g.head_dim))
        if self.score_shape is not None:
            x = self.score_shape.shape_q(x)
        return x if g.q_dtype == "f32" else bf16_bits_from_f32(x)

    def _segment(self, tag: int, index: int, length: int) -> Segment:
        g = self.geometry
        shape = (int(length), g.num_kv_heads, g.head_dim)
        rng = _rng(self.seed, tag, index)
        k = rng.standard_normal(shape, dtype=np.float32)
        v = rng.standard_normal(shape, dtype=np.float32)
        if self.score_shape is not None:
            k = self.score_shape.shape_k(k, shared=tag != 6)
        if g.kv_dtype == "f32":
            return Segment(k, v)
        if g.kv_dtype == "bf16":
            return Segment(bf16_bits_from_f32(k), bf16_bits_from_f32(v))
        kc, ks = _quantise_tiles(k, g.block_size)
        vc, vs = _quantise_tiles(v, g.block_size)
        return Segment(kc, vc, ks, vs)

    def prefix_kv(self, prompt: int) -> Segment:
        return self._segment(5, prompt, int(self.prefix_len[prompt]))

    def suffix_kv(self, request: int) -> Segment:
        return self._segment(6, request, int(self.suffix_len[request]))

    def root_kv(self, root: int) -> Segment:
        return self._segment(10, root, int(self.root_len[root]))

    # ---- unquantised sources (what a prefill or decode worker hands over) ----
    def _source(self, tag: int, index: int, tokens: int):
        """K, V [tokens, Hkv, d]: N(0,1) values times a per-token gain drawn log-uniformly from [1/4, 1]
        (so that tokens differ in magnitude while values stay in the range of the N(0,1) workloads), as bf16 bit patterns -- float32 for float32 pools."""
        g = self.geometry
        rng = _rng(self.seed, tag, index)
        out = []
        for _ in range(2):
            x = rng.standard_normal((int(tokens), g.num_kv_heads, g.head_dim), dtype=np.float32)
            gain = np.exp2(rng.uniform(-2.0, 0.0, size=(int(tokens), 1, 1))).astype(np.float32)
            x = x * gain
            out.append(x if g.kv_dtype == "f32" else bf16_bits_from_f32(x))
        return out[0], out[1]

    def prefix_source(self, prompt: int):
        return self._source(7, prompt, int(self.prefix_len[prompt]))

    def suffix_source(self, request: int):
        return self._source(8, request, int(self.suffix_len[request]))

    def root_source(self, root: int):
        return self._source(11, root, int(self.root_len[root]))

    def step_tokens(self, step: int):
        """K, V [R, Hkv, d] of the one token every request appends in decode step `step`."""
        return self._source(9, step, self.num_requests)


def _quantise_tiles(x: np.ndarray, block: int):
    """x [L, H, d] float32 -> (codes uint8 [L, H, d], scales float32 [ceil(L/B), H])."""
    length, heads, dim = x.shape
    nb = (length + block - 1) // block
    pad = np.zeros((nb * block, heads, dim), np.float32)
    pad[:length] = x
    tiles = pad.reshape(nb, block, heads, dim)
    absmax = np.abs(tiles).max(axis=(1, 3)).astype(np.float32)          # [nb, H]
    scale = np.where(absmax > 0, absmax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    codes = e4m3_encode(tiles / scale[:, None, :, None])
    return codes.reshape(nb * block, heads, dim)[:length].copy(), scale


@dataclass
class PoolData:
    """Physical KV pool as the decode GPU holds it.

    kv     : [num_blocks, Hkv, 2, B, d] storage dtype; [:, :, 0] = K, [:, :, 1] = V
    scales : [num_blocks, Hkv, 2] float32 (fp8 only, else None)
    Slots no request owns hold NaN patterns.
    """
    kv: np.ndarray
    scales: Optional[np.ndarray]


def fill_pool(w: Workload, prefix_blk_indptr, prefix_blk, suffix_blk_indptr, suffix_blk, root_blk_indptr=None,
              root_blk=None) -> PoolData:
    """Scatter every segment's stored bits into the pool at the blocks a block table names.

    The tables come from whichever layout builder is under test; this routine
    only copies bits (token j of a segment goes to slot j % B of the segment's
    block j // B).
    """
    g = w.geometry
    b = g.block_size
    kv = np.full((w.num_blocks, g.num_kv_heads, 2, b, g.head_dim), POISON[g.kv_dtype], dtype=STORAGE[g.kv_dtype])
    scales = None
    if g.kv_dtype == "fp8_e4m3":
        scales = np.full((w.num_blocks, g.num_kv_heads, 2), np.nan, dtype=np.float32)

    def put(seg: Segment, ids: np.ndarray):
        length = seg.k.shape[0]
        nfull = length // b
        for which, arr in ((0, seg.k), (1, seg.v)):
            if nfull:
                full = arr[: nfull * b].reshape(nfull, b, g.num_kv_heads, g.head_dim).transpose(0, 2, 1, 3)
                kv[ids[:nfull], :, which] = full
            rem = length - nfull * b
            if rem:
                kv[ids[nfull], :, which, :rem] = arr[nfull * b:].transpose(1, 0, 2)
        if scales is not None and length:
            scales[ids, :, 0] = seg.k_scale
            scales[ids, :, 1] = seg.v_scale

    prefix_blk = np.asarray(prefix_blk)
    suffix_blk = np.asarray(suffix_blk)
    for p in range(w.num_prompts):
        put(w.prefix_kv(p), prefix_blk[prefix_blk_indptr[p]:prefix_blk_indptr[p + 1]])
    for r in range(w.num_requests):
        put(w.suffix_kv(r), suffix_blk[suffix_blk_indptr[r]:suffix_blk_indptr[r + 1]])
    if w.num_roots:
        root_blk = np.asarray(root_blk)
        for t in range(w.num_roots):
            put(w.root_kv(t), root_blk[root_blk_indptr[t]:root_blk_indptr[t + 1]])
    return PoolData(kv, scales)


def ideal_bytes(w: Workload) -> int:
    """HBM bytes an ideal kernel moves: shared KV once + private KV (+ fp8 scales) + Q + O."""
    g = w.geometry
    total = int(w.prefix_len.astype(np.int64).sum() + w.suffix_len.astype(np.int64).sum()
                + w.root_len.astype(np.int64).sum()) * g.token_bytes
    if g.kv_dtype == "fp8_e4m3":
        total += w.blocks_needed() * g.num_kv_heads * 2 * 4
    total += 2 * w.num_requests * g.num_q_heads * g.head_dim * ELEM_BYTES[g.q_dtype]
    return total


def make_workload(name: str, geometry: Geometry, num_models: int, prefix_len: Sequence[int],
                  membership: Sequence[Sequence[int]], suffix_len: Sequence[int],
                  pool_factor: float = 1.0, seed: int = 0) -> Workload:
    """Build a workload from explicit lengths.

    membership[p] lists the models that decode on prompt p (ascending); requests are
    numbered prompt-major in that order and suffix_len follows the same numbering.
    """
    req_prompt: List[int] = []
    req_model: List[int] = []
    for p, models in enumerate(membership):
        for m in models:
            if not 0 <= m < num_models:
                raise ValueError("model index out of range")
            req_prompt.append(p)
            req_model.append(m)
    if len(suffix_len) != len(req_prompt) or len(membership) != len(prefix_len):
        raise ValueError("length lists do not match the membership")
    w = Workload(name, seed, geometry, num_models,
                 np.asarray(prefix_len, np.int32), np.asarray(req_prompt, np.int32),
                 np.asarray(req_model, np.int32), np.asarray(suffix_len, np.int32), 0, np.zeros(0, np.int32))
    needed = w.blocks_needed()
    w.num_blocks = int(np.ceil(pool_factor * needed)) if needed else 0
    w.free_order = _rng(seed, 3).permutation(w.num_blocks).astype(np.int32)
    return w


def make_tree_workload(name: str, geometry: Geometry, num_models: int, root_len: Sequence[int],
                       prompt_root: Sequence[int], prefix_len: Sequence[int], membership: Sequence[Sequence[int]],
                       suffix_len: Sequence[int], pool_factor: float = 1.0, seed: int = 0) -> Workload:
    """A workload with a third level: root_len[t] tokens that every prompt p with prompt_root[p] = t begins with (a
    common system prompt or shared document in front of each session's own context); prefix_len[p] is then the
    prompt's own part.  prompt_root[p] = -1: no root."""
    w = make_workload(name, geometry, num_models, prefix_len, membership, suffix_len, pool_factor, seed)
    w.root_len = np.asarray(root_len, np.int32)
    w.prompt_root = np.asarray(prompt_root, np.int32)
    if w.prompt_root.shape != w.prefix_len.shape:
        raise ValueError("one root index per prompt")
    needed = w.blocks_needed()
    w.num_blocks = int(np.ceil(pool_factor * needed)) if needed else 0
    w.free_order = _rng(seed, 3).permutation(w.num_blocks).astype(np.int32)
    return w


def named_tree_workload(name: str, seed: int = 0) -> Workload:
    """Three-level stand-ins for multi-agent sessions that all start from one system prompt / tool description:

    tree_tiny  1 root of 40 tokens under 2 of 3 prompts, fp32, 4 q / 2 kv heads, d 64
    tree_b8    1 root of 2048 tokens under 32 sessions, each session 2048 own tokens shared by M = 4 models,
               suffix U[1,512], 32/8 heads, d 128, bf16 (the 8B-shaped batch with half of every prefix in common)
    """
    if name == "tree_tiny":
        return make_tree_workload(name, Geometry(4, 2, 64, 16, "f32", "f32"), 2, [40], [0, -1, 0], [24, 50, 7],
                                  [[0, 1], [0], [1]], [3, 0, 9, 20], 1.0, seed)
    if name == "tree_b8":
        suffix = _rng(seed, 1).integers(1, 513, 128)
        return make_tree_workload(name, Geometry(32, 8, 128, 16, "bf16", "bf16"), 4, [2048], [0] * 32, [2048] * 32,
                                  [[0, 1, 2, 3]] * 32, suffix, 1.0, seed)
    raise ValueError(name)


def chunk_prefill_workload(name: str, geometry: Geometry, cached_len: Sequence[int], chunk_len: Sequence[int],
                           pool_factor: float = 1.0, seed: int = 0):
    """Partial prefill of P contexts (System Design, execution pipeline step 1): context p holds cached_len[p]
    tokens whose KV is cached and grows by chunk_len[p] new tokens.  Returns (workload, visible): the new tokens'
    KV continues the prompt's shared prefix (prefix length = cached + chunk), every new token is one request on
    its prompt (model index = position in the chunk, no private suffix), and visible[r] = cached + position + 1
    is how much of the prefix that token's query row attends to (causal order inside the chunk)."""
    cached = np.asarray(cached_len, np.int64)
    chunk = np.asarray(chunk_len, np.int64)
    if cached.shape != chunk.shape or (cached < 0).any() or (chunk < 1).any():
        raise ValueError("one cached length >= 0 and one chunk length >= 1 per context")
    membership = [list(range(int(c))) for c in chunk]
    w = make_workload(name, geometry, int(chunk.max()), (cached + chunk).tolist(), membership,
                      [0] * int(chunk.sum()), pool_factor, seed)
    visible = np.concatenate([cached[p] + 1 + np.arange(chunk[p]) for p in range(len(chunk))]).astype(np.int32)
    return w, visible


def named_chunk_prefill(name: str, seed: int = 0):
    """Partial-prefill stand-ins for a model switch in multi-agent traffic (the previous module's output segment
    is appended to the shared context and prefilled by the base module against the cached context):

    prefill_tiny  2 contexts, cached 40 / 7, chunks 19 / 30, 4 q / 2 kv heads, d 64, fp32
    prefill_b8    32 contexts, cached 4096, chunks U[64,256], 32/8 heads, d 128, bf16
    prefill_fp8   64 contexts, cached 8192, chunks U[64,256], 64/8 heads, bf16 Q, e4m3 KV
    """
    rng = _rng(seed, 1)
    if name == "prefill_tiny":
        return chunk_prefill_workload(name, Geometry(4, 2, 64, 16, "f32", "f32"), [40, 7], [19, 30], 1.0, seed)
    if name == "prefill_b8":
        return chunk_prefill_workload(name, Geometry(32, 8, 128, 16, "bf16", "bf16"), [4096] * 32,
                                      rng.integers(64, 257, 32), 1.0, seed)
    if name == "prefill_fp8":
        return chunk_prefill_workload(name, Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3"), [8192] * 64,
                                      rng.integers(64, 257, 64), 1.0, seed)
    raise ValueError(name)


def named_workload(name: str, seed: int = 0, models: Optional[int] = None) -> Workload:
    """The five benchmark configurations (synthetic stand-ins for multi-agent traffic).

    tiny     M=2, 1 prompt, prefix 256, suffix 8, 4 q / 2 kv heads, d 64, fp32
    b8       M=4, 32 prompts, prefix 4096, suffix U[1,512], 32/8 heads, d 128, bf16
    long     M=8, 8 prompts, prefix 32768, suffix U[256,2048], bf16, pool 1.5x
    mixed    M=6, 256 prompts, prefix log-uniform [512,16384], 2-6 models per prompt,
             suffix U[1,1024], bf16
    fp8_70b  M=4, 64 prompts, prefix 8192, suffix U[1,512], 64/8 heads, bf16 Q, e4m3 KV

    sessionsS  (S a number, e.g. sessions80) S concurrent multi-agent sessions, M=4 agents decoding on each session's
             context: context lengths uniform in [1024, 6144] (multi-turn agent contexts), suffix U[1,256], 8B-shaped
             heads, bf16 -- the shape of a sweep over the cap on concurrent sessions (Experiments, impact of max
             concurrent sessions): the shared KV footprint grows with S, an unshared system's with M S

    `models` overrides M for the configurations in which every model decodes on every prompt (b8, long,
    fp8_70b, sessionsS): same prompts and prefixes, M private suffixes per prompt (for sweeps over M).
    """
    len_rng = _rng(seed, 1)
    mem_rng = _rng(seed, 2)
    if name == "tiny":
        geo = Geometry(4, 2, 64, 16, "f32", "f32")
        return make_workload(name, geo, 2, [256], [[0, 1]], [8, 8], 1.0, seed)
    if name == "b8":
        geo = Geometry(32, 8, 128, 16, "bf16", "bf16")
        m, p = (models or 4), 32
        return make_workload(name, geo, m, [4096] * p, [list(range(m))] * p,
                             len_rng.integers(1, 513, size=p * m), 1.0, seed)
    if name == "long":
        geo = Geometry(32, 8, 128, 16, "bf16", "bf16")
        m, p = (models or 8), 8
        return make_workload(name, geo, m, [32768] * p, [list(range(m))] * p,
                             len_rng.integers(256, 2049, size=p * m), 1.5, seed)
    if name == "mixed":
        geo = Geometry(32, 8, 128, 16, "bf16", "bf16")
        m, p = 6, 256
        u = len_rng.uniform(np.log(512.0), np.log(16384.0), size=p)
        prefix = np.clip(np.floor(np.exp(u)), 512, 16384).astype(np.int64)
        sizes = mem_rng.integers(2, 7, size=p)
        membership = [sorted(mem_rng.choice(m, size=int(k), replace=False).tolist()) for k in sizes]
        nreq = int(sizes.sum())
        return make_workload(name, geo, m, prefix, membership, len_rng.integers(1, 1025, size=nreq), 1.0, seed)
    if name == "fp8_70b":
        geo = Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3")
        m, p = (models or 4), 64
        return make_workload(name, geo, m, [8192] * p, [list(range(m))] * p,
                             len_rng.integers(1, 513, size=p * m), 1.0, seed)
    if name.startswith("sessions") and name[8:].isdigit() and int(name[8:]) > 0:
        geo = Geometry(32, 8, 128, 16, "bf16", "bf16")
        m, p = (models or 4), int(name[8:])
        return make_workload(name, geo, m, len_rng.integers(1024, 6145, size=p), [list(range(m))] * p,
                             len_rng.integers(1, 257, size=p * m), 1.0, seed)
    raise KeyError(f"unknown workload {name!r}; choose from {CONFIG_NAMES} or sessions<S>")
