"""GPU: a context that lives across steps.  A decode batch over the cached contexts, then the partial prefill of the
segments appended to them (a layout that adopts the cached blocks and ingests only what is new), then the next decode
batch over the grown contexts -- tables, refcounts, pool bits and attention against the oracle at every step."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as oa
from oracle import kv_update as ku
from oracle import layout as ol
from helpers import errors

pytestmark = pytest.mark.gpu

B16 = 16


def _bits(rng, shape, gain=1.0):
    return wl.bf16_bits_from_f32((rng.standard_normal(shape) * gain).astype(np.float32))


class Side:
    """The library's pool and the oracle's, driven in lockstep over one device KV tensor / one numpy array."""

    def __init__(self, geo, num_blocks, kv_dtype):
        from paper_2602_12029_amd import binding as B
        from paper_2602_12029_amd.runtime import to_device
        self.B, self.geo_w = B, geo
        self.geo = B.geometry(geo.num_q_heads, geo.num_kv_heads, geo.head_dim, geo.block_size, "bf16", kv_dtype)
        order = np.random.default_rng(5).permutation(num_blocks).astype(np.int32)
        self.pool, self.opool = B.ps_pool_create(num_blocks, order), ol.BlockPool(num_blocks, order)
        shape = (num_blocks, geo.num_kv_heads, 2, geo.block_size, geo.head_dim)
        self.kv_ref = np.full(shape, wl.generate.POISON[kv_dtype], wl.generate.STORAGE[kv_dtype])
        self.sc_ref = np.full((num_blocks, geo.num_kv_heads, 2), np.nan, np.float32) if kv_dtype == "fp8_e4m3" else None
        self.kv = to_device(self.kv_ref, kv_dtype)
        self.scales = None if self.sc_ref is None else torch.from_numpy(self.sc_ref.copy()).cuda()
        self.kv_dtype = kv_dtype

    def layout(self, ctx, adopt, rp, rm, sl, q_bits):
        from paper_2602_12029_amd.runtime import DecodeBatch, to_device
        B = self.B
        lay = B.ps_kv_layout_adopt(self.pool, self.geo, ctx, adopt, rp, rm, sl)
        olay = ol.build_layout(self.opool, B16, ctx, rp, rm, sl, adopt=adopt)
        t = B.ps_layout_tables(lay, len(ctx), len(rp))
        for key in t:
            assert np.array_equal(t[key], getattr(olay, key)), key
        batch = DecodeBatch(lay, self.geo, len(rp), to_device(q_bits, "bf16"), self.kv, self.scales)
        return lay, olay, batch

    def ingest(self, batch, olay, which, segments, skip_blocks=None):
        """segments: per segment (k, v) bf16 bits of the tokens to store; skip_blocks: leading blocks left alone."""
        from paper_2602_12029_amd.runtime import to_device
        ids_of = (lambda s: olay.prefix_blk[olay.prefix_blk_indptr[s]:olay.prefix_blk_indptr[s + 1]]) if which == 0 else \
                 (lambda s: olay.suffix_blk[olay.suffix_blk_indptr[s]:olay.suffix_blk_indptr[s + 1]])
        for s, (k, v) in enumerate(segments):
            skip = 0 if skip_blocks is None else skip_blocks[s]
            if k.shape[0]:
                ku.ingest_segment(self.kv_ref, self.sc_ref, self.kv_dtype, ids_of(s)[skip:], k, v)
        parts = [seg for seg in segments if seg[0].shape[0]]
        if parts:
            batch.kv_ingest(which, to_device(np.concatenate([p[0] for p in parts]), "bf16"),
                            to_device(np.concatenate([p[1] for p in parts]), "bf16"))

    def check(self, batch, olay, q_bits, label, visible=None):
        from paper_2602_12029_amd.runtime import from_device
        batch.workspace.view(torch.float32).fill_(float("nan"))
        batch.decode_attention()
        torch.cuda.synchronize()
        ref, ref_lse = oa.decode_attention(q_bits, "bf16", self.kv_ref, self.sc_ref, self.kv_dtype, olay, None, visible)
        got = from_device(batch.out)
        max_abs, rel_rms, worst = errors(got, ref)
        print(f"[{label}] max_abs={max_abs:.3e} rel_rms={rel_rms:.3e} worst_req_rel_rms={worst:.3e}", flush=True)
        assert np.isfinite(got).all() and rel_rms <= 5e-3
        assert float((np.abs(got - ref) / np.maximum(1.0, np.abs(ref))).max()) <= 1e-2
        assert np.abs(from_device(batch.lse) - ref_lse).max() <= 2e-3
        # the pool holds the oracle's bits wherever a live block is concerned
        live = np.flatnonzero(self.opool.refcount > 0)
        got_kv = self.kv.cpu().view(torch.uint8 if self.kv_dtype == "fp8_e4m3" else torch.int16).numpy().reshape(self.kv_ref.shape)
        ref_kv = self.kv_ref.view(np.uint8 if self.kv_dtype == "fp8_e4m3" else np.int16)
        assert np.array_equal(self.B.ps_pool_refcounts(self.pool, len(self.opool.refcount)), self.opool.refcount)
        return got_kv, ref_kv, live


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_contexts_continued_over_decode_prefill_decode(kv_dtype):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    geo = wl.Geometry(32, 8, 128, B16, "bf16", kv_dtype)
    hkv, d, hq = geo.num_kv_heads, geo.head_dim, geo.num_q_heads
    rng = np.random.default_rng(73)
    side = Side(geo, 200, kv_dtype)
    B = side.B

    # ---- step 0: a decode batch over two cached contexts (everything handed over and ingested)
    ctx0 = np.array([300, 77])
    ctx_k = [_bits(rng, (n, hkv, d)) for n in ctx0]
    ctx_v = [_bits(rng, (n, hkv, d)) for n in ctx0]
    rp0, rm0, sl0 = [0, 0, 0, 1, 1], [0, 1, 2, 1, 3], [5, 0, 40, 17, 1]
    q0 = _bits(rng, (5, hq, d))
    d0, od0, b0 = side.layout(ctx0, [[], []], rp0, rm0, sl0, q0)
    side.ingest(b0, od0, 0, list(zip(ctx_k, ctx_v)))
    side.ingest(b0, od0, 1, [(_bits(rng, (n, hkv, d)), _bits(rng, (n, hkv, d))) for n in sl0])
    side.check(b0, od0, q0, f"session {kv_dtype}: decode over the cached contexts")

    # ---- step 1: the contexts grow by 50 and 130 tokens; the new tokens are prefilled against the cache
    grow = np.array([50, 130])
    ctx1 = ctx0 + grow
    new_k = [_bits(rng, (n, hkv, d)) for n in grow]
    new_v = [_bits(rng, (n, hkv, d)) for n in grow]
    ctx_k = [np.concatenate([a, b]) for a, b in zip(ctx_k, new_k)]
    ctx_v = [np.concatenate([a, b]) for a, b in zip(ctx_v, new_v)]
    t0 = B.ps_layout_tables(d0, 2, 5)
    full0 = [int(n) // B16 for n in ctx0]
    adopt1 = [t0["prefix_blk"][t0["prefix_blk_indptr"][p]:t0["prefix_blk_indptr"][p] + full0[p]].tolist() for p in range(2)]
    rp1 = [0] * 50 + [1] * 130
    rm1 = list(range(50)) + list(range(130))
    vis1 = np.concatenate([ctx0[p] + 1 + np.arange(grow[p]) for p in range(2)]).astype(np.int32)
    q1 = _bits(rng, (180, hq, d))
    p1, op1, b1 = side.layout(ctx1, adopt1, rp1, rm1, [0] * 180, q1)
    # only what the adopted blocks do not hold is handed over: the tail of the old context and the new tokens
    side.ingest(b1, op1, 0, [(ctx_k[p][full0[p] * B16:], ctx_v[p][full0[p] * B16:]) for p in range(2)], skip_blocks=full0)
    b1.set_visible(vis1)
    got_kv, ref_kv, live = side.check(b1, op1, q1, f"session {kv_dtype}: partial prefill of the appended segments", vis1)
    # adopted blocks were not rewritten, new ones hold the oracle's bits (full blocks compared; tails by attention)
    for p in range(2):
        ids = op1.prefix_blk[op1.prefix_blk_indptr[p]:op1.prefix_blk_indptr[p + 1]]
        n_full = int(ctx1[p]) // B16
        assert np.array_equal(got_kv[ids[:n_full]], ref_kv[ids[:n_full]])
    side.check(b0, od0, q0, f"session {kv_dtype}: the first batch still reads its own context")

    # ---- step 2: the first batch ends; the next decode batch runs over the grown contexts
    B.ps_layout_release(side.pool, d0)
    ol.release_layout(side.opool, od0)
    t1 = B.ps_layout_tables(p1, 2, 180)
    full1 = [int(n) // B16 for n in ctx1]
    adopt2 = [t1["prefix_blk"][t1["prefix_blk_indptr"][p]:t1["prefix_blk_indptr"][p] + full1[p]].tolist() for p in range(2)]
    rp2, rm2, sl2 = [0, 0, 1, 1, 1], [1, 3, 0, 1, 2], [9, 64, 0, 3, 130]
    q2 = _bits(rng, (5, hq, d))
    d2, od2, b2 = side.layout(ctx1, adopt2, rp2, rm2, sl2, q2)
    side.ingest(b2, od2, 0, [(ctx_k[p][full1[p] * B16:], ctx_v[p][full1[p] * B16:]) for p in range(2)], skip_blocks=full1)
    side.ingest(b2, od2, 1, [(_bits(rng, (n, hkv, d)), _bits(rng, (n, hkv, d))) for n in sl2])
    B.ps_layout_release(side.pool, p1)
    ol.release_layout(side.opool, op1)
    side.check(b2, od2, q2, f"session {kv_dtype}: decode over the grown contexts")
    B.ps_layout_release(side.pool, d2)
    ol.release_layout(side.opool, od2)
    assert not B.ps_pool_refcounts(side.pool, 200).any()
    assert np.array_equal(B.ps_pool_free_list(side.pool), np.array(side.opool.free, np.int32))
    B.ps_pool_destroy(side.pool)
