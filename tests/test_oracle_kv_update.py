"""Pins for the oracle's cache-writing side: e4m3 encoder, prefix ingest, per-step append, table growth.

None of these compares the oracle with itself: they use the format definition, an independently written
encoder/quantiser (the input generator's), exact round trips, error bounds, order-of-arrival identities,
scalar brute force, and a hand-worked table.
"""
import json
import os

import numpy as np
import pytest

import workloads as wl
from workloads import generate as gen
from oracle import attention as oa
from oracle import fp8
from oracle import kv_update as ku
from oracle import layout as ol

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layout_small.json")


def bf16(x):
    return wl.bf16_bits_from_f32(np.asarray(x, np.float32))


def bf16_to_f32(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- encoder
def test_encode_inverts_the_format_table():
    codes = np.arange(256, dtype=np.uint8)
    finite = codes[(codes & 0x7F) != 0x7F]
    assert (fp8.encode(fp8.decode(finite).astype(np.float32)) == finite).all()


def test_encode_ties_and_neighbours():
    pos = fp8.TABLE[:127]
    mid = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)          # exact in float32
    assert (mid.astype(np.float64) == (pos[:-1] + pos[1:]) / 2).all()
    lower = np.arange(126)
    even = np.where(lower % 2 == 0, lower, lower + 1)
    assert (fp8.encode(mid) == even).all()
    assert (fp8.encode(-mid) == (even | 0x80)).all()
    assert (fp8.encode(np.nextafter(mid, np.float32(0))) == lower).all()
    assert (fp8.encode(np.nextafter(mid, np.float32(np.inf))) == lower + 1).all()
    # no value above 448: saturate; signed zero keeps its sign
    assert fp8.encode(np.float32([448, 463.9, 464, 1e30, -1e30])).tolist() == [126, 126, 126, 126, 254]
    assert fp8.encode(np.float32([0.0, -0.0, 2.0 ** -11, -(2.0 ** -11)])).tolist() == [0, 128, 0, 128]


def test_encode_agrees_with_the_generators_encoder():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(300000) * rng.choice([1e-3, 0.02, 1, 30, 300], 300000)).astype(np.float32)
    assert (fp8.encode(x) == gen.e4m3_encode(x)).all()


# ---------------------------------------------------------------- ingest
def _empty_pool(nblk, hkv, bsz, d, kv_dtype):
    kv = np.full((nblk, hkv, 2, bsz, d), gen.POISON[kv_dtype], dtype=gen.STORAGE[kv_dtype])
    scales = np.full((nblk, hkv, 2), np.nan, np.float32) if kv_dtype == "fp8_e4m3" else None
    return kv, scales


@pytest.mark.parametrize("kv_dtype", ["bf16", "f32"])
def test_ingest_plain_formats_round_trip(kv_dtype):
    rng = np.random.default_rng(0)
    length, hkv, d, bsz = 37, 2, 8, 16
    k = rng.standard_normal((length, hkv, d)).astype(np.float32)
    v = rng.standard_normal((length, hkv, d)).astype(np.float32)
    ks, vs = (k, v) if kv_dtype == "f32" else (bf16(k), bf16(v))
    kv, _ = _empty_pool(9, hkv, bsz, d, kv_dtype)
    ids = [7, 2, 5]
    ku.ingest_segment(kv, None, kv_dtype, ids, ks, vs)
    kk, vv = oa.gather_segment(kv, None, kv_dtype, ids, length)
    assert (kk == oa.widen(ks, kv_dtype)).all() and (vv == oa.widen(vs, kv_dtype)).all()
    # the padding of the last block and every other block are untouched
    poison = gen.POISON[kv_dtype]
    tail = kv[5, :, :, length - 32:, :]
    assert np.isnan(tail).all() if kv_dtype == "f32" else (tail == poison).all()
    others = kv[[0, 1, 3, 4, 6, 8]]
    assert np.isnan(others).all() if kv_dtype == "f32" else (others == poison).all()


def test_ingest_e4m3_matches_the_generators_quantiser():
    rng = np.random.default_rng(1)
    length, hkv, d, bsz = 53, 3, 16, 16
    k = bf16_to_f32(bf16(rng.standard_normal((length, hkv, d)) * np.exp2(rng.uniform(-3, 3, (length, 1, 1)))))
    v = bf16_to_f32(bf16(rng.standard_normal((length, hkv, d))))
    kv, scales = _empty_pool(6, hkv, bsz, d, "fp8_e4m3")
    ids = [4, 0, 3, 1]
    ku.ingest_segment(kv, scales, "fp8_e4m3", ids, bf16(k), bf16(v))
    for which, x in ((0, k), (1, v)):
        codes, sc = gen._quantise_tiles(x, bsz)                   # independent implementation
        for i, blk in enumerate(ids):
            n = min(bsz, length - i * bsz)
            assert (scales[blk, :, which] == sc[i]).all()
            assert (kv[blk, :, which, :n, :] == codes[i * bsz:i * bsz + n].transpose(1, 0, 2)).all()
            assert (kv[blk, :, which, n:, :] == 0x7F).all()       # padding untouched


def test_ingest_e4m3_bounds_and_extremes():
    rng = np.random.default_rng(2)
    length, hkv, d, bsz = 32, 2, 32, 16
    k = bf16_to_f32(bf16(rng.standard_normal((length, hkv, d))))
    v = k.copy()
    v[16:, 1, :] = 0.0                                            # an all-zero tile
    kv, scales = _empty_pool(2, hkv, bsz, d, "fp8_e4m3")
    ku.ingest_segment(kv, scales, "fp8_e4m3", [1, 0], bf16(k), bf16(v))
    assert scales[0, 1, 1] == 1.0 and (kv[0, 1, 1] == 0).all()
    for i, blk in enumerate([1, 0]):
        for h in range(hkv):
            x = k[i * bsz:(i + 1) * bsz, h, :].astype(np.float64)
            s = float(scales[blk, h, 0])
            assert s == float(np.float32(np.abs(x).max()) / np.float32(448))
            deq = fp8.decode(kv[blk, h, 0]) * s
            y = np.abs(x) / s
            half_step = np.maximum(np.exp2(np.floor(np.log2(np.maximum(y, 2.0 ** -6))) - 4), 2.0 ** -10)
            assert (np.abs(deq - x) <= s * half_step * (1 + 1e-6)).all()
            top = np.abs(x) == np.abs(x).max()
            assert ((kv[blk, h, 0][top] & 0x7F) == 0x7E).all()   # the largest magnitude lands on 448


# ---------------------------------------------------------------- append
def _append_all(kv, scales, kv_dtype, blk, k_rows, v_rows, bsz):
    for slot in range(k_rows.shape[0]):
        ku.append_token(kv, scales, kv_dtype, blk * bsz + slot, k_rows[slot], v_rows[slot])


def test_append_plain_formats_store_the_bits():
    rng = np.random.default_rng(4)
    hkv, d, bsz = 2, 8, 4
    k = bf16(rng.standard_normal((bsz, hkv, d)))
    v = bf16(rng.standard_normal((bsz, hkv, d)))
    kv, _ = _empty_pool(3, hkv, bsz, d, "bf16")
    _append_all(kv, None, "bf16", 2, k[:3], v[:3], bsz)
    assert (kv[2, :, 0, :3] == k[:3].transpose(1, 0, 2)).all() and (kv[2, :, 1, :3] == v[:3].transpose(1, 0, 2)).all()
    assert (kv[2, :, :, 3] == 0x7FC0).all() and (kv[:2] == 0x7FC0).all()


def test_append_with_the_largest_token_first_equals_ingest():
    """If the first token of a tile has the largest magnitude the scale never changes, so token-by-token
    appends must store exactly what a whole-tile ingest stores."""
    rng = np.random.default_rng(5)
    hkv, d, bsz = 3, 16, 16
    k = rng.standard_normal((bsz, hkv, d)).astype(np.float32)
    v = rng.standard_normal((bsz, hkv, d)).astype(np.float32)
    k[0] *= 40.0
    v[0] *= 40.0
    kb, vb = bf16(k), bf16(v)
    kv_a, sc_a = _empty_pool(2, hkv, bsz, d, "fp8_e4m3")
    kv_b, sc_b = _empty_pool(2, hkv, bsz, d, "fp8_e4m3")
    _append_all(kv_a, sc_a, "fp8_e4m3", 1, kb, vb, bsz)
    ku.ingest_segment(kv_b, sc_b, "fp8_e4m3", [1], kb, vb)
    assert (kv_a == kv_b).all() and (sc_a[1] == sc_b[1]).all()


def test_append_scale_growth_properties():
    rng = np.random.default_rng(6)
    hkv, d, bsz = 2, 32, 16
    gains = np.exp2(np.linspace(-3, 3, bsz)).astype(np.float32)              # every token louder than the last
    k = bf16(rng.standard_normal((bsz, hkv, d)).astype(np.float32) * gains[:, None, None])
    v = bf16(rng.standard_normal((bsz, hkv, d)).astype(np.float32) * gains[::-1, None, None])  # V: quieter and quieter
    kv, sc = _empty_pool(1, hkv, bsz, d, "fp8_e4m3")
    kf, vf = bf16_to_f32(k), bf16_to_f32(v)
    for slot in range(bsz):
        before_codes, before_sc = kv.copy(), sc.copy()
        ku.append_token(kv, sc, "fp8_e4m3", slot, k[slot], v[slot])
        for which, xf in ((0, kf), (1, vf)):
            for h in range(hkv):
                cand = np.float32(np.float32(np.abs(xf[slot, h]).max()) / np.float32(448))
                want = cand if slot == 0 else max(before_sc[0, h, which], cand)
                assert sc[0, h, which] == want
                if slot and sc[0, h, which] == before_sc[0, h, which]:
                    assert (kv[0, h, which, :slot] == before_codes[0, h, which, :slot]).all()   # untouched bits
                elif slot:
                    old = fp8.decode(before_codes[0, h, which, :slot]) * float(before_sc[0, h, which])
                    new = fp8.decode(kv[0, h, which, :slot]) * float(sc[0, h, which])
                    y = np.abs(old) / float(sc[0, h, which])
                    half_step = np.maximum(np.exp2(np.floor(np.log2(np.maximum(y, 2.0 ** -6))) - 4), 2.0 ** -10)
                    assert (np.abs(new - old) <= float(sc[0, h, which]) * half_step * (1 + 1e-5)).all()
    # K grew with every token: final scale and the last token's codes are those of a whole-tile ingest
    kv_i, sc_i = _empty_pool(1, hkv, bsz, d, "fp8_e4m3")
    ku.ingest_segment(kv_i, sc_i, "fp8_e4m3", [0], k, v)
    assert (sc[0] == sc_i[0]).all()
    assert (kv[0, :, 0, bsz - 1] == kv_i[0, :, 0, bsz - 1]).all()
    # V never grew after its first token: everything equals the ingest
    assert (kv[0, :, 1] == kv_i[0, :, 1]).all()


def _scalar_encode(y: np.float32) -> int:
    """Nearest e4m3 value by exhaustive search over the 127 magnitudes (ties: even code)."""
    mag = abs(float(y))
    best = min(range(127), key=lambda c: (abs(fp8.decode_code(c) - mag), c % 2))
    return best | (0x80 if np.signbit(y) else 0)


def test_append_against_scalar_brute_force():
    rng = np.random.default_rng(7)
    bsz, d = 4, 4
    x = (rng.standard_normal((bsz, d)) * np.array([1.0, 0.5, 3.0, 7.0])[:, None]).astype(np.float32)
    x[1, 2] = 0.0
    xb = bf16(x)
    xf = bf16_to_f32(xb)
    kv, sc = _empty_pool(1, 1, bsz, d, "fp8_e4m3")
    codes, scale = [], None
    for slot in range(bsz):
        ku.append_token(kv, sc, "fp8_e4m3", slot, xb[slot][None], xb[slot][None])
        a = np.float32(max(abs(float(t)) for t in xf[slot]))
        cand = np.float32(a / np.float32(448))
        new = (cand if a > 0 else np.float32(1)) if slot == 0 else max(scale, cand)
        if slot and new != scale:
            codes = [[_scalar_encode(np.float32(np.float32(np.float32(fp8.decode_code(c)) * scale) / new)) for c in row] for row in codes]
        scale = new
        codes.append([_scalar_encode(np.float32(t / scale)) for t in xf[slot]])
        assert sc[0, 0, 0] == scale and sc[0, 0, 1] == scale
        assert kv[0, 0, 0, :slot + 1].tolist() == codes and kv[0, 0, 1, :slot + 1].tolist() == codes


def test_attention_after_appends_sees_the_concatenation():
    """Eq. 4 / Eq. 6: the cache after T steps is the old cache followed by the T new tokens."""
    w = wl.named_workload("tiny")
    g = w.geometry
    pool = ol.BlockPool(w.num_blocks + 4, None)
    lay = ol.build_layout(pool, g.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    data = wl.fill_pool(w, lay.prefix_blk_indptr, lay.prefix_blk, lay.suffix_blk_indptr, lay.suffix_blk)
    grown = np.full((w.num_blocks + 4,) + data.kv.shape[1:], np.nan, np.float32)
    grown[:w.num_blocks] = data.kv
    steps = 11                                                   # crosses a block boundary (Ls = 8, B = 16)
    new_k, new_v = [], []
    for t in range(steps):
        k_t, v_t = w.step_tokens(t)
        dest = ol.append_step(pool, lay)
        for r in range(w.num_requests):
            ku.append_token(grown, None, g.kv_dtype, dest[r], k_t[r], v_t[r])
        new_k.append(k_t)
        new_v.append(v_t)
    q = oa.widen(w.q_bits(), g.q_dtype)
    for r in range(w.num_requests):
        p = int(w.req_prompt[r])
        seg_p, seg_s = w.prefix_kv(p), w.suffix_kv(r)
        k_all = np.concatenate([seg_p.k, seg_s.k] + [nk[r][None] for nk in new_k]).astype(np.float64)
        v_all = np.concatenate([seg_p.v, seg_s.v] + [nv[r][None] for nv in new_v]).astype(np.float64)
        o_ref, lse_ref = oa.attention_state(q[r], k_all, v_all)
        k_got, v_got = oa.request_kv(grown, None, g.kv_dtype, lay, r)
        assert (k_got == k_all).all() and (v_got == v_all).all()
        o, lse = oa.attention_state(q[r], k_got, v_got)
        assert np.allclose(o, o_ref, atol=1e-12) and np.allclose(lse, lse_ref, atol=1e-12)


# ---------------------------------------------------------------- table growth
def test_append_step_hand_worked():
    g = json.load(open(GOLDEN))
    pool = ol.BlockPool(g["num_blocks"], g["free_order"])
    lay = ol.build_layout(pool, g["block_size"], g["prefix_len"], g["req_prompt"], g["req_model"], g["suffix_len"])
    prefix_before = (lay.prefix_blk_indptr.tolist(), lay.prefix_blk.tolist())
    for step in g["append"]["steps"]:
        if step.get("out_of_blocks"):
            snapshot = (lay.suffix_len.tolist(), lay.suffix_blk.tolist(), pool.refcount.tolist(), list(pool.free))
            with pytest.raises(ol.OutOfBlocks):
                ol.append_step(pool, lay, step["active"])
            assert snapshot == (lay.suffix_len.tolist(), lay.suffix_blk.tolist(), pool.refcount.tolist(), list(pool.free))
            continue
        dest = ol.append_step(pool, lay, step["active"])
        assert dest.tolist() == step["dest"]
        for name in ("suffix_len", "suffix_blk_indptr", "suffix_blk"):
            assert getattr(lay, name).tolist() == step[name], name
        assert pool.refcount.tolist() == step["refcount"] and list(pool.free) == step["free"]
    assert (lay.prefix_blk_indptr.tolist(), lay.prefix_blk.tolist()) == prefix_before
    assert int((pool.refcount > 0).sum()) == g["append"]["blocks_used_eq9_after"]
    ol.release_layout(pool, lay)
    assert list(pool.free) == g["append"]["free_after_release"] and not pool.refcount.any()


@pytest.mark.parametrize("name", ["tiny", "b8"])
def test_append_step_keeps_eq9(name):
    w = wl.named_workload(name)
    b = w.geometry.block_size
    extra = w.num_requests * 3
    pool = ol.BlockPool(w.num_blocks + extra, np.concatenate([w.free_order, np.arange(w.num_blocks, w.num_blocks + extra)]))
    lay = ol.build_layout(pool, b, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    rng = np.random.default_rng(0)
    seen = set()
    for t in range(2 * b + 1):
        active = rng.random(w.num_requests) < 0.8
        before = lay.suffix_len.copy()
        head = list(pool.free)
        dest = ol.append_step(pool, lay, active)
        assert (lay.suffix_len == before + active).all()
        took = [r for r in range(w.num_requests) if active[r] and before[r] % b == 0]
        assert list(pool.free) == head[len(took):]                 # blocks leave from the head, in request order
        for i, r in enumerate(took):
            assert lay.suffix_blk[lay.suffix_blk_indptr[r + 1] - 1] == head[i]
        assert (dest[~active] == -1).all()
        for r in np.nonzero(active)[0]:
            blk, slot = divmod(int(dest[r]), b)
            assert slot == before[r] % b and blk == lay.suffix_blk[lay.suffix_blk_indptr[r] + before[r] // b]
            assert dest[r] not in seen                             # no slot is handed out twice
            seen.add(int(dest[r]))
        used = int(((w.prefix_len.astype(np.int64) + b - 1) // b).sum() + ((lay.suffix_len.astype(np.int64) + b - 1) // b).sum())
        assert int((pool.refcount > 0).sum()) == used               # Eq. 9 with the grown private lengths
        assert (pool.refcount[lay.suffix_blk] == 1).all()
    ol.release_layout(pool, lay)
    assert not pool.refcount.any() and sorted(pool.free) == list(range(pool.num_blocks))
