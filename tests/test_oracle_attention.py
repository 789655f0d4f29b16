"""Pins for the fp64 attention oracle: brute force, closed forms, invariances, a library SDPA."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as oa
from oracle import layout as ol
from helpers import oracle_decode, oracle_setup


def _widen_with_library(bits, dtype):
    if dtype == "f32":
        return [float(x) for x in np.asarray(bits).ravel()], bits.shape
    if dtype == "bf16":
        t = torch.from_numpy(np.asarray(bits).view(np.int16).copy()).view(torch.bfloat16).double()
        return t.flatten().tolist(), bits.shape
    raise ValueError(dtype)


def _brute_force(w):
    """Dense attention over the *logical* sequences, explicit Python loops, math.exp only."""
    g = w.geometry
    G, d = g.group, g.head_dim
    qf, qs = _widen_with_library(w.q_bits(), g.q_dtype)
    out = np.zeros(qs)
    lse = np.zeros(qs[:2])

    def at(flat, shape, i, j, c):
        return flat[(i * shape[1] + j) * shape[2] + c]

    for r in range(w.num_requests):
        pre, suf = w.prefix_kv(int(w.req_prompt[r])), w.suffix_kv(r)
        toks = []
        for seg in (pre, suf):
            kf, ks = _widen_with_library(seg.k, g.kv_dtype)
            vf, _ = _widen_with_library(seg.v, g.kv_dtype)
            toks += [(kf, vf, ks, j) for j in range(ks[0])]
        for h in range(g.num_q_heads):
            kvh = h // G
            scores = []
            for kf, vf, ks, j in toks:
                scores.append(sum(at(qf, qs, r, h, c) * at(kf, ks, j, kvh, c) for c in range(d)) / math.sqrt(d))
            denom = sum(math.exp(s) for s in scores)            # tiny inputs: no overflow risk
            lse[r, h] = math.log(denom)
            for c in range(d):
                out[r, h, c] = sum(math.exp(s) / denom * at(vf, ks, j, kvh, c)
                                   for s, (kf, vf, ks, j) in zip(scores, toks))
    return out, lse


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16"])
def test_brute_force_on_tiny_inputs(kv_dtype):
    geo = wl.Geometry(4, 2, 8, 4, kv_dtype, kv_dtype)
    w = wl.make_workload("bf", geo, 3, [13, 6], [[0, 2], [1]], [5, 0, 3], pool_factor=1.5, seed=11)
    _, lay, data = oracle_setup(w)
    o, lse = oracle_decode(w, lay, data)
    bo, blse = _brute_force(w)
    assert np.abs(o - bo).max() < 1e-12 and np.abs(lse - blse).max() < 1e-12


def test_fp8_scales_enter_as_code_value_times_scale():
    geo = wl.Geometry(2, 1, 8, 4, "bf16", "fp8_e4m3")
    w = wl.make_workload("f8", geo, 1, [7], [[0]], [2], seed=12)
    _, lay, data = oracle_setup(w)
    k, v = oa.request_kv(data.kv, data.scales, "fp8_e4m3", lay, 0)
    seg = w.prefix_kv(0)
    lib = torch.from_numpy(seg.k.copy()).view(torch.float8_e4m3fn).double().numpy()
    for j in range(7):
        assert np.array_equal(k[j, 0], lib[j, 0] * float(seg.k_scale[j // 4, 0]))
    # dequantised values reproduce the N(0,1) source to e4m3 precision (relative step 2^-4 of the tile max)
    src = np.random.Generator(np.random.PCG64(np.random.SeedSequence([12, 5, 0]))).standard_normal((7, 1, 8), dtype=np.float32)
    assert np.abs(k[:7] - src).max() <= np.abs(src).max() * 2.0 ** -4


def test_placement_independence_is_bitwise():
    w = wl.named_workload("tiny", seed=5)
    _, lay1, d1 = oracle_setup(w)
    other = np.random.default_rng(99).permutation(w.num_blocks)
    _, lay2, d2 = oracle_setup(w, free_order=other)
    assert not np.array_equal(lay1.prefix_blk, lay2.prefix_blk)
    o1, l1 = oracle_decode(w, lay1, d1)
    o2, l2 = oracle_decode(w, lay2, d2)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_block_table_permutation_leaves_the_result():
    w = wl.named_workload("tiny", seed=6)
    _, lay, data = oracle_setup(w)
    o1, l1 = oracle_decode(w, lay, data)
    perm = np.random.default_rng(3).permutation(16)             # prefix is 16 full blocks
    lay.prefix_blk = lay.prefix_blk[perm]
    o2, l2 = oracle_decode(w, lay, data)
    assert np.abs(o1 - o2).max() < 1e-12 and np.abs(l1 - l2).max() < 1e-12


def test_split_and_merge_equals_unsplit():
    rng = np.random.default_rng(7)
    q = rng.standard_normal((4, 16))
    k = rng.standard_normal((50, 2, 16)) * 3
    v = rng.standard_normal((50, 2, 16))
    o, lse = oa.attention_state(q, k, v)
    for cuts in ([0, 50], [0, 1, 50], [0, 17, 17, 33, 50], [0, 0, 49, 50, 50]):
        parts = [oa.attention_state(q, k[a:b], v[a:b]) for a, b in zip(cuts[:-1], cuts[1:])]
        mo, ml = oa.merge_states(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]))
        assert np.abs(mo - o).max() < 1e-12 and np.abs(ml - lse).max() < 1e-12
    eo, el = oa.merge_states(np.zeros((2, 4, 16)), np.full((2, 4), -np.inf))
    assert not eo.any() and np.all(np.isneginf(el))
    zo, zl = oa.merge_states(np.zeros((0, 4, 16)), np.zeros((0, 4)))
    assert not zo.any() and np.all(np.isneginf(zl))


def test_merge_weights_against_a_hand_computed_case():
    # two states with lse ln1 and ln3 carry weights 1/4 and 3/4
    o, lse = oa.merge_states(np.array([[[4.0]], [[8.0]]]), np.array([[0.0], [math.log(3.0)]]))
    assert abs(o[0, 0] - 7.0) < 1e-14 and abs(lse[0] - math.log(4.0)) < 1e-14


def test_single_model_equals_library_sdpa():
    geo = wl.Geometry(8, 2, 32, 16, "bf16", "bf16")
    w = wl.make_workload("m1", geo, 1, [70, 33], [[0], [0]], [9, 16], seed=13)
    _, lay, data = oracle_setup(w)
    o, _ = oracle_decode(w, lay, data)
    q = torch.from_numpy(oa.widen(w.q_bits(), "bf16"))
    for r in range(2):
        k, v = oa.request_kv(data.kv, data.scales, "bf16", lay, r)
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(4, dim=0)     # [Hq, L, d]
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(4, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(q[r][:, None, :], kt, vt)[:, 0].numpy()
        assert np.abs(o[r] - ref).max() < 1e-10


def test_closed_forms():
    rng = np.random.default_rng(8)
    q = rng.standard_normal((4, 8))
    k = rng.standard_normal((9, 2, 8))
    v = rng.standard_normal((9, 2, 8))
    # one token: O = v, LSE = its score
    o, lse = oa.attention_state(q, k[:1], v[:1])
    assert np.abs(o - np.repeat(v[0], 2, axis=0)).max() < 1e-15
    assert np.abs(lse - np.array([q[h] @ k[0, h // 2] / math.sqrt(8) for h in range(4)])).max() < 1e-14
    # zero query: uniform weights
    o, lse = oa.attention_state(np.zeros((4, 8)), k, v)
    assert np.abs(o - np.repeat(v.mean(0), 2, axis=0)).max() < 1e-14 and np.abs(lse - math.log(9)).max() < 1e-14
    # constant values pass through
    o, _ = oa.attention_state(q, k, np.full((9, 2, 8), 2.5))
    assert np.abs(o - 2.5).max() < 1e-13
    # a dominant key takes all the weight
    kd = k.copy()
    kd[4, 0] = q[0] * 50
    o, _ = oa.attention_state(q, kd, v)
    assert np.abs(o[0] - v[4, 0]).max() < 1e-9
    # duplicating the KV set leaves O and adds log 2 to LSE
    o1, l1 = oa.attention_state(q, k, v)
    o2, l2 = oa.attention_state(q, np.concatenate([k, k]), np.concatenate([v, v]))
    assert np.abs(o1 - o2).max() < 1e-14 and np.abs(l2 - l1 - math.log(2)).max() < 1e-14
    # GQA mapping: q head h uses KV head h // group (changing KV head 1 leaves q heads 0, 1 alone)
    k2 = k.copy()
    k2[3, 1] += 1.0
    o3, _ = oa.attention_state(q, k2, v)
    assert np.array_equal(o3[:2], o1[:2]) and not np.allclose(o3[2:], o1[2:])
    # the scale is 1/sqrt(d): a large-norm query against two keys gives a sigmoid of the scaled gap
    qq = np.zeros((1, 4)); qq[0, 0] = 2.0
    kk = np.zeros((2, 1, 4)); kk[1, 0, 0] = 1.0
    vv = np.zeros((2, 1, 4)); vv[1, 0, 0] = 1.0
    o, _ = oa.attention_state(qq, kk, vv)
    assert abs(o[0, 0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15


def test_sharing_semantics():
    geo = wl.Geometry(4, 2, 16, 16, "f32", "f32")
    w = wl.make_workload("sh", geo, 2, [40], [[0, 1]], [5, 5], seed=14)
    _, lay, data = oracle_setup(w)
    q = w.q_bits().copy()
    q[1] = q[0]
    # give model 1 the same private tokens as model 0
    b0 = lay.suffix_blk[lay.suffix_blk_indptr[0]]
    b1 = lay.suffix_blk[lay.suffix_blk_indptr[1]]
    data.kv[b1] = data.kv[b0]
    o, _ = oa.decode_attention(q, "f32", data.kv, None, "f32", lay)
    assert np.array_equal(o[0], o[1])
    # both requests read the very same prefix blocks
    assert len(lay.prefix_blk) == 3
    # changing model 0's private tokens does not move model 1's output
    data.kv[b0, :, :, :5] += 1.0
    o2, _ = oa.decode_attention(q, "f32", data.kv, None, "f32", lay)
    assert np.array_equal(o2[1], o[1]) and not np.array_equal(o2[0], o[0])
    # changing a shared prefix token moves both
    data.kv[lay.prefix_blk[0], :, :, 0] += 1.0
    o3, _ = oa.decode_attention(q, "f32", data.kv, None, "f32", lay)
    assert not np.array_equal(o3[1], o2[1]) and not np.array_equal(o3[0], o2[0])


def test_segment_states_merge_to_the_whole():
    w = wl.named_workload("tiny", seed=9)
    _, lay, data = oracle_setup(w)
    g = w.geometry
    o, lse = oracle_decode(w, lay, data)
    (op, lp), (os_, ls) = oa.segment_states(w.q_bits(), g.q_dtype, data.kv, data.scales, g.kv_dtype, lay)
    mo, ml = oa.merge_states(np.stack([op, os_]), np.stack([lp, ls]))
    assert np.abs(mo - o).max() < 1e-13 and np.abs(ml - lse).max() < 1e-13


def test_slots_past_the_length_are_never_read():
    geo = wl.Geometry(2, 1, 8, 16, "bf16", "bf16")
    w = wl.make_workload("nan", geo, 2, [19], [[0, 1]], [1, 17], pool_factor=2.0, seed=15)
    _, lay, data = oracle_setup(w)
    o, lse = oracle_decode(w, lay, data)            # pool is NaN wherever no token lives
    assert np.isfinite(o).all() and np.isfinite(lse).all()
