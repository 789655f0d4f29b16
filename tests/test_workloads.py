"""Input generators: formats and determinism (CPU)."""
import numpy as np
import pytest
import torch

import workloads as wl


def test_bf16_rounding_matches_library():
    x = np.random.default_rng(1).standard_normal(100000).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]   # ties (to even) and a subnormal
    bits = wl.bf16_bits_from_f32(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)


def test_e4m3_encode_matches_library_and_saturates():
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(200000) * 100, rng.standard_normal(50000) * 0.01,
                        [0.0, -0.0, 448.0, 449.0, 463.9, 1e6, -1e6, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10]]).astype(np.float32)
    codes = wl.e4m3_encode(x)
    inside = np.abs(x) <= 448
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(codes[inside], ref[inside])
    assert np.all((codes[~inside] & 0x7F) == 0x7E)            # saturate, never NaN
    assert codes[np.argmax(x == np.float32(2.0 ** -10))] == 0  # tie between 0 and 2^-9 goes to even (0)
    assert codes[-1] == 2                                      # 3*2^-10 ties between codes 1 and 2 -> even


def test_named_shapes():
    t = wl.named_workload("tiny")
    assert t.num_requests == 2 and t.num_prompts == 1 and t.blocks_needed() == 18
    assert wl.ideal_bytes(t) == 262144 + 16384 + 4096
    assert sorted(t.free_order.tolist()) == list(range(18))
    b = wl.named_workload("b8")
    assert b.num_requests == 128 and b.suffix_len.min() >= 1 and b.suffix_len.max() <= 512
    lo = wl.named_workload("long")
    assert lo.num_blocks == int(np.ceil(1.5 * lo.blocks_needed()))
    mx = wl.named_workload("mixed")
    sizes = np.bincount(mx.req_prompt, minlength=256)
    assert sizes.min() >= 2 and sizes.max() <= 6 and mx.prefix_len.min() >= 512 and mx.prefix_len.max() <= 16384
    f8 = wl.named_workload("fp8_70b")
    assert f8.geometry.group == 8 and f8.geometry.token_bytes == 2048


def test_streams_are_reproducible_and_independent():
    a = wl.named_workload("tiny", seed=3)
    b = wl.named_workload("tiny", seed=3)
    assert np.array_equal(a.q_bits(), b.q_bits())
    assert np.array_equal(a.suffix_kv(1).v, b.suffix_kv(1).v)
    assert not np.array_equal(a.suffix_kv(0).k, a.suffix_kv(1).k)
    assert not np.array_equal(a.q_bits(), wl.named_workload("tiny", seed=4).q_bits())


def test_fp8_segment_scales():
    geo = wl.Geometry(2, 1, 16, 16, "bf16", "fp8_e4m3")
    w = wl.make_workload("x", geo, 1, [40], [[0]], [3], seed=5)
    seg = w.prefix_kv(0)
    assert seg.k.dtype == np.uint8 and seg.k_scale.shape == (3, 1)
    # the largest magnitude of every tile lands exactly on +-448
    for b in range(3):
        tile = seg.k[b * 16:(b + 1) * 16, 0]
        assert (tile & 0x7F).max() == 0x7E


def test_fill_pool_poisons_unowned_slots():
    geo = wl.Geometry(2, 1, 8, 4, "f32", "f32")
    w = wl.make_workload("x", geo, 1, [6], [[0]], [1], pool_factor=2.0, seed=6)
    pd = wl.fill_pool(w, [0, 2], [3, 1], [0, 1], [5])
    assert np.isnan(pd.kv[0]).all() and np.isnan(pd.kv[1, :, :, 2:]).all()
    assert np.array_equal(pd.kv[3, 0, 0], w.prefix_kv(0).k[:4, 0])
    assert np.array_equal(pd.kv[1, 0, 1, :2], w.prefix_kv(0).v[4:6, 0])
    assert np.array_equal(pd.kv[5, 0, 0, 0], w.suffix_kv(0).k[0, 0])
