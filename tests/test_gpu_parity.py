"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element by element.

Bars: block tables bit-exact (checked when a case is set up); fp32 inputs max-abs and relative RMS
<= 1e-5; bf16 / fp8 inputs max-abs <= 1e-2 and relative RMS <= 5e-3 (fp32 accumulation).
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as oa

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from gpu_helpers import GpuCase
    return GpuCase


def _check(case, requests=None, label="", short_rows=False):
    """short_rows: the case has rows that see only a handful of tokens, so some |O| exceed 1 (see the helper)."""
    from gpu_helpers import check_against_oracle
    return check_against_oracle(case, requests, label, scaled_bar=short_rows)


def _variants(w):
    g = w.geometry
    spb = g.block_size // 16
    mfma = g.q_dtype == "bf16" and g.kv_dtype != "f32" and g.head_dim == 128 and g.block_size % 16 == 0 and spb & (spb - 1) == 0
    return ["wave", "mfma"] if mfma else ["wave"]


def test_tiny_fp32_default_and_split(gpu):
    case = gpu(wl.named_workload("tiny"))
    case.poison_workspace()
    case.batch.decode_attention()
    _check(case, label="tiny default plan")
    for pc, sc in ((32, 32), (64, 32), (96, 4096)):
        case.replan(pc, sc)
        case.poison_workspace()
        case.batch.decode_attention()
        _check(case, label=f"tiny chunks {pc}/{sc}")
    case.close()


def test_separate_passes_and_partial_states(gpu):
    """ps_prefix_attention / ps_suffix_attention partial states, merged per segment, match the oracle's segment states."""
    from paper_2602_12029_amd import binding as B
    w = wl.named_workload("tiny", seed=2)
    case = gpu(w)
    case.replan(64, 32)
    case.poison_workspace()
    case.batch.prefix_attention()
    case.batch.suffix_attention()
    case.batch.merge_states()
    _check(case, label="tiny three calls")
    o_ws, lse_ws = [x.cpu().double().numpy() for x in case.batch.workspace_views()]
    assert np.isfinite(o_ws).all()                                   # every slot was written
    plan = B.ps_layout_plan(case.layout, w.num_requests)
    g = w.geometry
    (op, lp), (os_, ls) = oa.segment_states(case.q_bits, g.q_dtype, case.data.kv, case.data.scales, g.kv_dtype, case.olay)
    for r in range(w.num_requests):
        s0, s1 = plan["slot_base"][r], plan["slot_base"][r + 1]
        n_pre = 4                                                    # 256 tokens in chunks of 64
        mo, ml = oa.merge_states(o_ws[s0:s0 + n_pre], lse_ws[s0:s0 + n_pre])
        assert np.abs(mo - op[r]).max() < 1e-5 and np.abs(ml - lp[r]).max() < 1e-5
        mo, ml = oa.merge_states(o_ws[s0 + n_pre:s1], lse_ws[s0 + n_pre:s1])
        assert np.abs(mo - os_[r]).max() < 1e-5 and np.abs(ml - ls[r]).max() < 1e-5
    case.close()


@pytest.mark.parametrize("name", ["ragged_bf16", "many_models", "ragged_fp8"])
def test_kv_cache_policies_give_the_same_bits(gpu, name):
    """Streamed (non-temporal) and cacheable K/V loads are the same arithmetic: outputs agree bit for bit, and with
    the oracle; the automatic choice is one of the two."""
    from paper_2602_12029_amd import binding as B
    spec = next(s for s in RAGGED if s[0] == name)
    _, geo, models, prefix, membership, suffix = spec
    w = wl.make_workload(name, geo, models, prefix, membership, suffix, pool_factor=1.5, seed=23)
    case = gpu(w)
    outs = {}
    for policy in (B.PS_KV_POLICY_STREAM, B.PS_KV_POLICY_CACHEABLE, B.PS_KV_POLICY_AUTO):
        case.replan(prefix_variant="mfma", suffix_variant="mfma", kv_cache_policy=policy)
        case.poison_workspace()
        case.batch.decode_attention()
        _check(case, label=f"{name} policy {policy}", short_rows=True)
        outs[policy] = (case.batch.out.clone(), case.batch.lse.clone())
    for policy in (B.PS_KV_POLICY_CACHEABLE, B.PS_KV_POLICY_AUTO):
        assert torch.equal(outs[policy][0].view(torch.int16), outs[B.PS_KV_POLICY_STREAM][0].view(torch.int16))
        assert torch.equal(outs[policy][1].view(torch.int32), outs[B.PS_KV_POLICY_STREAM][1].view(torch.int32))
    case.close()


def test_merge_states_alone_on_caller_built_workspace(gpu):
    w = wl.named_workload("tiny", seed=3)
    case = gpu(w)
    case.replan(32, 32)
    o_ws, lse_ws = case.batch.workspace_views()
    gen = torch.Generator().manual_seed(5)
    o_host = torch.randn(o_ws.shape, generator=gen)
    lse_host = torch.randn(lse_ws.shape, generator=gen) * 3
    lse_host[1] = float("-inf")                                      # an empty partial state
    o_host[1] = 0
    o_ws.copy_(o_host)
    lse_ws.copy_(lse_host)
    case.batch.merge_states()
    torch.cuda.synchronize()
    from paper_2602_12029_amd import binding as B
    plan = B.ps_layout_plan(case.layout, w.num_requests)
    got_o, got_lse = case.batch.out.cpu().double().numpy(), case.batch.lse.cpu().double().numpy()
    for r in range(w.num_requests):
        s0, s1 = plan["slot_base"][r], plan["slot_base"][r + 1]
        ro, rl = oa.merge_states(o_host[s0:s1].double().numpy(), lse_host[s0:s1].double().numpy())
        assert np.abs(got_o[r] - ro).max() < 1e-5 and np.abs(got_lse[r] - rl).max() < 1e-5
    case.close()


RAGGED = [
    # name, geometry, models, prefix_len, membership, suffix_len
    ("ragged_f32", wl.Geometry(4, 2, 64, 16, "f32", "f32"), 3, [1, 130, 517], [[0], [0, 2], [0, 1, 2]],
     [0, 33, 1, 16, 0, 250]),
    ("ragged_bf16", wl.Geometry(32, 8, 128, 16, "bf16", "bf16"), 4, [700, 31, 1025], [[0, 1, 2, 3], [1], [0, 3]],
     [5, 0, 129, 64, 17, 1, 300]),
    ("ragged_fp8", wl.Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3"), 4, [515, 48], [[0, 1, 2, 3], [2, 3]],
     [1, 47, 0, 200, 16, 33]),
    ("block32_bf16", wl.Geometry(8, 2, 128, 32, "bf16", "bf16"), 2, [333, 64], [[0, 1], [1]], [40, 0, 97]),
    ("d64_bf16", wl.Geometry(8, 2, 64, 16, "bf16", "bf16"), 2, [200], [[0, 1]], [9, 70]),
    ("d256_f32", wl.Geometry(4, 1, 256, 16, "f32", "f32"), 2, [100], [[0, 1]], [3, 40]),
    ("many_models", wl.Geometry(32, 2, 128, 16, "bf16", "bf16"), 10, [300], [list(range(10))], list(range(1, 11))),
    ("block64_fp8", wl.Geometry(16, 2, 128, 64, "bf16", "fp8_e4m3"), 3, [450, 64], [[0, 1, 2], [1]], [70, 1, 200, 129]),
    ("block48_bf16", wl.Geometry(8, 2, 128, 48, "bf16", "bf16"), 2, [200], [[0, 1]], [50, 7]),
]


@pytest.mark.parametrize("spec", RAGGED, ids=[s[0] for s in RAGGED])
def test_ragged_shapes(gpu, spec):
    name, geo, models, prefix, membership, suffix = spec
    w = wl.make_workload(name, geo, models, prefix, membership, suffix, pool_factor=1.5, seed=17)
    case = gpu(w)
    for variant in _variants(w):
        for pc, sc in ((0, 0), (64, 32), (256, 96)):
            case.replan(pc, sc, variant, variant)
            case.poison_workspace()
            case.batch.decode_attention()
            _check(case, label=f"{name} {variant} chunks {pc}/{sc}", short_rows=True)
    case.close()


@pytest.mark.parametrize("pool_layout", ["token_major", "planes"])
@pytest.mark.parametrize("spec", [RAGGED[0], RAGGED[1], RAGGED[2], RAGGED[7]], ids=lambda s: s[0])
def test_pool_layouts_through_the_strides(gpu, spec, pool_layout):
    """The pool is addressed through the four strides only: the same bits in two other physical layouts (all heads of
    a token side by side; K and V caches a whole pool apart) give the same attention, on both kernel families."""
    name, geo, models, prefix, membership, suffix = spec
    w = wl.make_workload(name, geo, models, prefix, membership, suffix, pool_factor=1.5, seed=23)
    case = gpu(w, pool_layout=pool_layout)
    for variant in _variants(w):
        for pc, sc in ((0, 0), (64, 32)):
            case.replan(pc, sc, variant, variant)
            case.poison_workspace()
            case.batch.decode_attention()
            _check(case, label=f"{name} {pool_layout} {variant} chunks {pc}/{sc}", short_rows=True)
    case.close()


def test_long_item_lists_per_workgroup(gpu):
    """Few workgroups, hundreds of small items each: the persistent kernel's item pipeline, its header ring
    refills and every kind of item boundary (waves without a tile, one-tile items, ragged tails)."""
    geo = wl.Geometry(32, 8, 128, 16, "bf16", "bf16")
    rng = np.random.default_rng(23)
    w = wl.make_workload("lists", geo, 3, [1999, 700, 33, 1024, 2500, 64], [[0, 1, 2]] * 6,
                         rng.integers(0, 200, 18).tolist(), pool_factor=1.3, seed=23)
    case = gpu(w)
    from paper_2602_12029_amd import binding as B
    for pc, sc, cus in ((64, 32, 1), (32, 32, 2), (128, 64, 3)):
        case.replan(pc, sc, "mfma", "mfma", num_cus=cus)
        sch = B.ps_layout_schedule(case.layout, 2)
        if cus <= 2:
            assert np.diff(sch["indptr"]).max() > 128      # more items per workgroup than the header ring holds
        case.poison_workspace()
        case.batch.decode_attention()
        _check(case, label=f"lists chunks {pc}/{sc} on {cus} CU", short_rows=True)
    case.close()


def test_request_without_tokens_gives_zero_and_neg_inf(gpu):
    geo = wl.Geometry(4, 2, 64, 16, "f32", "f32")
    w = wl.make_workload("empty", geo, 2, [0, 40], [[0], [0, 1]], [0, 0, 3], seed=19)
    case = gpu(w)
    case.poison_workspace()
    case.batch.decode_attention()
    torch.cuda.synchronize()
    assert not case.batch.out[0].any() and torch.isneginf(case.batch.lse[0]).all()
    _check(case)
    case.close()


@pytest.mark.parametrize("name", ["b8", "fp8_70b", "long", "mixed", "sessions40"])
def test_full_size_all_outputs(gpu, name):
    """Full benchmark configurations (and one point of the concurrent-sessions sweep), default plan (the launch configuration bench.py times), every output of every
    request against the oracle at the literal bars; bitwise repeatable (no float atomics anywhere)."""
    w = wl.named_workload(name)
    case = gpu(w)
    case.poison_workspace()
    case.batch.decode_attention()
    torch.cuda.synchronize()
    first = case.batch.out.clone()
    case.batch.decode_attention()
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), case.batch.out.view(torch.int16))
    _check(case)
    case.close()


def test_read_probe_runs_every_pattern_and_refuses_bad_arguments(gpu):
    """ps_probe_read is a measurement aid: every footprint runs to completion on a buffer with a ragged tail (only
    whole 8 KiB units are read), and bad arguments are refused before anything is launched."""
    from paper_2602_12029_amd import binding as B
    buf = torch.zeros(3 * 8192 + 100, dtype=torch.uint8, device="cuda:0")
    stream = int(torch.cuda.current_stream().cuda_stream)
    for pattern in range(4):
        for wgs in (1, 7):
            B.ps_probe_read(buf.data_ptr(), buf.numel(), pattern, wgs, stream)
    B.ps_probe_read(buf.data_ptr(), 100, 0, 4, stream)          # less than one unit: nothing to read
    pow2 = torch.zeros(4 * 8192, dtype=torch.uint8, device="cuda:0")
    for pattern in (4, 5, 6):                                   # scrambled chunk order: power-of-two chunk counts only
        B.ps_probe_read(pow2.data_ptr(), pow2.numel(), pattern, 3, stream)
    torch.cuda.synchronize()
    for bad in ((0, buf.numel(), 0, 4), (buf.data_ptr(), -1, 0, 4), (buf.data_ptr(), buf.numel(), 7, 4),
                (buf.data_ptr(), buf.numel(), 4, 4),
                (buf.data_ptr(), buf.numel(), 0, 0), (buf.data_ptr() + 8, buf.numel() - 8, 0, 4)):
        with pytest.raises(B.PsError):
            B.ps_probe_read(*bad, stream)
    torch.cuda.synchronize()
