"""GPU parity with per-request visible prefix lengths (partial prefill of new context tokens against the shared
cache): the HIP path through the C ABI against the fp64 oracle, element by element, same bars as the decode step."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from gpu_helpers import GpuCase
    return GpuCase


def _run(case, visible, label, requests=None):
    from gpu_helpers import check_against_oracle
    case.poison_workspace()
    case.batch.decode_attention()
    return check_against_oracle(case, requests, label, visible, scaled_bar=True)   # rows that see a few tokens


def _variants(w):
    g = w.geometry
    return ["wave", "mfma"] if (g.q_dtype == "bf16" and g.kv_dtype != "f32" and g.head_dim == 128) else ["wave"]


def test_tiny_fp32_random_lengths(gpu):
    w = wl.named_workload("tiny")
    case = gpu(w)
    rng = np.random.default_rng(1)
    full = w.prefix_len[w.req_prompt]
    for trial, visible in enumerate([np.array([0, 256]), np.array([1, 255]), rng.integers(0, 257, 2), full]):
        for pc, sc in ((0, 0), (32, 32), (96, 4096)):
            case.replan(pc, sc)
            case.set_visible(visible)
            _run(case, visible, f"tiny visible {visible.tolist()} chunks {pc}/{sc}")
    case.set_visible(None)                                   # back to the plain decode step
    _run(case, None, "tiny, limits removed")
    case.close()


SHAPES = [
    ("vis_f32", wl.Geometry(4, 2, 64, 16, "f32", "f32"), 3, [1, 130, 517], [[0], [0, 2], [0, 1, 2]], [0, 33, 1, 16, 0, 250]),
    ("vis_bf16", wl.Geometry(32, 8, 128, 16, "bf16", "bf16"), 4, [700, 31, 1025], [[0, 1, 2, 3], [1], [0, 3]],
     [5, 0, 129, 64, 17, 1, 300]),
    ("vis_fp8", wl.Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3"), 4, [515, 48], [[0, 1, 2, 3], [2, 3]],
     [1, 47, 0, 200, 16, 33]),
    ("vis_block64_fp8", wl.Geometry(16, 2, 128, 64, "bf16", "fp8_e4m3"), 3, [450, 64], [[0, 1, 2], [1]], [70, 1, 200, 129]),
    ("vis_many_rows", wl.Geometry(32, 2, 128, 16, "bf16", "bf16"), 10, [300], [list(range(10))], list(range(0, 10))),
]


@pytest.mark.parametrize("spec", SHAPES, ids=[s[0] for s in SHAPES])
def test_random_lengths_with_private_suffixes(gpu, spec):
    """Requests that see random parts of their prompt's prefix (none and all included) and keep their own suffix."""
    name, geo, models, prefix, membership, suffix = spec
    w = wl.make_workload(name, geo, models, prefix, membership, suffix, pool_factor=1.5, seed=29)
    case = gpu(w)
    rng = np.random.default_rng(31)
    full = w.prefix_len[w.req_prompt]
    for trial in range(3):
        visible = rng.integers(0, full + 1)
        visible[trial % len(visible)] = 0
        visible[(trial + 1) % len(visible)] = full[(trial + 1) % len(visible)]
        for variant in _variants(w):
            for pc, sc in ((0, 0), (64, 32), (256, 96)):
                case.replan(pc, sc, variant, variant)
                case.set_visible(visible)
                _run(case, visible, f"{name} #{trial} {variant} chunks {pc}/{sc}")
    case.close()


def test_nothing_visible_and_no_suffix_gives_zero_and_neg_inf(gpu):
    geo = wl.Geometry(8, 2, 128, 16, "bf16", "bf16")
    w = wl.make_workload("blind", geo, 3, [100], [[0, 1, 2]], [0, 0, 5], seed=37)
    case = gpu(w)
    visible = np.array([0, 60, 0])
    for variant in ("wave", "mfma"):
        case.replan(32, 32, variant, variant)
        case.set_visible(visible)
        _run(case, visible, f"blind {variant}")
        assert not case.batch.out[0].float().any() and torch.isneginf(case.batch.lse[0]).all()
    case.close()


CHUNKS = [
    # name, geometry, cached lengths, chunk lengths
    ("chunk_f32", wl.Geometry(4, 2, 64, 16, "f32", "f32"), [40, 7, 0], [19, 30, 5]),
    ("chunk_bf16", wl.Geometry(32, 8, 128, 16, "bf16", "bf16"), [1000, 0, 333], [200, 70, 17]),
    ("chunk_fp8", wl.Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3"), [515, 2048], [100, 33]),
    ("chunk_block32_bf16", wl.Geometry(8, 2, 128, 32, "bf16", "bf16"), [300], [150]),
    # token ranges of one to four tiles, ending on, just before and just after a tile boundary, with 68 to 260 rows per
    # KV head: the first and last rounds of the prefill kernel's tile ring, waves without rows, partly filled row tiles
    ("chunk_edges_bf16", wl.Geometry(32, 8, 128, 16, "bf16", "bf16"), [0, 1, 31, 33, 64, 95], [17, 20, 33, 40, 64, 65]),
    ("chunk_edges_fp8_block32", wl.Geometry(64, 8, 128, 32, "bf16", "fp8_e4m3"), [0, 30, 63, 97], [9, 34, 33, 31]),
]


@pytest.mark.parametrize("spec", CHUNKS, ids=[s[0] for s in CHUNKS])
def test_causal_chunk_prefill(gpu, spec):
    """New context tokens prefilled against the cached context: token i of a chunk sees cached + i + 1 tokens."""
    name, geo, cached, chunk = spec
    w, visible = wl.chunk_prefill_workload(name, geo, cached, chunk, pool_factor=1.3, seed=41)
    case = gpu(w)
    for variant in _variants(w):
        for pc, sc in ((0, 0), (64, 32), (512, 96)):
            case.replan(pc, sc, variant, variant)
            case.set_visible(visible)
            _run(case, visible, f"{name} {variant} chunks {pc}/{sc}")
    case.close()


@pytest.mark.parametrize("name", ["prefill_b8", "prefill_fp8"])
def test_full_size_chunk_prefill_sampled_rows(gpu, name):
    """Benchmark-sized partial prefill, default plan: a seeded sample of query rows (first and last token of a
    chunk included) computed one by one by the oracle; every output finite; bitwise repeatable."""
    w, visible = wl.named_chunk_prefill(name)
    case = gpu(w)
    case.set_visible(visible)
    first_rows = np.flatnonzero(visible == visible.min())[:2].tolist()
    sample = sorted(set(np.random.default_rng(43).choice(w.num_requests, size=24, replace=False).tolist())
                    | set(first_rows) | {w.num_requests - 1})
    _run(case, visible, name, requests=sample)
    assert torch.isfinite(case.batch.out.float()).all()
    first = case.batch.out.clone()
    case.batch.decode_attention()
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), case.batch.out.view(torch.int16))
    case.close()
