"""GPU parity with a third sharing level (a context several prompts begin with, stored once and read by every request
below it): the HIP path through the C ABI against the fp64 oracle, element by element, same bars as the decode step."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import kv_update as ku

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from gpu_helpers import GpuCase
    return GpuCase


def _run(case, label, visible=None, requests=None, short_rows=True):
    """short_rows: the case has rows that see only a handful of tokens, so some |O| exceed 1 (see the helper)."""
    from gpu_helpers import check_against_oracle
    case.poison_workspace()
    case.batch.decode_attention()
    return check_against_oracle(case, requests, label, visible, scaled_bar=short_rows)


def _variants(w):
    g = w.geometry
    return ["wave", "mfma"] if (g.q_dtype == "bf16" and g.kv_dtype != "f32" and g.head_dim == 128) else ["wave"]


def test_tree_tiny_fp32(gpu):
    case = gpu(wl.named_tree_workload("tree_tiny"))
    for pc, sc in ((0, 0), (16, 16), (32, 4096)):
        case.replan(pc, sc)
        _run(case, f"tree_tiny chunks {pc}/{sc}")
    case.close()


TREES = [
    # name, geometry, models, root_len, prompt_root, prefix_len, membership, suffix_len
    ("tree_f32", wl.Geometry(4, 2, 64, 16, "f32", "f32"), 3, [70, 0], [0, -1, 1, 0], [1, 130, 40, 0],
     [[0], [0, 2], [1], [0, 1, 2]], [0, 33, 1, 16, 0, 250, 3]),
    ("tree_bf16", wl.Geometry(32, 8, 128, 16, "bf16", "bf16"), 4, [515, 100], [0, 0, 1, -1], [300, 31, 0, 700],
     [[0, 1, 2, 3], [1], [0, 3], [2]], [5, 0, 129, 64, 17, 1, 300, 40]),
    ("tree_fp8", wl.Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3"), 4, [333], [0, 0], [515, 48],
     [[0, 1, 2, 3], [2, 3]], [1, 47, 0, 200, 16, 33]),
    # 24 requests x 4 heads = 96 rows below the root: row-split root items on the matrix cores
    ("tree_wide_bf16", wl.Geometry(8, 2, 128, 16, "bf16", "bf16"), 3, [700], [0] * 8, [64, 0, 33, 200, 16, 90, 128, 1],
     [[0, 1, 2]] * 8, list(range(24))),
    ("tree_block64_fp8", wl.Geometry(16, 2, 128, 64, "bf16", "fp8_e4m3"), 3, [450, 64], [0, 1, 0], [70, 64, 0],
     [[0, 1, 2], [1], [0, 2]], [70, 1, 200, 129, 0, 5]),
]


@pytest.mark.parametrize("spec", TREES, ids=[s[0] for s in TREES])
def test_ragged_trees(gpu, spec):
    name, geo, models, root_len, prompt_root, prefix, membership, suffix = spec
    w = wl.make_tree_workload(name, geo, models, root_len, prompt_root, prefix, membership, suffix, pool_factor=1.5, seed=47)
    case = gpu(w)
    for variant in _variants(w):
        for pc, sc in ((0, 0), (64, 32), (256, 96)):
            case.replan(pc, sc, variant, variant)
            _run(case, f"{name} {variant} chunks {pc}/{sc}")
    # visible lengths cut the prompts' own prefixes, the roots stay whole
    rng = np.random.default_rng(53)
    visible = rng.integers(0, w.prefix_len[w.req_prompt] + 1)
    case.replan(64, 32)
    case.set_visible(visible)
    _run(case, f"{name} with visible lengths", visible)
    case.close()


def test_tree_b8_all_outputs(gpu):
    """Benchmark-sized three-level batch, default plan (the launch configuration bench.py times), every output."""
    w = wl.named_tree_workload("tree_b8")
    case = gpu(w)
    _run(case, "tree_b8", short_rows=False)
    first = case.batch.out.clone()
    case.batch.decode_attention()
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), case.batch.out.view(torch.int16))
    case.close()


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_root_ingest_bit_exact_then_attention(gpu, kv_dtype):
    """ps_kv_ingest(which = 2) stores the roots from a contiguous source: pool bits and scales equal the oracle's."""
    from paper_2602_12029_amd.runtime import to_device
    geo = wl.Geometry(16, 2, 128, 16, "bf16", kv_dtype)
    w = wl.make_tree_workload("ing", geo, 2, [100, 37], [0, 1, 0], [20, 64, 0], [[0, 1], [0], [1]], [3, 0, 18, 40],
                              pool_factor=1.2, seed=59)
    case = gpu(w)
    lay = case.olay
    src = [w.root_source(t) for t in range(w.num_roots)]                 # unquantised K, V per root
    kv_ref, sc_ref = case.data.kv.copy(), None if case.data.scales is None else case.data.scales.copy()
    for t in range(w.num_roots):
        ids = lay.root_blk[lay.root_blk_indptr[t]:lay.root_blk_indptr[t + 1]]
        ku.ingest_segment(kv_ref, sc_ref, kv_dtype, ids, src[t][0], src[t][1])
    src_k = to_device(np.concatenate([s[0] for s in src]), "bf16")
    src_v = to_device(np.concatenate([s[1] for s in src]), "bf16")
    case.batch.kv_ingest(2, src_k, src_v)
    torch.cuda.synchronize()
    got = case.batch.kv.cpu().view(torch.uint8 if kv_dtype == "fp8_e4m3" else torch.int16).numpy()
    ref = kv_ref.view(np.uint8 if kv_dtype == "fp8_e4m3" else np.int16)
    owned = np.zeros(kv_ref.shape[:1] + kv_ref.shape[2:4], bool)       # [block, K|V, slot]: slots of root tokens
    for t in range(w.num_roots):
        ids = lay.root_blk[lay.root_blk_indptr[t]:lay.root_blk_indptr[t + 1]]
        for j in range(int(w.root_len[t])):
            owned[ids[j // 16], :, j % 16] = True
    mask = np.broadcast_to(owned[:, None, :, :, None], ref.shape)
    assert np.array_equal(got.reshape(ref.shape)[mask], ref[mask])
    if kv_dtype == "fp8_e4m3":
        assert np.array_equal(case.batch.scales.cpu().numpy()[lay.root_blk], sc_ref[lay.root_blk])
    case.data.kv[:] = kv_ref                                               # the oracle now reads what was ingested
    if sc_ref is not None:
        case.data.scales[:] = sc_ref
    _run(case, f"after root ingest ({kv_dtype})")
    case.close()
