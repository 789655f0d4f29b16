"""GPU: staging of a batch's KV blocks in host memory and their reload into other physical blocks -- the staged image
bit for bit against the oracle's, then the resumed batch's attention against the oracle on the oracle's own resumed
layout, same bars as the decode step."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layout as ol
from oracle import staging as ost

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from gpu_helpers import GpuCase
    return GpuCase


def _raw(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.uint8).numpy()


CASES = [
    ("stage_f32", wl.Geometry(4, 2, 64, 16, "f32", "f32"), False),
    ("stage_bf16", wl.Geometry(32, 8, 128, 16, "bf16", "bf16"), True),
    ("stage_fp8", wl.Geometry(64, 8, 128, 16, "bf16", "fp8_e4m3"), False),
    ("stage_fp8_block64_tree", wl.Geometry(16, 2, 128, 64, "bf16", "fp8_e4m3"), True),
]


@pytest.mark.parametrize("spec", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("host_image", [False, True], ids=["device_image", "pinned_host_image"])
def test_park_overwrite_resume(gpu, spec, host_image):
    from gpu_helpers import check_against_oracle
    from paper_2602_12029_amd import binding as B
    name, geo, tree = spec
    if tree:
        w = wl.make_tree_workload(name, geo, 3, [130], [0, -1, 0], [300, 31, 0], [[0, 1, 2], [1], [0, 2]],
                                  [5, 0, 129, 64, 17, 33], pool_factor=1.6, seed=67)
    else:
        w = wl.make_workload(name, geo, 3, [333, 48], [[0, 1, 2], [1]], [40, 0, 97, 16], pool_factor=1.6, seed=67)
    case = gpu(w)
    case.poison_workspace()
    case.batch.decode_attention()
    check_against_oracle(case, label=f"{name} before parking", scaled_bar=True)
    first = case.batch.out.clone()

    # stage out: the image equals the oracle's, bit for bit
    bb, scales_off, total = B.ps_stage_layout(case.layout)
    image = torch.zeros(total, dtype=torch.uint8, device="cpu", pin_memory=True) if host_image else \
        torch.zeros(total, dtype=torch.uint8, device="cuda:0")
    case.batch.stage_out(image)
    torch.cuda.synchronize()
    ref_kv, ref_scales = ost.stage_out(case.data.kv, case.data.scales, case.olay)
    got = _raw(image)
    assert np.array_equal(got[:ref_kv.nbytes], ref_kv.reshape(-1).view(np.uint8))
    if ref_scales is not None:
        assert np.array_equal(got[scales_off:scales_off + ref_scales.nbytes], ref_scales.reshape(-1).view(np.uint8))

    # park; the pool is used by somebody else meanwhile (everything overwritten, free list rotated on both sides)
    case.batch.park(case.pool)
    ost.park_layout(case.opool, case.olay)
    with pytest.raises(B.PsError) as e:
        case.batch.decode_attention()
    assert e.value.status == B.PS_ERR_INVALID_ARG
    case.batch.kv.view(torch.uint8).fill_(0x7f)
    if case.batch.scales is not None:
        case.batch.scales.fill_(float("nan"))
    other = B.ps_kv_layout(case.pool, case.geo, [3 * geo.block_size], [0], [0], [0])      # takes three blocks ...
    ol.build_layout(case.opool, geo.block_size, [3 * geo.block_size], [0], [0], [0])
    case.batch.resume(case.pool)                                                          # ... so these are others
    ost.resume_layout(case.opool, case.olay)
    t = B.ps_layout_tables(case.layout, w.num_prompts, w.num_requests)
    assert np.array_equal(t["prefix_blk"], case.olay.prefix_blk) and np.array_equal(t["suffix_blk"], case.olay.suffix_blk)
    case.batch.stage_in(image)
    torch.cuda.synchronize()
    # the oracle's pool gets the oracle's image back
    case.data.kv[:] = wl.generate.POISON[geo.kv_dtype]
    if case.data.scales is not None:
        case.data.scales[:] = np.nan
    ost.stage_in(case.data.kv, case.data.scales, case.olay, ref_kv, ref_scales)
    ids = ost.table_order(case.olay)
    pool_bits = _raw(case.batch.kv).reshape(case.data.kv.shape[0], -1)
    assert np.array_equal(pool_bits[ids], case.data.kv.reshape(case.data.kv.shape[0], -1).view(np.uint8)[ids])
    case.poison_workspace()
    case.batch.decode_attention()
    check_against_oracle(case, label=f"{name} after resume", scaled_bar=True)
    assert torch.equal(first.view(torch.uint8), case.batch.out.view(torch.uint8))        # same bits as before parking
    B.ps_layout_release(case.pool, other)
    case.close()
