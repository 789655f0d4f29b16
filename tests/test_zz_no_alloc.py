"""ps_decode_attention_static (the entry point for callers that cannot allocate: its partial states go to a buffer in
the library's device image) against ps_decode_attention on the same inputs, through the C ABI.

Both run the same kernels, so the outputs must agree bit for bit (and with the fp64 oracle at the usual bars).  Two
calls in a row share the one static buffer; the second batch is smaller than the first, so stale partial states of
the first call lie behind the ones the second call writes.  A batch whose partial states exceed the buffer is refused
before anything is launched."""
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


def _static_step(case):
    from paper_2602_12029_amd import binding as B
    b = case.batch
    B.ps_decode_attention_static(case.layout, b.tables.data_ptr(), b.q.data_ptr(), b.kv.data_ptr(),
                                 b.scales.data_ptr() if b.scales is not None else 0, b.out.data_ptr(), b.lse.data_ptr(),
                                 int(torch.cuda.current_stream().cuda_stream))


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_static_workspace_matches_caller_workspace_twice_in_a_row(gpu, kv_dtype):
    from gpu_helpers import check_against_oracle
    from paper_2602_12029_amd import binding as B
    geo = wl.Geometry(32, 8, 128, 16, "bf16", kv_dtype) if kv_dtype == "bf16" else wl.Geometry(64, 8, 128, 16, "bf16", kv_dtype)
    big = wl.make_workload("static_big", geo, 4, [3000, 700, 1025], [[0, 1, 2, 3], [1], [0, 3]],
                           [5, 0, 129, 640, 17, 1, 300], pool_factor=1.3, seed=101)
    small = wl.make_workload("static_small", geo, 2, [200], [[0, 1]], [9, 70], pool_factor=1.5, seed=103)
    cases = [gpu(big), gpu(small)]
    assert B.ps_workspace_bytes(cases[1].layout) < B.ps_workspace_bytes(cases[0].layout) <= B.PS_STATIC_WORKSPACE_BYTES
    reference = []
    for case in cases:                                  # the existing entry point, caller-owned workspace
        case.poison_workspace()
        case.batch.decode_attention()
        torch.cuda.synchronize()
        reference.append((case.batch.out.clone(), case.batch.lse.clone()))
    for case in cases:                                  # the two static calls, back to back on one stream
        case.poison_workspace()
        _static_step(case)
    torch.cuda.synchronize()
    for case, (ref_out, ref_lse) in zip(cases, reference):
        assert torch.equal(_bits(case.batch.out), _bits(ref_out))
        assert torch.equal(_bits(case.batch.lse), _bits(ref_lse))
        # the caller's workspace was not touched by the static call (still poisoned)
        assert torch.isnan(case.batch.workspace.view(torch.float32)).all()
        check_against_oracle(case, label=f"{case.w.name} {kv_dtype} static workspace", scaled_bar=True)
    for case in cases:
        case.close()


def test_static_workspace_refuses_a_batch_that_does_not_fit(gpu):
    from paper_2602_12029_amd import binding as B
    # 64 requests x 32 q heads x 130 splits of 32 tokens x 516 B of partial state = 137 MB > 64 MiB
    geo = wl.Geometry(32, 8, 128, 16, "bf16", "bf16")
    w = wl.make_workload("static_too_big", geo, 64, [4100], [list(range(64))], [1] * 64, seed=107)
    case = gpu(w)
    case.replan(32, 32, "mfma", "mfma")
    assert B.ps_workspace_bytes(case.layout) > B.PS_STATIC_WORKSPACE_BYTES
    case.batch.out.zero_()
    with pytest.raises(B.PsError) as err:
        _static_step(case)
    assert err.value.status == B.PS_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert not case.batch.out.float().any()             # nothing ran
    case.batch.decode_attention()                       # the ordinary entry point still serves the batch
    torch.cuda.synchronize()
    assert torch.isfinite(case.batch.out.float()).all()
    case.close()
