"""GPU parity for the cache-writing entry points (ps_kv_ingest, ps_kv_append, ps_layout_append) through the C ABI.

Bars: everything stored is byte / index work or a quantised code decided in float32 on both sides, so pools,
scales and destinations are compared bit for bit; attention over the grown caches keeps the bars of the
attention tests (fp32 1e-5 / 1e-5, bf16 and e4m3 max-abs 1e-2 and relative RMS 5e-3).
"""
import numpy as np
import pytest
import torch

import workloads as wl
from workloads import generate as gen
from helpers import errors, oracle_decode
from oracle import fp8
from oracle import kv_update as ku
from oracle import layout as ol

pytestmark = pytest.mark.gpu

TOL = {"f32": (1e-5, 1e-5), "bf16": (1e-2, 5e-3), "fp8_e4m3": (1e-2, 5e-3)}


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from gpu_helpers import GpuCase
    return GpuCase


def _bits(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> integer bit patterns on the host."""
    view = {torch.bfloat16: torch.int16, torch.float32: torch.int32, torch.uint8: torch.uint8}[t.dtype]
    return t.view(view).cpu().numpy()


def _host_bits(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    return a.view({4: np.int32, 2: np.int16, 1: np.uint8}[a.dtype.itemsize])


def _same_pool(case, label):
    torch.cuda.synchronize()
    got = _bits(case.batch.kv).transpose(np.argsort(case.pool_axes))     # back to the dense axis order
    assert np.array_equal(got, _host_bits(case.data.kv)), f"{label}: pool bits differ"
    if case.data.scales is not None:
        assert np.array_equal(_bits(case.batch.scales), _host_bits(case.data.scales)), f"{label}: scales differ"


def _workloads():
    bf = wl.Geometry(8, 2, 128, 16, "bf16", "bf16")
    f8 = wl.Geometry(8, 2, 128, 16, "bf16", "fp8_e4m3")
    member = [[0], [1, 2], [0, 1, 2], [2]]
    pre, suf = [1, 333, 1000, 16], [0, 5, 17, 77, 300, 1, 16]
    return [
        wl.make_workload("tiny_f32", wl.Geometry(4, 2, 64, 16, "f32", "f32"), 2, [256], [[0, 1]], [8, 8], 2.0, seed=1),
        wl.make_workload("rag_bf16", bf, 3, pre, member, suf, 1.6, seed=2),
        wl.make_workload("rag_fp8", f8, 3, pre, member, suf, 1.6, seed=3),
        wl.make_workload("blk64_fp8", wl.Geometry(8, 2, 128, 64, "bf16", "fp8_e4m3"), 3, pre, member, suf, 2.0, seed=4),
        wl.make_workload("blk48_f32", wl.Geometry(4, 2, 64, 48, "f32", "f32"), 3, pre, member, suf, 2.0, seed=5),
    ]


def _poison(case):
    """Both pools (device and oracle side) back to the poison pattern: nothing stored yet."""
    g = case.w.geometry
    case.data.kv[...] = gen.POISON[g.kv_dtype]
    bits = torch.from_numpy(_host_bits(case.data.kv)).to(case.batch.kv.device)
    case.batch.kv.view(-1).copy_(bits.view(case.batch.kv.dtype).view(-1))   # one value everywhere: any axis order
    if case.data.scales is not None:
        case.data.scales[...] = np.float32("nan")
        case.batch.scales.copy_(torch.from_numpy(case.data.scales).to(case.batch.scales.device))


def _ragged(parts, dtype, device, pad=False):
    """Concatenate [L_i, Hkv, d] sources back to back; pad=True leaves gaps between heads and tokens."""
    from paper_2602_12029_amd.runtime import to_device
    parts = [p for p in parts if p.shape[0]]
    if not parts:
        return None
    flat = to_device(np.concatenate(parts, axis=0), "f32" if dtype == "f32" else "bf16", device)
    if not pad:
        return flat
    t, h, d = flat.shape
    wide = torch.zeros((t, h + 1, d + 16), dtype=flat.dtype, device=device)
    wide[:, :h, :d] = flat
    return wide[:, :h, :d]


def _ingest_both_sides(case, pad=False):
    w, g = case.w, case.w.geometry
    for which in (0, 1):
        n = w.num_prompts if which == 0 else w.num_requests
        src = [w.prefix_source(i) if which == 0 else w.suffix_source(i) for i in range(n)]
        k_dev = _ragged([s[0] for s in src], g.kv_dtype, case.batch.kv.device, pad)
        v_dev = _ragged([s[1] for s in src], g.kv_dtype, case.batch.kv.device, pad)
        if k_dev is None:
            continue
        case.batch.kv_ingest(which, k_dev, v_dev)
        indptr, blk = (case.olay.prefix_blk_indptr, case.olay.prefix_blk) if which == 0 else \
                      (case.olay.suffix_blk_indptr, case.olay.suffix_blk)
        for i in range(n):
            ku.ingest_segment(case.data.kv, case.data.scales, g.kv_dtype, blk[indptr[i]:indptr[i + 1]], src[i][0], src[i][1])


@pytest.mark.parametrize("pad,pool_layout", [(False, "dense"), (True, "dense"), (True, "token_major"), (False, "planes")])
def test_ingest_bit_exact(gpu, pad, pool_layout):
    for w in _workloads():
        print(f"ingest {w.name} pad={pad} pool {pool_layout}", flush=True)
        case = gpu(w, pool_layout=pool_layout)
        _poison(case)
        _ingest_both_sides(case, pad)
        _same_pool(case, w.name)
        case.close()


def test_e4m3_encoder_on_every_bf16_value_in_range(gpu):
    """Tiles that hold a 448 have scale 1, so their codes are the encoder applied to the raw values: sweeps
    every bf16 value of magnitude <= 448 (both signs, zeros, the subnormal range of e4m3) through K; V
    carries the same values times 0.37 (a scale that is not a power of two, so the division matters)."""
    top = int(np.float32(448.0).view(np.uint32) >> 16)
    vals = np.arange(0, top + 1, dtype=np.uint16)
    vals = np.concatenate([vals, vals | np.uint16(0x8000)])
    per_tile = 16 * 128 - 1
    tiles = -(-len(vals) // per_tile)
    k = np.zeros((tiles, 16 * 128), np.uint16)
    for i in range(tiles):
        chunk = vals[i * per_tile:(i + 1) * per_tile]
        k[i, 0] = top << 0                                        # 448.0
        k[i, 1:1 + len(chunk)] = chunk
    k = k.reshape(tiles * 16, 1, 128)
    kf = (k.astype(np.uint32) << np.uint32(16)).view(np.float32)
    v = wl.bf16_bits_from_f32(kf * np.float32(0.37))
    geo = wl.Geometry(1, 1, 128, 16, "bf16", "fp8_e4m3")
    w = wl.make_workload("sweep", geo, 1, [tiles * 16], [[0]], [0], seed=9)
    case = gpu(w)
    _poison(case)
    from paper_2602_12029_amd.runtime import to_device
    case.batch.kv_ingest(0, to_device(k, "bf16"), to_device(v, "bf16"))
    ku.ingest_segment(case.data.kv, case.data.scales, "fp8_e4m3", case.olay.prefix_blk, k, v)
    torch.cuda.synchronize()
    ids = case.olay.prefix_blk
    assert (case.data.scales[ids, 0, 0] == 1.0).all()
    _same_pool(case, "encoder sweep")
    case.close()


def _append_steps(case, steps, rng, check_each=False):
    from paper_2602_12029_amd.runtime import to_device
    w, g = case.w, case.w.geometry
    for t in range(steps):
        active = None if t % 4 == 0 else (rng.random(w.num_requests) < 0.7).astype(np.int32)
        k_t, v_t = w.step_tokens(t)
        src_dtype = "f32" if g.kv_dtype == "f32" else "bf16"
        dest = case.batch.append_step(case.pool, to_device(k_t, src_dtype), to_device(v_t, src_dtype), active)
        odest = ol.append_step(case.opool, case.olay, active)
        assert np.array_equal(dest, odest), f"step {t}: destinations differ"
        for r in np.nonzero(odest >= 0)[0]:
            ku.append_token(case.data.kv, case.data.scales, g.kv_dtype, odest[r], k_t[r], v_t[r])
        if check_each:
            _same_pool(case, f"{w.name} step {t}")


@pytest.mark.parametrize("pool_layout", ["dense", "token_major"])
def test_append_bit_exact(gpu, pool_layout):
    for w in _workloads():
        print(f"append {w.name} pool {pool_layout}", flush=True)
        case = gpu(w, pool_layout=pool_layout)
        rng = np.random.default_rng(11)
        _append_steps(case, 2 * w.geometry.block_size + 3 if w.geometry.block_size <= 16 else 70, rng, check_each=w.geometry.block_size <= 16)
        _same_pool(case, w.name)
        if case.data.scales is not None:                            # the inputs did make scales grow
            assert len(np.unique(case.data.scales[case.olay.suffix_blk])) > 8
        case.close()


def test_decode_loop_matches_oracle(gpu):
    """Hand-off, then decode steps: ingest both segment kinds, then append + attend repeatedly."""
    from paper_2602_12029_amd.runtime import from_device
    for w in _workloads()[:4]:
        print(f"decode loop {w.name}", flush=True)
        case = gpu(w)
        _poison(case)
        _ingest_both_sides(case)
        rng = np.random.default_rng(13)
        for phase in range(3):
            _append_steps(case, 7, rng)
            case.poison_workspace()
            case.batch.decode_attention()
            torch.cuda.synchronize()
            ref_o, ref_lse = oracle_decode(w, case.olay, case.data)
            max_abs, rel_rms, worst = errors(from_device(case.batch.out), ref_o)
            print(f"  phase {phase}: max_abs={max_abs:.3e} rel_rms={rel_rms:.3e} worst_req={worst:.3e}", flush=True)
            tol_abs, tol_rms = TOL[w.geometry.kv_dtype]
            assert max_abs <= tol_abs and rel_rms <= tol_rms
        _same_pool(case, w.name)
        case.close()


@pytest.mark.parametrize("name", ["b8", "fp8_70b"])
def test_ingest_full_size_sampled(gpu, name):
    """Benchmark-size hand-off in the launch configuration the bench times; the oracle checks a sample of
    the stored tiles (it would need minutes for all of them)."""
    w = wl.named_workload(name)
    g = w.geometry
    case = gpu(w)
    dev = case.batch.kv.device
    rng = np.random.default_rng(17)
    t_all = int(w.prefix_len.astype(np.int64).sum())
    # one seeded draw for the whole ragged tensor (the per-prompt generators would take a minute on this size)
    k = wl.bf16_bits_from_f32(rng.standard_normal((t_all, g.num_kv_heads, g.head_dim), dtype=np.float32)
                              * np.exp2(rng.uniform(-2, 2, (t_all, 1, 1))).astype(np.float32))
    v = wl.bf16_bits_from_f32(rng.standard_normal((t_all, g.num_kv_heads, g.head_dim), dtype=np.float32))
    from paper_2602_12029_amd.runtime import to_device
    case.batch.kv.view(torch.uint8).fill_(0x7F)
    case.batch.kv_ingest(0, to_device(k, "bf16", dev), to_device(v, "bf16", dev))
    torch.cuda.synchronize()
    got = _bits(case.batch.kv).reshape(case.data.kv.shape)
    got_sc = None if case.batch.scales is None else case.batch.scales.cpu().numpy()
    tok0 = np.concatenate([[0], np.cumsum(w.prefix_len.astype(np.int64))])
    b = g.block_size
    checked = 0
    for _ in range(600):
        p = int(rng.integers(w.num_prompts))
        i = int(rng.integers(-(-int(w.prefix_len[p]) // b)))
        blk = int(case.olay.prefix_blk[case.olay.prefix_blk_indptr[p] + i])
        lo = int(tok0[p]) + i * b
        hi = min(lo + b, int(tok0[p + 1]))
        ref_kv = np.full((blk + 1,) + case.data.kv.shape[1:], gen.POISON[g.kv_dtype], case.data.kv.dtype)
        ref_sc = None if got_sc is None else np.full((blk + 1, g.num_kv_heads, 2), np.nan, np.float32)
        ku.ingest_segment(ref_kv, ref_sc, g.kv_dtype, [blk], k[lo:hi], v[lo:hi])
        assert np.array_equal(got[blk], _host_bits(ref_kv[blk])), (p, i)
        if got_sc is not None:
            assert np.array_equal(got_sc[blk], ref_sc[blk]), (p, i)
        checked += 1
    # blocks that belong to no prefix were not touched
    untouched = np.setdiff1d(np.arange(w.num_blocks), case.olay.prefix_blk)
    assert (got[untouched[:64]].view(np.uint8) == 0x7F).all()
    print(f"{name}: {checked} tiles checked bit for bit", flush=True)
    case.close()
