"""Host side of the C-ABI library (no GPU): exported symbols, bit-exact block tables, plan invariants, errors."""
import json
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import layout as ol
from paper_2602_12029_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert headers == ["prefillshare.h", "prefillshare_probe.h"]
    header = "".join(open(os.path.join(ROOT, "include", f)).read() for f in headers)
    declared = set(re.findall(r"\b(ps_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = B._lib()
    for name in declared:
        assert hasattr(lib, name)
    assert B.ps_strerror(B.PS_ERR_OOM).startswith("not enough")


def _both(w, geo=None):
    g = w.geometry
    geo = geo or B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype)
    pool = B.ps_pool_create(w.num_blocks, w.free_order)
    opool = ol.BlockPool(w.num_blocks, w.free_order)
    if w.num_roots:
        lay = B.ps_kv_layout_tree(pool, geo, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        olay = ol.build_layout_tree(opool, g.block_size, w.root_len, w.prompt_root, w.prefix_len, w.req_prompt,
                                    w.req_model, w.suffix_len)
    else:
        lay = B.ps_kv_layout(pool, geo, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
        olay = ol.build_layout(opool, g.block_size, w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    return pool, lay, opool, olay


@pytest.mark.parametrize("name", ["tiny", "b8", "long", "mixed", "fp8_70b", "sessions40"])
def test_tables_bit_exact_against_oracle_policy(name):
    w = wl.named_workload(name)
    pool, lay, opool, olay = _both(w)
    t = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
    for key in ("prefix_blk_indptr", "prefix_blk", "group_indptr", "group_req", "suffix_blk_indptr", "suffix_blk"):
        assert np.array_equal(t[key], getattr(olay, key)), key
    assert np.array_equal(B.ps_pool_refcounts(pool, w.num_blocks), opool.refcount)
    assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
    B.ps_layout_release(pool, lay)
    ol.release_layout(opool, olay)
    assert np.array_equal(B.ps_pool_refcounts(pool, w.num_blocks), opool.refcount)
    assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
    B.ps_pool_destroy(pool)


def test_hand_worked_instance():
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "layout_small.json")))
    geo = B.geometry(4, 2, 64, g["block_size"], "f32", "f32")
    pool = B.ps_pool_create(g["num_blocks"], g["free_order"])
    lay = B.ps_kv_layout(pool, geo, g["prefix_len"], g["req_prompt"], g["req_model"], g["suffix_len"])
    t = B.ps_layout_tables(lay, 2, 3)
    for key, val in g["expect"].items():
        if key in t:
            assert t[key].tolist() == val, key
    assert B.ps_pool_refcounts(pool, 8).tolist() == g["expect"]["refcount"]
    assert B.ps_pool_free_list(pool).tolist() == g["expect"]["free_after_build"]
    B.ps_layout_release(pool, lay)
    assert B.ps_pool_free_list(pool).tolist() == g["expect"]["free_after_release"]
    B.ps_pool_destroy(pool)


def test_random_batches_against_oracle_policy():
    rng = np.random.default_rng(21)
    for trial in range(30):
        bsz = int(rng.choice([1, 4, 16, 48]))
        num_p = int(rng.integers(1, 6))
        num_m = int(rng.integers(1, 5))
        membership = [sorted(rng.choice(num_m, size=int(rng.integers(1, num_m + 1)), replace=False).tolist())
                      for _ in range(num_p)]
        nreq = sum(len(m) for m in membership)
        geo = wl.Geometry(4, 2, 64, bsz, "f32", "f32")
        w = wl.make_workload("r", geo, num_m, rng.integers(0, 200, num_p), membership, rng.integers(0, 70, nreq),
                             pool_factor=float(rng.uniform(1.0, 2.0)), seed=trial)
        pool, lay, opool, olay = _both(w)
        t = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
        for key in t:
            assert np.array_equal(t[key], getattr(olay, key)), (trial, key)
        assert np.array_equal(B.ps_pool_refcounts(pool, w.num_blocks), opool.refcount)
        B.ps_layout_release(pool, lay)
        ol.release_layout(opool, olay)
        assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
        B.ps_pool_destroy(pool)


def _check_plan(w, lay, plan, visible=None):
    """Chunks tile every segment exactly once per KV head and request (the prefix up to the request's visible
    length); slots are consistent; an item is marked exactly where one of its rows sees less than its range."""
    g = w.geometry
    items, slot_base = plan["items"], plan["slot_base"]
    t = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
    nprefix_blk = int(t["prefix_blk_indptr"][-1])
    req_list = B.ps_layout_request_list(lay)
    R = w.num_requests
    assert np.array_equal(req_list[:R], t["group_req"]) and np.array_equal(req_list[R:2 * R], np.arange(R))
    rt = B.ps_layout_root_tables(lay)
    nsuffix_blk = int(t["suffix_blk_indptr"][-1])
    assert np.array_equal(req_list[2 * R:2 * R + len(rt["root_group_req"])], rt["root_group_req"])
    root_of = [int(w.prompt_root[w.req_prompt[r]]) if w.num_roots else -1 for r in range(R)]
    seen = np.asarray(w.prefix_len)[np.asarray(w.req_prompt)] if visible is None else np.asarray(visible)
    cover = {}                                             # (request, kv head) -> list of (kind, begin, end, slot)
    readers = {}                                           # (segment, token begin, kv head) -> items reading that range
    for blk_off, t0, t1, req_off, n_req, head, split, kind in items.tolist():
        readers[(blk_off, t0, head)] = readers.get((blk_off, t0, head), 0) + 1
    for blk_off, t0, t1, req_off, n_req, head, split, kind in items.tolist():
        assert t1 > t0 >= 0 and n_req >= 1 and 0 <= head < g.num_kv_heads and 0 <= kind <= 31
        assert bool(kind & 16) == (readers[(blk_off, t0, head)] > 1)       # bit 4: several row groups read the range
        assert n_req * g.group <= (256 if kind & 4 else 64) or n_req == 1     # rows one item may carry
        assert t0 % g.block_size == 0
        reqs = req_list[req_off:req_off + n_req].tolist()
        assert len(reqs) == n_req
        if kind & 8:                                                     # a root segment: everybody below sees all of it
            assert not kind & 3
            roots = {root_of[r] for r in reqs}
            assert len(roots) == 1 and min(roots) >= 0
            root = roots.pop()
            assert blk_off == nprefix_blk + nsuffix_blk + rt["root_blk_indptr"][root] and t1 <= w.root_len[root]
            for r in reqs:
                cover.setdefault((r, head), []).append((-1, t0, t1, split))
        elif kind & 1:
            assert n_req == 1 and not kind & 6
            r = reqs[0]
            assert blk_off == nprefix_blk + t["suffix_blk_indptr"][r] and t1 <= w.suffix_len[r]
            cover.setdefault((r, head), []).append((1, t0, t1, split))
        else:
            assert len({int(w.req_prompt[r]) for r in reqs}) == 1
            p = int(w.req_prompt[reqs[0]])
            assert blk_off == t["prefix_blk_indptr"][p] and t1 <= w.prefix_len[p]
            assert t1 <= max(seen[r] for r in reqs)                     # nothing streamed that no row sees
            assert bool(kind & 2) == any(seen[r] < t1 for r in reqs)
            for r in reqs:
                assert seen[r] > t0                                      # every row sees into the item
                cover.setdefault((r, head), []).append((0, t0, min(t1, int(seen[r])), split))
    for r in range(R):
        nslots = int(slot_base[r + 1] - slot_base[r])
        for head in range(g.num_kv_heads):
            chunks = sorted(cover.get((r, head), []), key=lambda c: c[3])
            assert [c[3] for c in chunks] == list(range(nslots))           # every slot written exactly once
            root_len = int(w.root_len[root_of[r]]) if root_of[r] >= 0 else 0
            for kind, length in ((-1, root_len), (0, int(seen[r])), (1, int(w.suffix_len[r]))):
                spans = sorted((c[1], c[2]) for c in chunks if c[0] == kind)
                pos = 0
                for a, b in spans:
                    assert a == pos
                    pos = b
                assert pos == length
            kinds = [c[0] for c in chunks]
            assert kinds == sorted(kinds)                                   # root splits, prefix splits, suffix splits


def test_visible_lengths_plan_invariants_and_errors():
    geo = wl.Geometry(8, 2, 64, 16, "f32", "f32")
    rng = np.random.default_rng(5)
    w = wl.make_workload("vis", geo, 9, [333, 1000, 40], [list(range(9)), [0, 3, 4, 8], [1, 2]],
                         rng.integers(0, 90, 15), seed=3)
    pool, lay, _, _ = _both(w)
    full = np.asarray(w.prefix_len)[np.asarray(w.req_prompt)]
    before = B.ps_layout_plan(lay, w.num_requests)
    tables = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
    refs = B.ps_pool_refcounts(pool, w.num_blocks)
    for trial in range(6):
        visible = rng.integers(0, full + 1)
        if trial == 0:
            visible[:] = 0                                   # nothing visible anywhere: no prefix item at all
        if trial == 1:
            visible = full.copy()                            # everything visible: nothing is marked
        for pc, sc in ((0, 0), (32, 32), (64, 16), (4096, 4096)):
            B.ps_layout_replan(lay, B.plan_options(pc, sc))
            B.ps_layout_set_visible(lay, w.num_requests, visible)
            plan = B.ps_layout_plan(lay, w.num_requests)
            _check_plan(w, lay, plan, visible)
            if trial == 0:
                assert not (plan["items"][:, 7] & 1 == 0).any()
            if trial == 1:
                assert not (plan["items"][:, 7] & 2).any()
    # block tables and refcounts are untouched by visibility
    after = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
    assert all(np.array_equal(tables[k], after[k]) for k in tables)
    assert np.array_equal(refs, B.ps_pool_refcounts(pool, w.num_blocks))
    # out-of-range lengths are rejected and leave the layout as it was
    B.ps_layout_replan(lay, None)
    B.ps_layout_set_visible(lay, w.num_requests, None)
    for bad in (full + (np.arange(15) == 4), -(np.arange(15) == 7).astype(np.int32)):
        with pytest.raises(B.PsError) as e:
            B.ps_layout_set_visible(lay, w.num_requests, bad)
        assert e.value.status == B.PS_ERR_INVALID_ARG
    again = B.ps_layout_plan(lay, w.num_requests)
    assert np.array_equal(before["items"], again["items"]) and np.array_equal(before["slot_base"], again["slot_base"])
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


def test_causal_chunk_plan_skips_what_no_row_sees():
    """A chunk of new tokens on one prompt, token i seeing cached + i + 1 tokens.  Wavefront kernel: row groups of
    64 / G requests; a group's items end at its last row's length, and fully visible ranges are not marked.
    Matrix-core kernels: the group's 160 rows fit one row-split item per token range and KV head."""
    geo = wl.Geometry(8, 2, 128, 16, "bf16", "bf16")
    cached, chunk = 100, 40
    w = wl.make_workload("chunk", geo, chunk, [cached + chunk], [list(range(chunk))], [0] * chunk, seed=0)
    pool, lay, _, _ = _both(w)
    visible = np.arange(cached + 1, cached + chunk + 1)
    for variant, ranges in ((B.PS_VARIANT_WAVE, [(0, 64), (64, 116), (64, 128), (128, 140)]),
                            (B.PS_VARIANT_AUTO, [(0, 64), (64, 128), (128, 140)])):
        B.ps_layout_replan(lay, B.plan_options(64, 32, variant, variant))
        B.ps_layout_set_visible(lay, chunk, visible)
        plan = B.ps_layout_plan(lay, chunk)
        _check_plan(w, lay, plan, visible)
        items = plan["items"]
        assert sorted({(a, b) for a, b in items[:, 1:3].tolist()}) == ranges
        assert not (items[items[:, 2] <= 100][:, 7] & 2).any()                # the old cache is seen by every row
        assert (np.diff(plan["slot_base"]) == np.ceil(visible / 64)).all()    # partial states only where a row sees in
        if variant == B.PS_VARIANT_AUTO:
            assert len(items) == 3 * 2 and items[:, 7].tolist() == [4, 4, 6, 6, 2, 2]   # row-split items lead
            assert items[items[:, 1] == 0][:, 4].tolist() == [40, 40]         # all 40 requests in one item per KV head
            # the last range is seen by 12 requests = 48 rows: an ordinary item, the only kind in the schedule
            assert B.ps_layout_schedule(lay, 0)["items"][:, 7].tolist() == [2, 2]
        else:
            assert not (items[:, 7] & 4).any()
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


@pytest.mark.parametrize("name", ["tiny", "b8", "mixed"])
def test_default_plan_invariants(name):
    w = wl.named_workload(name)
    pool, lay, _, _ = _both(w)
    _check_plan(w, lay, B.ps_layout_plan(lay, w.num_requests))
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


def test_replan_invariants_ragged_and_empty_segments():
    geo = wl.Geometry(8, 2, 64, 16, "f32", "f32")
    w = wl.make_workload("rag", geo, 3, [0, 1, 333, 1000], [[0], [1, 2], [0, 1, 2], [2]], [0, 5, 0, 77, 300, 1, 16],
                         seed=3)
    pool, lay, _, _ = _both(w)
    for pc, sc in ((0, 0), (32, 32), (64, 16), (1000, 1), (4096, 4096)):
        B.ps_layout_replan(lay, B.plan_options(pc, sc))
        plan = B.ps_layout_plan(lay, w.num_requests)
        _check_plan(w, lay, plan)
    # request 0 has no tokens at all: it owns no slot
    plan = B.ps_layout_plan(lay, w.num_requests)
    assert plan["slot_base"][1] == plan["slot_base"][0]
    slots, off = B.ps_workspace_layout(lay)
    assert slots == plan["slot_base"][-1] and off == slots * 8 * 64 * 4
    assert B.ps_workspace_bytes(lay) == slots * 8 * 65 * 4
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


@pytest.mark.parametrize("name", ["b8", "mixed", "fp8_70b"])
def test_schedules_cover_every_item_once_and_balance(name):
    w = wl.named_workload(name)
    pool, lay, _, _ = _both(w)
    items = B.ps_layout_plan(lay, w.num_requests)["items"]
    sets = {0: items[items[:, 7] & 1 == 0], 1: items[items[:, 7] & 1 == 1], 2: items}
    for which, expect in sets.items():
        sch = B.ps_layout_schedule(lay, which)
        assert sch, "bf16 / fp8 workloads run on the matrix-core kernel"
        got = sch["items"]
        key = lambda a: sorted(map(tuple, a.tolist()))
        assert key(got) == key(expect)                                   # a permutation of the set
        ip = sch["indptr"]
        assert ip[0] == 0 and ip[-1] == len(got) and np.all(np.diff(ip) >= 1)
        assert len(ip) - 1 <= 512
        cost = (got[:, 2] - got[:, 1]) + 64
        loads = np.array([cost[a:b].sum() for a, b in zip(ip[:-1], ip[1:])])
        assert loads.max() - loads.min() <= cost.max()                   # longest-processing-time-first bound
        for a, b in zip(ip[:-1], ip[1:]):
            assert np.all(np.diff(cost[a:b]) <= 0)                       # each list longest first
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


def test_kernel_family_selection():
    def variants(geo):
        w = wl.make_workload("v", geo, 1, [64], [[0]], [8], seed=1)
        pool, lay, _, _ = _both(w)
        plan = B.ps_layout_plan(lay, 1)
        sch = B.ps_layout_schedule(lay, 2)
        B.ps_layout_release(pool, lay)
        B.ps_pool_destroy(pool)
        return plan["prefix_variant"], plan["suffix_variant"], bool(sch)
    assert variants(wl.Geometry(8, 2, 128, 16, "bf16", "bf16")) == (B.PS_VARIANT_MFMA, B.PS_VARIANT_MFMA, True)
    assert variants(wl.Geometry(8, 2, 128, 64, "bf16", "fp8_e4m3")) == (B.PS_VARIANT_MFMA, B.PS_VARIANT_MFMA, True)
    # fp32 inputs, other head sizes and block sizes that are not 16 * 2^k go to the wavefront-reduction kernel
    assert variants(wl.Geometry(8, 2, 128, 16, "f32", "f32")) == (B.PS_VARIANT_WAVE, B.PS_VARIANT_WAVE, False)
    assert variants(wl.Geometry(8, 2, 64, 16, "bf16", "bf16")) == (B.PS_VARIANT_WAVE, B.PS_VARIANT_WAVE, False)
    assert variants(wl.Geometry(8, 2, 128, 48, "bf16", "bf16")) == (B.PS_VARIANT_WAVE, B.PS_VARIANT_WAVE, False)


def test_kernel_family_follows_the_span_of_a_block_head_slice():
    """The matrix-core kernels use 32-bit byte offsets inside a (block, head) slice; a pool whose K and V planes lie
    2 GiB or more apart is planned onto the wavefront kernel (64-bit addresses), and asking for the matrix-core
    kernel on it is refused."""
    def planned(kv_stride):
        geo = B.geometry(8, 2, 128, 16, "bf16", "bf16", strides=(2 * 16 * 128, 16 * 128, kv_stride, 128))
        pool = B.ps_pool_create(8)
        lay = B.ps_kv_layout(pool, geo, [64], [0], [0], [8])
        plan = B.ps_layout_plan(lay, 1)
        forced = None
        try:
            B.ps_layout_replan(lay, B.plan_options(0, 0, B.PS_VARIANT_MFMA, B.PS_VARIANT_MFMA))
        except Exception as e:  # noqa: BLE001 - the binding raises on any non-zero status
            forced = str(e)
        B.ps_layout_release(pool, lay)
        B.ps_pool_destroy(pool)
        return plan["prefix_variant"], plan["suffix_variant"], forced
    near = planned((1 << 30) - 16 * 128 - 8)      # the slice ends 16 bytes below 2 GiB (bf16: 2 bytes per element)
    assert near[:2] == (B.PS_VARIANT_MFMA, B.PS_VARIANT_MFMA) and near[2] is None
    far = planned((1 << 30) - 16 * 128)           # ... and exactly at 2 GiB
    assert far[:2] == (B.PS_VARIANT_WAVE, B.PS_VARIANT_WAVE) and far[2] is not None


def test_many_models_split_into_row_chunks():
    geo = wl.Geometry(32, 2, 64, 16, "f32", "f32")           # group of 16: at most 4 requests per item
    w = wl.make_workload("many", geo, 10, [64], [list(range(10))], [1] * 10, seed=4)
    pool, lay, _, _ = _both(w)
    plan = B.ps_layout_plan(lay, w.num_requests)
    _check_plan(w, lay, plan)
    prefix = plan["items"][plan["items"][:, 7] & 1 == 0]
    assert (prefix[:, 7] == 16).all()                         # three row groups read every range
    assert sorted(prefix[prefix[:, 5] == 0][:, 4].tolist()) == [2, 4, 4]
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


def test_error_paths():
    geo = B.geometry(4, 2, 64, 16, "f32", "f32")
    pool = B.ps_pool_create(3, [2, 0, 1])

    def status(fn, *a):
        with pytest.raises(B.PsError) as e:
            fn(*a)
        return e.value.status

    assert status(B.ps_kv_layout, pool, geo, [33], [0], [0], [1]) == B.PS_ERR_OOM
    assert B.ps_pool_free_list(pool).tolist() == [2, 0, 1] and not B.ps_pool_refcounts(pool, 3).any()
    assert status(B.ps_kv_layout, pool, geo, [16], [0, 0], [1, 1], [1, 1]) == B.PS_ERR_INVALID_ARG
    assert status(B.ps_kv_layout, pool, geo, [16, 16], [0], [0], [1]) == B.PS_ERR_INVALID_ARG
    assert status(B.ps_kv_layout, pool, geo, [16], [1], [0], [1]) == B.PS_ERR_INVALID_ARG
    assert status(B.ps_kv_layout, pool, geo, [-1], [0], [0], [1]) == B.PS_ERR_INVALID_ARG
    assert status(B.ps_kv_layout, pool, B.geometry(6, 4, 64, 16, "f32", "f32"), [16], [0], [0], [1]) == B.PS_ERR_SHAPE
    assert status(B.ps_kv_layout, pool, B.geometry(4, 2, 64, 16, "f32", 7), [16], [0], [0], [1]) == B.PS_ERR_UNSUPPORTED
    assert status(B.ps_kv_layout, pool, B.geometry(4, 2, 64, 16, "f32", "bf16", (2048, 1024, 512, 33)),
                  [16], [0], [0], [1]) == B.PS_ERR_SHAPE
    assert status(B.ps_pool_create, 3, [0, 0, 1]) == B.PS_ERR_INVALID_ARG
    assert B.ps_pool_free_list(pool).tolist() == [2, 0, 1]
    # releasing against a pool that does not hold the references is refused and changes nothing
    lay = B.ps_kv_layout(pool, geo, [16], [0], [0], [1])
    other = B.ps_pool_create(3)
    assert status(B.ps_layout_release, other, lay) == B.PS_ERR_REFCOUNT
    assert not B.ps_pool_refcounts(other, 3).any()
    # forcing the MFMA variant on fp32 inputs is refused
    assert status(B.ps_layout_replan, lay, B.plan_options(prefix_variant=B.PS_VARIANT_MFMA)) == B.PS_ERR_UNSUPPORTED
    # an unknown K/V cache policy is refused; the known ones are accepted and change no table
    assert status(B.ps_layout_replan, lay, B.plan_options(kv_cache_policy=3)) == B.PS_ERR_INVALID_ARG
    before = B.ps_layout_plan(lay, 1)["items"].copy()
    for policy in (B.PS_KV_POLICY_STREAM, B.PS_KV_POLICY_CACHEABLE, B.PS_KV_POLICY_AUTO):
        B.ps_layout_replan(lay, B.plan_options(kv_cache_policy=policy))
        assert np.array_equal(B.ps_layout_plan(lay, 1)["items"], before)
    B.ps_layout_release(pool, lay)
    assert B.ps_pool_num_free(pool) == 3
    B.ps_pool_destroy(other)
    B.ps_pool_destroy(pool)


# ---- table growth (ps_layout_append) -------------------------------------------------------------------
def _same_state(w, pool, lay, opool, olay):
    t = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
    for key in t:
        assert np.array_equal(t[key], getattr(olay, key)), key
    lens = B.ps_layout_lengths(lay, w.num_prompts, w.num_requests)
    assert np.array_equal(lens["suffix_len"], olay.suffix_len) and np.array_equal(lens["prefix_len"], olay.prefix_len)
    assert np.array_equal(B.ps_pool_refcounts(pool, opool.num_blocks), opool.refcount)
    assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))


def test_append_hand_worked_instance():
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "layout_small.json")))
    geo = B.geometry(4, 2, 64, g["block_size"], "f32", "f32")
    pool = B.ps_pool_create(g["num_blocks"], g["free_order"])
    lay = B.ps_kv_layout(pool, geo, g["prefix_len"], g["req_prompt"], g["req_model"], g["suffix_len"])
    for step in g["append"]["steps"]:
        if step.get("out_of_blocks"):
            before = (B.ps_layout_tables(lay, 2, 3)["suffix_blk"].tolist(), B.ps_pool_free_list(pool).tolist())
            with pytest.raises(B.PsError) as e:
                B.ps_layout_append(pool, lay, 3, step["active"])
            assert e.value.status == B.PS_ERR_OOM
            assert before == (B.ps_layout_tables(lay, 2, 3)["suffix_blk"].tolist(), B.ps_pool_free_list(pool).tolist())
            continue
        dest = B.ps_layout_append(pool, lay, 3, step["active"])
        assert dest.tolist() == step["dest"]
        t = B.ps_layout_tables(lay, 2, 3)
        assert t["suffix_blk_indptr"].tolist() == step["suffix_blk_indptr"] and t["suffix_blk"].tolist() == step["suffix_blk"]
        assert B.ps_layout_lengths(lay, 2, 3)["suffix_len"].tolist() == step["suffix_len"]
        assert B.ps_pool_refcounts(pool, 8).tolist() == step["refcount"] and B.ps_pool_free_list(pool).tolist() == step["free"]
    B.ps_layout_release(pool, lay)
    assert B.ps_pool_free_list(pool).tolist() == g["append"]["free_after_release"]
    B.ps_pool_destroy(pool)


def test_append_bit_exact_against_oracle_policy_and_plan_invariants():
    import dataclasses
    rng = np.random.default_rng(5)
    for trial in range(12):
        bsz = int(rng.choice([1, 4, 16, 48]))
        num_p, num_m = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        membership = [sorted(rng.choice(num_m, size=int(rng.integers(1, num_m + 1)), replace=False).tolist())
                      for _ in range(num_p)]
        nreq = sum(len(m) for m in membership)
        geo = wl.Geometry(4, 2, 64, bsz, "f32", "f32")
        w = wl.make_workload("r", geo, num_m, rng.integers(0, 100, num_p), membership, rng.integers(0, 40, nreq),
                             pool_factor=float(rng.uniform(1.3, 2.5)), seed=100 + trial)
        pool, lay, opool, olay = _both(w)
        for step in range(int(rng.integers(3, 3 * bsz + 6))):
            active = None if step % 3 == 0 else (rng.random(nreq) < 0.6).astype(np.int32)
            try:
                odest = ol.append_step(opool, olay, active)
            except ol.OutOfBlocks:
                with pytest.raises(B.PsError) as e:
                    B.ps_layout_append(pool, lay, nreq, active)
                assert e.value.status == B.PS_ERR_OOM
                _same_state(w, pool, lay, opool, olay)           # a refused step changes nothing on either side
                break
            dest = B.ps_layout_append(pool, lay, nreq, active)
            assert np.array_equal(dest, odest), (trial, step)
            _same_state(w, pool, lay, opool, olay)
        grown = dataclasses.replace(w, suffix_len=olay.suffix_len.copy())
        _check_plan(grown, lay, B.ps_layout_plan(lay, nreq))
        B.ps_layout_release(pool, lay)
        ol.release_layout(opool, olay)
        assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
        B.ps_pool_destroy(pool)


def test_append_keeps_the_plan_options():
    w = wl.named_workload("b8")
    pool = B.ps_pool_create(w.num_blocks + w.num_requests, None)
    g = w.geometry
    lay = B.ps_kv_layout(pool, B.geometry(g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_size, g.q_dtype, g.kv_dtype),
                         w.prefix_len, w.req_prompt, w.req_model, w.suffix_len)
    B.ps_layout_replan(lay, B.plan_options(1024, 64))
    before = B.ps_layout_plan(lay, w.num_requests)["items"]
    B.ps_layout_append(pool, lay, w.num_requests)
    after = B.ps_layout_plan(lay, w.num_requests)["items"]
    assert (after[after[:, 7] == 0][:, 2] - after[after[:, 7] == 0][:, 1]).max() == 1024
    assert (after[after[:, 7] == 1][:, 2] - after[after[:, 7] == 1][:, 1]).max() <= 64
    assert len(after) >= len(before)
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


TREE_KEYS = ("root_blk_indptr", "root_blk", "root_group_indptr", "root_group_req")


def test_tree_hand_worked_instance():
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "layout_tree_small.json")))
    geo = B.geometry(4, 2, 64, g["block_size"], "f32", "f32")
    pool = B.ps_pool_create(g["num_blocks"], g["free_order"])
    lay = B.ps_kv_layout_tree(pool, geo, g["root_len"], g["prompt_root"], g["prefix_len"], g["req_prompt"], g["req_model"],
                              g["suffix_len"])
    t = dict(B.ps_layout_tables(lay, 3, 4), **B.ps_layout_root_tables(lay))
    e = g["expect"]
    for key in t:
        assert t[key].tolist() == e[key], key
    assert B.ps_pool_refcounts(pool, 12).tolist() == e["refcount"]
    assert B.ps_pool_free_list(pool).tolist() == e["free_after_build"]
    B.ps_layout_release(pool, lay)
    assert B.ps_pool_free_list(pool).tolist() == e["free_after_release"]
    assert not B.ps_pool_refcounts(pool, 12).any()
    B.ps_pool_destroy(pool)


def test_tree_random_batches_against_oracle_policy_and_plan_invariants():
    rng = np.random.default_rng(33)
    for trial in range(20):
        bsz = int(rng.choice([4, 16, 48]))
        num_t = int(rng.integers(1, 4))
        num_p = int(rng.integers(num_t, num_t + 4))
        num_m = int(rng.integers(1, 5))
        prompt_root = np.concatenate([np.arange(num_t), rng.integers(-1, num_t, num_p - num_t)])   # every root is used
        rng.shuffle(prompt_root)
        membership = [sorted(rng.choice(num_m, size=int(rng.integers(1, num_m + 1)), replace=False).tolist())
                      for _ in range(num_p)]
        nreq = sum(len(m) for m in membership)
        geo = wl.Geometry(8, 2, 64, bsz, "f32", "f32")
        w = wl.make_tree_workload("t", geo, num_m, rng.integers(0, 150, num_t), prompt_root, rng.integers(0, 200, num_p),
                                  membership, rng.integers(0, 70, nreq), pool_factor=float(rng.uniform(1.0, 2.0)), seed=trial)
        pool, lay, opool, olay = _both(w)
        t = dict(B.ps_layout_tables(lay, w.num_prompts, w.num_requests), **B.ps_layout_root_tables(lay))
        for key in t:
            assert np.array_equal(t[key], getattr(olay, key)), (trial, key)
        assert np.array_equal(B.ps_pool_refcounts(pool, w.num_blocks), opool.refcount)
        for pc, sc in ((0, 0), (32, 16), (64, 4096)):
            B.ps_layout_replan(lay, B.plan_options(pc, sc))
            _check_plan(w, lay, B.ps_layout_plan(lay, w.num_requests))
        if trial % 4 == 0:                                   # visible lengths cut the prompts' own prefixes, never a root
            visible = rng.integers(0, np.asarray(w.prefix_len)[np.asarray(w.req_prompt)] + 1)
            B.ps_layout_set_visible(lay, w.num_requests, visible)
            _check_plan(w, lay, B.ps_layout_plan(lay, w.num_requests), visible)
        B.ps_layout_release(pool, lay)
        ol.release_layout(opool, olay)
        assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
        B.ps_pool_destroy(pool)


def test_tree_errors_leave_the_pool_untouched():
    geo = B.geometry(4, 2, 64, 4, "f32", "f32")
    pool = B.ps_pool_create(4, [3, 1, 0, 2])
    cases = [([9], [0], [4], [0], [0], [1], B.PS_ERR_OOM),               # needs 3 + 1 + 1 blocks
             ([4], [1], [4], [0], [0], [1], B.PS_ERR_INVALID_ARG),       # unknown root
             ([4, 4], [0], [4], [0], [0], [1], B.PS_ERR_INVALID_ARG),    # a root no prompt begins with
             ([-1], [0], [4], [0], [0], [1], B.PS_ERR_INVALID_ARG)]      # negative root length
    for root_len, prompt_root, prefix, rp, rm, sl, status in cases:
        with pytest.raises(B.PsError) as e:
            B.ps_kv_layout_tree(pool, geo, root_len, prompt_root, prefix, rp, rm, sl)
        assert e.value.status == status
        assert B.ps_pool_free_list(pool).tolist() == [3, 1, 0, 2] and not B.ps_pool_refcounts(pool, 4).any()
    B.ps_pool_destroy(pool)


def test_root_groups_stay_in_the_persistent_launch_unless_the_batch_is_a_prefill():
    w = wl.named_tree_workload("tree_b8")
    pool, lay, _, _ = _both(w)
    plan = B.ps_layout_plan(lay, w.num_requests)
    _check_plan(w, lay, plan)
    items = plan["items"]
    roots = items[items[:, 7] & 8 != 0]
    assert len(roots) and (roots[:, 7] == 8 | 16).all() and roots[:, 4].max() == 16   # 128 requests x 4 heads: 8 x 64 rows
    sch = B.ps_layout_schedule(lay, 2)
    assert len(sch["items"]) == len(items)                                          # one launch holds everything
    # with visible lengths set (a partial-prefill batch) groups of more than 64 rows go to the prefill kernel
    visible = np.asarray(w.prefix_len)[np.asarray(w.req_prompt)] - 1
    B.ps_layout_set_visible(lay, w.num_requests, visible)
    plan = B.ps_layout_plan(lay, w.num_requests)
    _check_plan(w, lay, plan, visible)
    items = plan["items"]
    roots = items[items[:, 7] & 8 != 0]
    assert (roots[:, 7] == 12 | 16).all() and roots[:, 4].max() == 64 and (items[:len(roots), 7] & 4).all()
    sch = B.ps_layout_schedule(lay, 2)
    assert not (sch["items"][:, 7] & 4).any() and len(sch["items"]) == len(items) - len(roots)
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


def test_park_and_resume_hand_worked_sequence():
    """The sequence of tests/test_oracle_staging.py::test_hand_worked_park_and_resume through the C ABI."""
    geo = B.geometry(4, 2, 64, 4, "f32", "f32")
    pool = B.ps_pool_create(8, [3, 1, 7, 0, 2, 6, 5, 4])
    a = B.ps_kv_layout(pool, geo, [6], [0, 0], [0, 1], [1, 5])
    assert B.ps_layout_state(a) == (5, False)
    B.ps_layout_park(pool, a)
    assert B.ps_pool_free_list(pool).tolist() == [6, 5, 4, 0, 1, 2, 3, 7] and not B.ps_pool_refcounts(pool, 8).any()
    assert B.ps_layout_state(a) == (5, True)
    t = B.ps_layout_tables(a, 1, 2)
    assert (t["prefix_blk"] == -1).all() and (t["suffix_blk"] == -1).all()      # a parked layout names no block
    with pytest.raises(B.PsError) as e:
        B.ps_layout_park(pool, a)
    assert e.value.status == B.PS_ERR_INVALID_ARG
    b = B.ps_kv_layout(pool, geo, [4], [0], [0], [9])
    assert B.ps_layout_tables(b, 1, 1)["suffix_blk"].tolist() == [5, 4, 0]
    with pytest.raises(B.PsError) as e:
        B.ps_layout_resume(pool, a)
    assert e.value.status == B.PS_ERR_OOM and B.ps_pool_free_list(pool).tolist() == [1, 2, 3, 7]
    assert B.ps_layout_state(a) == (5, True)
    B.ps_layout_release(pool, b)
    B.ps_layout_resume(pool, a)
    t = B.ps_layout_tables(a, 1, 2)
    assert t["prefix_blk"].tolist() == [1, 2] and t["suffix_blk"].tolist() == [3, 7, 0]
    assert B.ps_pool_free_list(pool).tolist() == [4, 5, 6]
    assert B.ps_pool_refcounts(pool, 8).tolist() == [1, 2, 2, 1, 0, 0, 0, 1]
    with pytest.raises(B.PsError):
        B.ps_layout_resume(pool, a)
    # a parked layout can be released without touching the pool
    B.ps_layout_park(pool, a)
    free = B.ps_pool_free_list(pool).tolist()
    B.ps_layout_release(pool, a)
    assert B.ps_pool_free_list(pool).tolist() == free and not B.ps_pool_refcounts(pool, 8).any()
    B.ps_pool_destroy(pool)


def test_park_resume_random_batches_against_oracle_and_parked_layouts_refuse_work():
    from oracle import staging as ost
    rng = np.random.default_rng(61)
    for trial in range(10):
        geo = wl.Geometry(8, 2, 64, int(rng.choice([4, 16])), "f32", "f32")
        w = wl.make_tree_workload("p", geo, 3, rng.integers(0, 60, 2), [0, 1, -1, 0], rng.integers(0, 120, 4),
                                  [[0, 1, 2], [1], [0, 2], [2]], rng.integers(0, 50, 7), pool_factor=2.0, seed=trial)
        pool, lay, opool, olay = _both(w)
        assert B.ps_blocks_needed(geo.block_size, w.prefix_len, w.suffix_len, w.root_len) == w.blocks_needed() == \
            ost.blocks_needed(geo.block_size, w.prefix_len, w.suffix_len, w.root_len) == B.ps_layout_state(lay)[0]
        B.ps_layout_replan(lay, B.plan_options(32, 16))
        before = B.ps_layout_plan(lay, w.num_requests)
        B.ps_layout_park(pool, lay)
        ost.park_layout(opool, olay)
        assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
        with pytest.raises(B.PsError) as e:                                # no table growth while parked
            B.ps_layout_append(pool, lay, w.num_requests)
        assert e.value.status == B.PS_ERR_INVALID_ARG
        B.ps_layout_resume(pool, lay)
        ost.resume_layout(opool, olay)
        t = dict(B.ps_layout_tables(lay, w.num_prompts, w.num_requests), **B.ps_layout_root_tables(lay))
        for key in ("prefix_blk", "suffix_blk", "root_blk", "prefix_blk_indptr", "suffix_blk_indptr", "root_blk_indptr"):
            assert np.array_equal(t[key], getattr(olay, key)), (trial, key)
        assert np.array_equal(B.ps_pool_refcounts(pool, w.num_blocks), opool.refcount)
        after = B.ps_layout_plan(lay, w.num_requests)                      # same plan, options kept
        assert np.array_equal(before["items"], after["items"]) and np.array_equal(before["slot_base"], after["slot_base"])
        _check_plan(w, lay, after)
        bb, so, tot = B.ps_stage_layout(lay)
        assert bb == 2 * 2 * geo.block_size * 64 * 4 and tot == w.blocks_needed() * bb and so % 256 == 0 and so >= tot
        B.ps_layout_release(pool, lay)
        B.ps_pool_destroy(pool)
    with pytest.raises(B.PsError):
        B.ps_blocks_needed(16, [5], [-1])


def test_adopted_blocks_hand_worked_and_rules():
    """tests/test_oracle_layout.py::test_adopted_blocks_hand_worked and ::test_adoption_rules through the C ABI."""
    geo = B.geometry(4, 2, 64, 4, "f32", "f32")
    pool = B.ps_pool_create(10)
    a = B.ps_kv_layout(pool, geo, [10], [0, 0], [0, 1], [2, 5])
    c = B.ps_kv_layout_adopt(pool, geo, [14], [[0, 1]], [0, 0, 0], [0, 1, 2], [0, 3, 0])
    t = B.ps_layout_tables(c, 1, 3)
    assert t["prefix_blk"].tolist() == [0, 1, 6, 7] and t["suffix_blk"].tolist() == [8]
    assert B.ps_pool_refcounts(pool, 10).tolist() == [5, 5, 2, 1, 1, 1, 3, 3, 1, 0] and B.ps_pool_free_list(pool).tolist() == [9]
    assert B.ps_layout_state(c) == (5, False)
    B.ps_layout_release(pool, a)
    assert B.ps_pool_refcounts(pool, 10).tolist() == [3, 3, 0, 0, 0, 0, 3, 3, 1, 0]
    assert B.ps_pool_free_list(pool).tolist() == [9, 2, 3, 4, 5]
    B.ps_layout_release(pool, c)
    assert not B.ps_pool_refcounts(pool, 10).any() and B.ps_pool_free_list(pool).tolist() == [9, 2, 3, 4, 5, 0, 1, 6, 7, 8]
    B.ps_pool_destroy(pool)
    pool = B.ps_pool_create(6)
    a = B.ps_kv_layout(pool, geo, [9], [0], [0], [0])
    bad = [([11], [[0, 1, 2]], [0], B.PS_ERR_INVALID_ARG),      # only full blocks: 3 * 4 > 11
           ([12], [[0, 5]], [0], B.PS_ERR_INVALID_ARG),         # block 5 is not alive
           ([12, 12], [[0], [0]], [0, 1], B.PS_ERR_INVALID_ARG),  # named twice
           ([24], [[0, 1]], [0], B.PS_ERR_OOM)]                 # needs 4 more, 3 free
    for prefix, adopt, rp, status in bad:
        with pytest.raises(B.PsError) as e:
            B.ps_kv_layout_adopt(pool, geo, prefix, adopt, rp, [0] * len(rp), [0] * len(rp))
        assert e.value.status == status
        assert B.ps_pool_refcounts(pool, 6).tolist() == [1, 1, 1, 0, 0, 0] and B.ps_pool_free_list(pool).tolist() == [3, 4, 5]
    b = B.ps_kv_layout_adopt(pool, geo, [4], [[]], [0], [0], [0])                   # adopting nothing
    assert B.ps_layout_tables(b, 1, 1)["prefix_blk"].tolist() == [3]
    B.ps_layout_release(pool, a)
    B.ps_layout_release(pool, b)
    assert not B.ps_pool_refcounts(pool, 6).any()
    B.ps_pool_destroy(pool)


def test_adoption_random_chains_against_oracle():
    """Contexts continued over several steps: each step's layout adopts the full prefix blocks of the one before, which
    is then released; tables, refcounts and free lists stay equal to the oracle's throughout."""
    rng = np.random.default_rng(71)
    for trial in range(8):
        bsz = int(rng.choice([4, 16]))
        geo = B.geometry(8, 2, 64, bsz, "f32", "f32")
        num_p = int(rng.integers(1, 4))
        pool, opool = B.ps_pool_create(400), ol.BlockPool(400)
        ctx = rng.integers(1, 60, num_p)
        prev = prev_o = None
        for step in range(4):
            membership = [sorted(rng.choice(4, size=int(rng.integers(1, 4)), replace=False).tolist()) for _ in range(num_p)]
            rp = [p for p, m in enumerate(membership) for _ in m]
            rm = [x for m in membership for x in m]
            sl = rng.integers(0, 40, len(rp))
            if prev is None:
                adopt = [[] for _ in range(num_p)]
            else:
                pt = B.ps_layout_tables(prev, num_p, prev_nreq)
                adopt = [pt["prefix_blk"][pt["prefix_blk_indptr"][p]:pt["prefix_blk_indptr"][p] + int(prev_ctx[p]) // bsz].tolist()
                         for p in range(num_p)]
            lay = B.ps_kv_layout_adopt(pool, geo, ctx, adopt, rp, rm, sl)
            olay = ol.build_layout(opool, bsz, ctx, rp, rm, sl, adopt=adopt)
            t = B.ps_layout_tables(lay, num_p, len(rp))
            for key in t:
                assert np.array_equal(t[key], getattr(olay, key)), (trial, step, key)
            if prev is not None:
                B.ps_layout_release(pool, prev)
                ol.release_layout(opool, prev_o)
            assert np.array_equal(B.ps_pool_refcounts(pool, 400), opool.refcount)
            assert np.array_equal(B.ps_pool_free_list(pool), np.array(opool.free, np.int32))
            prev, prev_o, prev_ctx, prev_nreq = lay, olay, ctx.copy(), len(rp)
            ctx = ctx + rng.integers(0, 50, num_p)                      # the contexts grow
        B.ps_layout_release(pool, prev)
        ol.release_layout(opool, prev_o)
        assert not B.ps_pool_refcounts(pool, 400).any()
        B.ps_pool_destroy(pool)


@pytest.mark.parametrize("tree", [False, True])
def test_plan_stays_valid_over_many_decode_steps(tree):
    """Appends mostly patch the plan instead of rebuilding it: after every step the plan must still tile every segment
    at its current length, and the schedules must hold exactly the plan's items (chunk sizes of 32 / 64 tokens make
    segments outgrow their chunks all the time, which plans afresh)."""
    import copy
    geo = wl.Geometry(32, 8, 128, 16, "bf16", "bf16")
    rng = np.random.default_rng(79)
    if tree:
        w = wl.make_tree_workload("steps", geo, 3, [100], [0, -1, 0], [300, 31, 0], [[0, 1, 2], [1], [0, 2]],
                                  [5, 0, 129, 64, 17, 33], pool_factor=3.0, seed=1)
    else:
        w = wl.make_workload("steps", geo, 3, [333, 48], [[0, 1, 2], [1]], [40, 0, 97, 16], pool_factor=3.0, seed=1)
    pool, lay, opool, olay = _both(w)
    cur = copy.copy(w)
    cur.suffix_len = w.suffix_len.copy()
    for pc, sc in ((0, 0), (64, 32), (256, 64)):
        B.ps_layout_replan(lay, B.plan_options(pc, sc))
        for step in range(40):
            active = (rng.random(w.num_requests) < 0.7).astype(np.int32)
            dest = B.ps_layout_append(pool, lay, w.num_requests, active)
            odest = ol.append_step(opool, olay, active)
            assert np.array_equal(dest, odest)
            cur.suffix_len = cur.suffix_len + active
            t = B.ps_layout_tables(lay, w.num_prompts, w.num_requests)
            assert np.array_equal(t["suffix_blk"], olay.suffix_blk) and np.array_equal(t["suffix_blk_indptr"], olay.suffix_blk_indptr)
            plan = B.ps_layout_plan(lay, w.num_requests)
            _check_plan(cur, lay, plan)
            sch = B.ps_layout_schedule(lay, 2)
            key = lambda a: sorted(map(tuple, a.tolist()))
            assert key(sch["items"]) == key(plan["items"])
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)


def test_chunk_aim_follows_the_spread_of_the_shared_segments():
    """Where two workgroups share a compute unit, shared segments of unequal lengths are cut at 0.6 of a compute
    unit's share of the batch's token-heads, segments of equal length at a whole share (the split plan is this build's
    own design: the paper has no kernel; the rule is a measured one, see the planner)."""
    def prefix_item_tokens(name, num_cus=256):
        w = wl.named_workload(name)
        pool, lay, _, _ = _both(w)
        B.ps_layout_replan(lay, B.plan_options(0, 0, 0, 0, num_cus, 0))
        items = B.ps_layout_plan(lay, w.num_requests)["items"]
        shared = items[items[:, 7] & 1 == 0]
        total = (int(w.prefix_len.astype(np.int64).sum()) + int(w.suffix_len.astype(np.int64).sum())) * w.geometry.num_kv_heads
        B.ps_layout_release(pool, lay)
        B.ps_pool_destroy(pool)
        return (shared[:, 2] - shared[:, 1]), total
    tok, total = prefix_item_tokens("sessions40")              # contexts of 1024 .. 6144 tokens, 16 rows per group
    aim = -(-(total * 3 // 5) // 256)
    assert tok.max() <= -(-aim // 32) * 32 and tok.max() > aim // 2
    tok, _ = prefix_item_tokens("b8")                          # 32 prefixes of 4096 tokens: stay whole
    assert set(tok.tolist()) == {4096}


def test_prefill_items_take_whole_contexts_where_the_share_allows():
    """Partial-prefill batches: a context a little over the chunk aim is not cut in two, and the prefill kernel's items
    are not held to the persistent kernel's 8192 tokens (its ranges are walked one scalar block id per tile)."""
    for name, contexts in (("prefill_b8", 32), ("prefill_fp8", 64)):
        w, visible = wl.named_chunk_prefill(name)
        pool, lay, _, _ = _both(w)
        B.ps_layout_replan(lay, B.plan_options(0, 0, 0, 0, 256, 0))
        B.ps_layout_set_visible(lay, w.num_requests, visible)
        plan = B.ps_layout_plan(lay, w.num_requests)
        _check_plan(w, lay, plan, visible)
        items = plan["items"]
        assert np.all(items[:, 7] & 4)                               # every group is wide: row-split items only
        # one token range per context, except the shortest contexts, whose items fill the launch's last round in pieces
        whole = {blk for blk in set(items[:, 0].tolist()) if np.all(items[items[:, 0] == blk][:, 1] == 0)}
        assert len(set(items[:, 0].tolist())) == contexts and len(whole) >= contexts // 2
        cut = items[~np.isin(items[:, 0], list(whole))]
        longest_cut = (cut[:, 2] - cut[:, 1]).max() if len(cut) else 0
        assert longest_cut < (items[:, 2] - items[:, 1]).max()
        if name == "prefill_fp8":
            assert (items[:, 2] - items[:, 1]).max() > 8192
        B.ps_layout_release(pool, lay)
        B.ps_pool_destroy(pool)


def test_long_prefill_chunks_fall_back_where_few_requests_see_far():
    """A chunk longer than the persistent kernel's items hold is kept only if every chunk of the context goes to the
    prefill kernel; here two of forty requests see past the first 100 tokens, so the far chunk would be an ordinary
    8-row item and the context is cut at the ordinary size instead."""
    geo = wl.Geometry(32, 8, 128, 16, "bf16", "bf16")
    n, length = 40, 60000
    w = wl.make_workload("far", geo, n, [length], [list(range(n))], [0] * n, seed=0)
    pool, lay, _, _ = _both(w)
    visible = np.full(n, 100, np.int32)
    visible[-2:] = length
    B.ps_layout_replan(lay, B.plan_options(0, 0, 0, 0, 4, 0))       # four compute units: a share of 120 k token-heads
    B.ps_layout_set_visible(lay, n, visible)
    plan = B.ps_layout_plan(lay, n)
    _check_plan(w, lay, plan, visible)
    items = plan["items"]
    ordinary = items[(items[:, 7] & 4) == 0]
    assert len(ordinary) and (ordinary[:, 2] - ordinary[:, 1]).max() <= 8192
    assert (items[:, 2] - items[:, 1]).max() <= 8192
    # all forty seeing everything: one row-split range, longer than an ordinary item may be
    B.ps_layout_set_visible(lay, n, np.full(n, length, np.int32))
    plan = B.ps_layout_plan(lay, n)
    _check_plan(w, lay, plan, np.full(n, length, np.int32))
    items = plan["items"]
    assert np.all(items[:, 7] & 4) and (items[:, 2] - items[:, 1]).max() > 8192
    B.ps_layout_release(pool, lay)
    B.ps_pool_destroy(pool)
