"""ctypes binding of libprefillshare.so: same names as include/prefillshare.h.

Host arrays are numpy int32 arrays; device pointers and the stream are plain
integers (e.g. torch.Tensor.data_ptr(), torch.cuda.current_stream().cuda_stream).
Every wrapper raises PsError on a non-zero status.  Opaque handles are returned
as ctypes void pointers.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

PS_OK, PS_ERR_INVALID_ARG, PS_ERR_SHAPE, PS_ERR_OOM, PS_ERR_REFCOUNT, PS_ERR_UNSUPPORTED, PS_ERR_DEVICE, PS_ERR_TOO_LARGE = range(8)
PS_STATIC_WORKSPACE_BYTES = 64 << 20
PS_F32, PS_BF16, PS_FP8_E4M3 = 0, 1, 2
PS_VARIANT_AUTO, PS_VARIANT_WAVE, PS_VARIANT_MFMA = 0, 1, 2
PS_KV_POLICY_AUTO, PS_KV_POLICY_STREAM, PS_KV_POLICY_CACHEABLE = 0, 1, 2
DTYPE_CODE = {"f32": PS_F32, "bf16": PS_BF16, "fp8_e4m3": PS_FP8_E4M3}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libprefillshare.so")

EXPORTS = [
    "ps_pool_create", "ps_pool_destroy", "ps_pool_num_free", "ps_pool_free_list", "ps_pool_refcounts",
    "ps_kv_layout", "ps_layout_release", "ps_layout_tables", "ps_layout_replan", "ps_layout_plan",
    "ps_layout_schedule", "ps_layout_device_bytes", "ps_layout_upload", "ps_workspace_bytes", "ps_workspace_layout",
    "ps_prefix_attention", "ps_suffix_attention", "ps_prefix_suffix_attention", "ps_merge_states", "ps_decode_attention",
    "ps_layout_lengths", "ps_layout_append", "ps_kv_append", "ps_kv_ingest",
    "ps_layout_set_visible", "ps_layout_request_list", "ps_kv_layout_tree", "ps_layout_root_tables",
    "ps_kv_layout_adopt", "ps_blocks_needed", "ps_layout_state", "ps_stage_layout", "ps_kv_stage_out", "ps_kv_stage_in", "ps_layout_park",
    "ps_layout_resume", "ps_probe_read", "ps_decode_attention_static",
    "ps_strerror", "ps_last_hip_error",
]


# entry points that enqueue device work or query the HIP runtime (csrc/abi.hip); the rest is host-only (csrc/layout.cpp)
DEVICE_EXPORTS = {
    "ps_layout_upload", "ps_prefix_attention", "ps_suffix_attention", "ps_prefix_suffix_attention", "ps_merge_states",
    "ps_decode_attention", "ps_decode_attention_static", "ps_kv_append", "ps_kv_ingest", "ps_kv_stage_out", "ps_kv_stage_in",
    "ps_probe_read",
    "ps_last_hip_error",
}
# Test hook: path of a build of the host side alone (block pool, tables, split plan) under AddressSanitizer / UBSan
# (`python -m paper_2602_12029_amd.build --sanitize`).  The device entry points do not exist in it, so nothing can
# compute through it; it serves the CPU-only sanitizer run of the host tests.
HOST_ONLY_LIB_ENV = "PREFILLSHARE_HOST_ONLY_LIB"


class PsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().ps_strerror(status).decode()
        if status == PS_ERR_DEVICE:
            msg += f" [hip error {_lib().ps_last_hip_error()}]"
        super().__init__(f"{where}: {msg} (status {status})")


class ps_geometry(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("q_dtype", C.c_int32), ("kv_dtype", C.c_int32),
                ("kv_stride_block", C.c_int64), ("kv_stride_head", C.c_int64),
                ("kv_stride_kv", C.c_int64), ("kv_stride_tok", C.c_int64)]


class ps_plan_options(C.Structure):
    _fields_ = [("prefix_chunk_tokens", C.c_int32), ("suffix_chunk_tokens", C.c_int32),
                ("prefix_variant", C.c_int32), ("suffix_variant", C.c_int32), ("num_cus", C.c_int32),
                ("kv_cache_policy", C.c_int32)]


_LIB = None
_I32P = C.POINTER(C.c_int32)


def _lib():
    global _LIB
    if _LIB is None:
        host_only = os.environ.get(HOST_ONLY_LIB_ENV)
        path = host_only or LIB_PATH
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_2602_12029_amd.build` "
                              "(there is no CPU fallback)")
        if not host_only:
            # The caller's device memory and streams come from PyTorch, so the library has to bind to the
            # HIP runtime PyTorch ships: importing torch first makes the loader resolve libamdhip64 to it.
            import torch  # noqa: F401
        lib = C.CDLL(path)
        lib.ps_strerror.restype = C.c_char_p
        lib.ps_strerror.argtypes = [C.c_int32]
        lib.ps_layout_device_bytes.restype = C.c_int64
        lib.ps_workspace_bytes.restype = C.c_int64
        for name in EXPORTS:
            if not (host_only and name in DEVICE_EXPORTS):
                getattr(lib, name)                  # fail early if a symbol is missing
        _LIB = lib
    return _LIB


def _check(status: int, where: str):
    if status != PS_OK:
        raise PsError(status, where)


def _i32(a):
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(_I32P)


def _view(ptr, n) -> np.ndarray:
    if n == 0:
        return np.zeros(0, np.int32)
    return np.ctypeslib.as_array(ptr, shape=(n,)).copy()


def geometry(num_q_heads, num_kv_heads, head_dim, block_size, q_dtype, kv_dtype, strides=None) -> ps_geometry:
    """strides = (block, head, kv, tok) in elements; default is the dense [blk][Hkv][2][B][d] pool."""
    if strides is None:
        tok = head_dim
        kv = block_size * tok
        head = 2 * kv
        strides = (num_kv_heads * head, head, kv, tok)
    return ps_geometry(num_q_heads, num_kv_heads, head_dim, block_size,
                       DTYPE_CODE.get(q_dtype, q_dtype), DTYPE_CODE.get(kv_dtype, kv_dtype), *strides)


def plan_options(prefix_chunk_tokens=0, suffix_chunk_tokens=0, prefix_variant=0, suffix_variant=0, num_cus=0,
                 kv_cache_policy=0):
    return ps_plan_options(prefix_chunk_tokens, suffix_chunk_tokens, prefix_variant, suffix_variant, num_cus,
                           kv_cache_policy)


# ---- pool ------------------------------------------------------------------------------------------
def ps_pool_create(num_blocks: int, free_order=None):
    out = C.c_void_p()
    if free_order is None:
        st = _lib().ps_pool_create(C.c_int32(num_blocks), None, C.byref(out))
    else:
        arr, p = _i32(free_order)
        if arr.shape != (num_blocks,):
            raise ValueError("free_order must have num_blocks entries")
        st = _lib().ps_pool_create(C.c_int32(num_blocks), p, C.byref(out))
    _check(st, "ps_pool_create")
    return out


def ps_pool_destroy(pool):
    _check(_lib().ps_pool_destroy(pool), "ps_pool_destroy")


def ps_pool_num_free(pool) -> int:
    out = C.c_int32()
    _check(_lib().ps_pool_num_free(pool, C.byref(out)), "ps_pool_num_free")
    return out.value


def ps_pool_free_list(pool) -> np.ndarray:
    n = ps_pool_num_free(pool)
    buf = np.zeros(max(n, 1), np.int32)
    cnt = C.c_int32()
    _check(_lib().ps_pool_free_list(pool, buf.ctypes.data_as(_I32P), C.c_int32(n), C.byref(cnt)), "ps_pool_free_list")
    return buf[:cnt.value].copy()


def ps_pool_refcounts(pool, num_blocks: int) -> np.ndarray:
    p = _I32P()
    _check(_lib().ps_pool_refcounts(pool, C.byref(p)), "ps_pool_refcounts")
    return _view(p, num_blocks)


# ---- layout ----------------------------------------------------------------------------------------
def ps_kv_layout(pool, geo: ps_geometry, prefix_len, req_prompt, req_model, suffix_len):
    pl, plp = _i32(prefix_len)
    rp, rpp = _i32(req_prompt)
    rm, rmp = _i32(req_model)
    sl, slp = _i32(suffix_len)
    if not (rp.shape == rm.shape == sl.shape):
        raise ValueError("request arrays differ in length")
    out = C.c_void_p()
    st = _lib().ps_kv_layout(pool, C.byref(geo), C.c_int32(pl.size), plp, C.c_int32(rp.size), rpp, rmp, slp, C.byref(out))
    _check(st, "ps_kv_layout")
    return out


def ps_kv_layout_tree(pool, geo: ps_geometry, root_len, prompt_root, prefix_len, req_prompt, req_model, suffix_len):
    """Three-level table: roots (contexts several prompts begin with), prompts, requests."""
    rl, rlp = _i32(root_len)
    pr, prp = _i32(prompt_root)
    pl, plp = _i32(prefix_len)
    rp, rpp = _i32(req_prompt)
    rm, rmp = _i32(req_model)
    sl, slp = _i32(suffix_len)
    if not (rp.shape == rm.shape == sl.shape) or pr.shape != pl.shape:
        raise ValueError("array lengths do not match")
    out = C.c_void_p()
    st = _lib().ps_kv_layout_tree(pool, C.byref(geo), C.c_int32(rl.size), rlp, C.c_int32(pl.size), prp, plp,
                                  C.c_int32(rp.size), rpp, rmp, slp, C.byref(out))
    _check(st, "ps_kv_layout_tree")
    return out


def ps_kv_layout_adopt(pool, geo: ps_geometry, prefix_len, adopt, req_prompt, req_model, suffix_len):
    """adopt: per prompt, the list of block ids (full blocks of the beginning of its prefix) taken over from a
    layout that still holds them."""
    pl, plp = _i32(prefix_len)
    rp, rpp = _i32(req_prompt)
    rm, rmp = _i32(req_model)
    sl, slp = _i32(suffix_len)
    if len(adopt) != pl.size or not (rp.shape == rm.shape == sl.shape):
        raise ValueError("array lengths do not match")
    indptr = np.zeros(pl.size + 1, np.int32)
    indptr[1:] = np.cumsum([len(a) for a in adopt])
    ai, aip = _i32(indptr)
    ab, abp = _i32(np.concatenate([np.asarray(a, np.int32) for a in adopt]) if pl.size else np.zeros(0, np.int32))
    out = C.c_void_p()
    st = _lib().ps_kv_layout_adopt(pool, C.byref(geo), C.c_int32(pl.size), plp, aip, abp, C.c_int32(rp.size), rpp, rmp,
                                   slp, C.byref(out))
    _check(st, "ps_kv_layout_adopt")
    return out


def ps_layout_root_tables(layout) -> dict:
    n = C.c_int32()
    ptrs = [_I32P() for _ in range(4)]
    _check(_lib().ps_layout_root_tables(layout, C.byref(n), *[C.byref(p) for p in ptrs]), "ps_layout_root_tables")
    bi = _view(ptrs[0], n.value + 1)
    gi = _view(ptrs[2], n.value + 1)
    return {"root_blk_indptr": bi, "root_blk": _view(ptrs[1], int(bi[-1])),
            "root_group_indptr": gi, "root_group_req": _view(ptrs[3], int(gi[-1]))}


def ps_layout_release(pool, layout):
    _check(_lib().ps_layout_release(pool, layout), "ps_layout_release")


def ps_layout_tables(layout, num_prompts: int, num_requests: int) -> dict:
    ptrs = [_I32P() for _ in range(6)]
    _check(_lib().ps_layout_tables(layout, *[C.byref(p) for p in ptrs]), "ps_layout_tables")
    pbi = _view(ptrs[0], num_prompts + 1)
    gi = _view(ptrs[2], num_prompts + 1)
    sbi = _view(ptrs[4], num_requests + 1)
    return {"prefix_blk_indptr": pbi, "prefix_blk": _view(ptrs[1], int(pbi[-1])),
            "group_indptr": gi, "group_req": _view(ptrs[3], num_requests),
            "suffix_blk_indptr": sbi, "suffix_blk": _view(ptrs[5], int(sbi[-1]))}


def ps_layout_lengths(layout, num_prompts: int, num_requests: int) -> dict:
    pl, sl = _I32P(), _I32P()
    _check(_lib().ps_layout_lengths(layout, C.byref(pl), C.byref(sl)), "ps_layout_lengths")
    return {"prefix_len": _view(pl, num_prompts), "suffix_len": _view(sl, num_requests)}


def ps_layout_append(pool, layout, num_requests: int, active=None) -> np.ndarray:
    """One decode step of table growth; returns dest[R] (block * B + slot of each new token, -1 = inactive)."""
    if active is None:
        ap = None
    else:
        arr, ap = _i32(active)
        if arr.size != num_requests:
            raise ValueError("active mask has the wrong length")
    dest = _I32P()
    _check(_lib().ps_layout_append(pool, layout, ap, C.byref(dest)), "ps_layout_append")
    return _view(dest, num_requests)


def ps_layout_replan(layout, options: ps_plan_options | None = None):
    st = _lib().ps_layout_replan(layout, C.byref(options) if options is not None else None)
    _check(st, "ps_layout_replan")


def ps_layout_plan(layout, num_requests: int) -> dict:
    n = C.c_int32()
    items, slots = _I32P(), _I32P()
    pv, sv = C.c_int32(), C.c_int32()
    _check(_lib().ps_layout_plan(layout, C.byref(n), C.byref(items), C.byref(slots), C.byref(pv), C.byref(sv)),
           "ps_layout_plan")
    return {"items": _view(items, n.value * 8).reshape(-1, 8), "slot_base": _view(slots, num_requests + 1),
            "prefix_variant": pv.value, "suffix_variant": sv.value}


def ps_layout_set_visible(layout, num_requests: int, prefix_visible=None):
    """Per-request visible prefix lengths (None = everything); the plan is re-derived."""
    if prefix_visible is None:
        vp = None
    else:
        arr, vp = _i32(prefix_visible)
        if arr.size != num_requests:
            raise ValueError("prefix_visible has the wrong length")
    _check(_lib().ps_layout_set_visible(layout, vp), "ps_layout_set_visible")


def ps_layout_request_list(layout) -> np.ndarray:
    n, lst = C.c_int32(), _I32P()
    _check(_lib().ps_layout_request_list(layout, C.byref(n), C.byref(lst)), "ps_layout_request_list")
    return _view(lst, n.value)


def ps_layout_schedule(layout, which: int) -> dict:
    """which: 0 prefix items, 1 suffix items, 2 both.  Returns {} where the set does not use the MFMA kernel."""
    n = C.c_int32()
    items, indptr = _I32P(), _I32P()
    _check(_lib().ps_layout_schedule(layout, C.c_int32(which), C.byref(n), C.byref(items), C.byref(indptr)),
           "ps_layout_schedule")
    if n.value == 0:
        return {}
    ip = _view(indptr, n.value + 1)
    return {"indptr": ip, "items": _view(items, int(ip[-1]) * 8).reshape(-1, 8)}


def ps_layout_device_bytes(layout) -> int:
    return int(_lib().ps_layout_device_bytes(layout))


def ps_layout_upload(layout, dev_tables: int, stream: int = 0):
    _check(_lib().ps_layout_upload(layout, C.c_void_p(dev_tables), C.c_void_p(stream)), "ps_layout_upload")


def ps_workspace_bytes(layout) -> int:
    return int(_lib().ps_workspace_bytes(layout))


def ps_workspace_layout(layout):
    n, off = C.c_int64(), C.c_int64()
    _check(_lib().ps_workspace_layout(layout, C.byref(n), C.byref(off)), "ps_workspace_layout")
    return n.value, off.value


# ---- attention passes ------------------------------------------------------------------------------
def _p(x):
    return C.c_void_p(int(x) if x else None)


def ps_prefix_attention(layout, dev_tables, q, kv_pool, kv_scales, workspace, stream=0):
    _check(_lib().ps_prefix_attention(layout, _p(dev_tables), _p(q), _p(kv_pool), _p(kv_scales), _p(workspace),
                                      _p(stream)), "ps_prefix_attention")


def ps_suffix_attention(layout, dev_tables, q, kv_pool, kv_scales, workspace, stream=0):
    _check(_lib().ps_suffix_attention(layout, _p(dev_tables), _p(q), _p(kv_pool), _p(kv_scales), _p(workspace),
                                      _p(stream)), "ps_suffix_attention")


def ps_prefix_suffix_attention(layout, dev_tables, q, kv_pool, kv_scales, workspace, stream=0):
    _check(_lib().ps_prefix_suffix_attention(layout, _p(dev_tables), _p(q), _p(kv_pool), _p(kv_scales),
                                             _p(workspace), _p(stream)), "ps_prefix_suffix_attention")


def ps_merge_states(layout, dev_tables, workspace, out, out_lse=0, stream=0):
    _check(_lib().ps_merge_states(layout, _p(dev_tables), _p(workspace), _p(out), _p(out_lse), _p(stream)),
           "ps_merge_states")


def ps_decode_attention(layout, dev_tables, q, kv_pool, kv_scales, workspace, out, out_lse=0, stream=0):
    _check(_lib().ps_decode_attention(layout, _p(dev_tables), _p(q), _p(kv_pool), _p(kv_scales), _p(workspace),
                                      _p(out), _p(out_lse), _p(stream)), "ps_decode_attention")


def ps_decode_attention_static(layout, dev_tables, q, kv_pool, kv_scales, out, out_lse=0, stream=0):
    _check(_lib().ps_decode_attention_static(layout, _p(dev_tables), _p(q), _p(kv_pool), _p(kv_scales), _p(out),
                                             _p(out_lse), _p(stream)), "ps_decode_attention_static")


def ps_kv_append(layout, dev_tables, new_k, new_v, kv_pool, kv_scales, stream=0):
    _check(_lib().ps_kv_append(layout, _p(dev_tables), _p(new_k), _p(new_v), _p(kv_pool), _p(kv_scales), _p(stream)),
           "ps_kv_append")


def ps_kv_ingest(layout, dev_tables, which: int, src_k, src_v, src_stride_tok: int, src_stride_head: int, kv_pool,
                 kv_scales, stream=0):
    _check(_lib().ps_kv_ingest(layout, _p(dev_tables), C.c_int32(which), _p(src_k), _p(src_v), C.c_int64(src_stride_tok),
                               C.c_int64(src_stride_head), _p(kv_pool), _p(kv_scales), _p(stream)), "ps_kv_ingest")


# ---- staging of cold KV and admission ----------------------------------------------------------------
def ps_blocks_needed(block_size: int, prefix_len, suffix_len, root_len=()) -> int:
    rl, rlp = _i32(root_len)
    pl, plp = _i32(prefix_len)
    sl, slp = _i32(suffix_len)
    out = C.c_int64()
    _check(_lib().ps_blocks_needed(C.c_int32(block_size), C.c_int32(rl.size), rlp, C.c_int32(pl.size), plp,
                                   C.c_int32(sl.size), slp, C.byref(out)), "ps_blocks_needed")
    return out.value


def ps_layout_state(layout):
    """(blocks the layout takes, parked?)"""
    n, parked = C.c_int64(), C.c_int32()
    _check(_lib().ps_layout_state(layout, C.byref(n), C.byref(parked)), "ps_layout_state")
    return n.value, bool(parked.value)


def ps_stage_layout(layout):
    """(bytes per block, offset of the e4m3 scales, total bytes) of the layout's staging image."""
    bb, so, tot = C.c_int64(), C.c_int64(), C.c_int64()
    _check(_lib().ps_stage_layout(layout, C.byref(bb), C.byref(so), C.byref(tot)), "ps_stage_layout")
    return bb.value, so.value, tot.value


def ps_kv_stage_out(layout, dev_tables, kv_pool, kv_scales, image, stream=0):
    _check(_lib().ps_kv_stage_out(layout, _p(dev_tables), _p(kv_pool), _p(kv_scales), _p(image), _p(stream)),
           "ps_kv_stage_out")


def ps_kv_stage_in(layout, dev_tables, image, kv_pool, kv_scales, stream=0):
    _check(_lib().ps_kv_stage_in(layout, _p(dev_tables), _p(image), _p(kv_pool), _p(kv_scales), _p(stream)),
           "ps_kv_stage_in")


def ps_probe_read(dev_buf, nbytes: int, pattern: int, num_workgroups: int, stream=0):
    _check(_lib().ps_probe_read(_p(dev_buf), C.c_int64(nbytes), C.c_int32(pattern), C.c_int32(num_workgroups),
                                _p(stream)), "ps_probe_read")


def ps_layout_park(pool, layout):
    _check(_lib().ps_layout_park(pool, layout), "ps_layout_park")


def ps_layout_resume(pool, layout):
    _check(_lib().ps_layout_resume(pool, layout), "ps_layout_resume")


def ps_strerror(status: int) -> str:
    return _lib().ps_strerror(status).decode()


def ps_last_hip_error() -> int:
    return int(_lib().ps_last_hip_error())
