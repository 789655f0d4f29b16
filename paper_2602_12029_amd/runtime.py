"""PyTorch plumbing around the C ABI: device buffers and the current stream.

Nothing here computes: tensors are allocated with torch, raw pointers and the
stream handle go to the library, and every step of the path runs in its kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def to_device(bits: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Stored bits (float32 / uint16 bf16 patterns / uint8 e4m3 codes) -> device tensor, bit for bit."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(bits, np.float32)).to(device)
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(bits, np.uint16).view(np.int16)).to(device).view(torch.bfloat16)
    if dtype == "fp8_e4m3":
        return torch.from_numpy(np.ascontiguousarray(bits, np.uint8)).to(device)
    raise ValueError(dtype)


def from_device(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float64 numpy (bf16 widened exactly)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


class DecodeBatch:
    """Device-side state of one decode batch: uploaded tables, workspace, Q, output."""

    def __init__(self, layout, geometry: B.ps_geometry, num_requests: int, q: torch.Tensor, kv: torch.Tensor,
                 scales: torch.Tensor | None = None):
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required: the attention path has no CPU fallback")
        self.layout, self.geometry, self.num_requests = layout, geometry, num_requests
        self.q, self.kv, self.scales = q, kv, scales
        self.device = q.device
        self.out = torch.empty_like(q)
        self.lse = torch.empty((num_requests, geometry.num_q_heads), dtype=torch.float32, device=self.device)
        self.tables = None
        self.workspace = None
        self._sync_plan()

    def _sync_plan(self):
        nbytes = B.ps_layout_device_bytes(self.layout)
        self.tables = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        B.ps_layout_upload(self.layout, self.tables.data_ptr(), _stream())
        torch.cuda.current_stream().synchronize()
        self.workspace = torch.empty(B.ps_workspace_bytes(self.layout), dtype=torch.uint8, device=self.device)

    def replan(self, options: B.ps_plan_options | None):
        B.ps_layout_replan(self.layout, options)
        self._sync_plan()

    def set_visible(self, prefix_visible=None):
        """Limit how much of its prompt's shared prefix every request sees (None = all of it)."""
        B.ps_layout_set_visible(self.layout, self.num_requests, prefix_visible)
        self._sync_plan()

    def _sc(self):
        return self.scales.data_ptr() if self.scales is not None else 0

    def prefix_attention(self):
        B.ps_prefix_attention(self.layout, self.tables.data_ptr(), self.q.data_ptr(), self.kv.data_ptr(), self._sc(),
                              self.workspace.data_ptr(), _stream())

    def suffix_attention(self):
        B.ps_suffix_attention(self.layout, self.tables.data_ptr(), self.q.data_ptr(), self.kv.data_ptr(), self._sc(),
                              self.workspace.data_ptr(), _stream())

    def merge_states(self, with_lse=True):
        B.ps_merge_states(self.layout, self.tables.data_ptr(), self.workspace.data_ptr(), self.out.data_ptr(),
                          self.lse.data_ptr() if with_lse else 0, _stream())

    def decode_attention(self, with_lse=True, kv: torch.Tensor | None = None):
        B.ps_decode_attention(self.layout, self.tables.data_ptr(), self.q.data_ptr(),
                              (self.kv if kv is None else kv).data_ptr(), self._sc(), self.workspace.data_ptr(),
                              self.out.data_ptr(), self.lse.data_ptr() if with_lse else 0, _stream())

    def kv_ingest(self, which: int, src_k: torch.Tensor, src_v: torch.Tensor):
        """Store every segment of one kind (0 prefixes, 1 suffixes) from ragged [T, Hkv, d] sources."""
        assert src_k.stride(2) == 1 and src_v.stride() == src_k.stride()
        B.ps_kv_ingest(self.layout, self.tables.data_ptr(), which, src_k.data_ptr(), src_v.data_ptr(),
                       src_k.stride(0), src_k.stride(1), self.kv.data_ptr(), self._sc(), _stream())

    def append_step(self, pool, new_k: torch.Tensor, new_v: torch.Tensor, active=None):
        """One decode step of cache growth: tables grow on the host and are uploaded again, then the new
        tokens ([R, Hkv, d], contiguous) are stored.  Returns the destinations the host chose."""
        dest = B.ps_layout_append(pool, self.layout, self.num_requests, active).copy()
        self._sync_plan()
        assert new_k.is_contiguous() and new_v.is_contiguous()
        B.ps_kv_append(self.layout, self.tables.data_ptr(), new_k.data_ptr(), new_v.data_ptr(), self.kv.data_ptr(),
                       self._sc(), _stream())
        return dest

    def stage_out(self, image: torch.Tensor):
        """Copy the batch's blocks (and e4m3 scales) into `image`: uint8, device memory or pinned host memory."""
        B.ps_kv_stage_out(self.layout, self.tables.data_ptr(), self.kv.data_ptr(), self._sc(), image.data_ptr(), _stream())

    def stage_in(self, image: torch.Tensor):
        B.ps_kv_stage_in(self.layout, self.tables.data_ptr(), image.data_ptr(), self.kv.data_ptr(), self._sc(), _stream())

    def park(self, pool):
        """Hand the batch's blocks back to the pool (after stage_out has completed)."""
        torch.cuda.current_stream().synchronize()
        B.ps_layout_park(pool, self.layout)

    def resume(self, pool):
        """Take blocks again and upload the new tables; stage_in then restores the contents."""
        B.ps_layout_resume(pool, self.layout)
        self._sync_plan()

    def workspace_views(self):
        """(o [slots, Hq, d] fp32, lse [slots, Hq] fp32) views of the partial-state workspace."""
        slots, off = B.ps_workspace_layout(self.layout)
        g = self.geometry
        o = self.workspace[:off].view(torch.float32).view(slots, g.num_q_heads, g.head_dim)
        lse = self.workspace[off:off + slots * g.num_q_heads * 4].view(torch.float32).view(slots, g.num_q_heads)
        return o, lse
