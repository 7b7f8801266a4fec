"""PyTorch plumbing around the C ABI: device memory for the pool, pinned host staging for
fills, stream handles.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _to_host_tensor(a, dtype: int, pin: bool) -> torch.Tensor:
    """numpy fp32 array (values already representable) or torch CPU tensor -> contiguous CPU
    tensor of the pool's element type, pinned if asked."""
    if isinstance(a, np.ndarray):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    else:
        t = a
    t = t.to(torch.bfloat16 if dtype == B.LORA_BF16 else torch.float32).contiguous()
    if pin and not t.is_pinned():
        p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        p.copy_(t)
        t = p
    return t


class LoraPool:
    """Owns the device buffer the cache lives in and the cache handle."""

    def __init__(self, proj: Sequence[Sequence[int]], n_layers: int, class_rank: Sequence[int], class_slots: Sequence[int],
                 dtype: int, max_tokens: int, max_segments: int, n_plans: int = 2, mfma_min_tokens: int = 0,
                 device: str = "cuda:0", flags: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("LoraPool needs a GPU: the library has no CPU path")
        self.proj = [tuple(p) for p in proj]
        self.dtype = dtype
        self.device = torch.device(device)
        self.cfg = B.make_config(proj, n_layers, class_rank, class_slots, dtype, max_tokens, max_segments, n_plans, mfma_min_tokens, flags)
        self.bytes = B.lora_cache_bytes_required(self.cfg)
        if self.bytes == 0:
            raise B.LoraError(B.LORA_E_INVAL, "lora_cache_bytes_required")
        self.buf = torch.empty(self.bytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.buf.data_ptr() + 255) // 256 * 256
        rc, self.handle = B.lora_cache_create(self.cfg, base, self.bytes)
        B.check(rc, "lora_cache_create")
        self._host_keep: List[torch.Tensor] = []

    def close(self) -> None:
        if getattr(self, "handle", None) is not None:
            torch.cuda.synchronize(self.device)
            B.lora_cache_destroy(self.handle)
            self.handle = None
            self.buf = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- fills -----------------------------------------------------------------
    def fill(self, slot: int, adapter_id: int, rank: int, alpha: float, layer: int, proj: int, A, Bm,
             stream: Optional[torch.cuda.Stream] = None, pin: bool = True) -> None:
        ta, tb = _to_host_tensor(A, self.dtype, pin), _to_host_tensor(Bm, self.dtype, pin)
        h_in, h_out = self.proj[proj]
        assert tuple(ta.shape) == (h_in, rank) and tuple(tb.shape) == (rank, h_out)
        self._host_keep += [ta, tb]
        st = stream.cuda_stream if stream is not None else torch.cuda.current_stream(self.device).cuda_stream
        B.check(B.lora_cache_fill_slot(self.handle, slot, adapter_id, rank, alpha, layer, proj, ta.data_ptr(), tb.data_ptr(), st),
                "lora_cache_fill_slot")

    def fills_done(self) -> None:
        """Call after synchronizing the fill stream(s): drops the host staging tensors."""
        self._host_keep.clear()

    # -- apply -----------------------------------------------------------------
    def _stream(self, stream) -> int:
        return stream.cuda_stream if stream is not None else torch.cuda.current_stream(self.device).cuda_stream

    def apply(self, layer: int, proj: int, x: torch.Tensor, base_out: torch.Tensor, seg_offsets, seg_slot, seg_rank,
              scale: float, stream: Optional[torch.cuda.Stream] = None) -> None:
        assert x.is_cuda and base_out.is_cuda and x.is_contiguous() and base_out.is_contiguous()
        B.check(B.lora_apply(self.handle, layer, proj, x.data_ptr(), base_out.data_ptr(), x.shape[0], seg_offsets, seg_slot,
                             seg_rank, scale, self._stream(stream)), "lora_apply")

    def plan(self, T: int, seg_offsets, seg_slot, seg_rank, stream: Optional[torch.cuda.Stream] = None):
        rc, p = B.lora_plan_create(self.handle, T, seg_offsets, seg_slot, seg_rank, self._stream(stream))
        B.check(rc, "lora_plan_create")
        return p

    def apply_plan(self, plan, layer: int, proj: int, x: torch.Tensor, base_out: torch.Tensor, scale: float,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
        assert x.is_cuda and base_out.is_cuda and x.is_contiguous() and base_out.is_contiguous()
        B.check(B.lora_apply_plan(self.handle, plan, layer, proj, x.data_ptr(), base_out.data_ptr(), scale, self._stream(stream)),
                "lora_apply_plan")

    def check_fault(self, stream: Optional[torch.cuda.Stream] = None) -> None:
        """Synchronizes the stream and raises if a kernel gave up a bounded wait."""
        rc, fault = B.lora_cache_check_fault(self.handle, self._stream(stream))
        B.check(rc, "lora_cache_check_fault")
        if fault:
            raise RuntimeError("a LoRA apply kernel gave up waiting for its intermediate; outputs are invalid")

    def plan_destroy(self, plan) -> None:
        B.check(B.lora_plan_destroy(self.handle, plan), "lora_plan_destroy")
