"""Glue used by the tests, the smoke check and the benchmark: lay a generated instance
(workloads.Instance) out in a LoraPool, upload activations, run the library, measure error.
No arithmetic of the method happens here; comparisons are plain numpy."""
from __future__ import annotations

from typing import Dict, Iterable, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B
from .pool import LoraPool

CLASS_RANKS = (8, 16, 32, 64, 128)  # the paper's five adapter ranks (section 5.1)


def slot_layout(ranks: np.ndarray, class_rank: Sequence[int] = CLASS_RANKS) -> Tuple[np.ndarray, np.ndarray]:
    """(class_slots, slot_of_adapter): every pool adapter gets its own slot in the smallest
    class that holds its rank; slot ids run class by class, adapters in index order."""
    cr = np.asarray(class_rank)
    cls = np.searchsorted(cr, ranks)
    assert (cls < len(cr)).all(), "rank above the largest class"
    class_slots = np.bincount(cls, minlength=len(cr)).astype(np.int32)
    first = np.concatenate([[0], np.cumsum(class_slots)[:-1]])
    slot_of = np.empty(len(ranks), np.int32)
    nxt = first.copy()
    for a, k in enumerate(cls):
        slot_of[a] = nxt[k]
        nxt[k] += 1
    return class_slots, slot_of


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == B.LORA_BF16 else torch.float32


def to_device(a: np.ndarray, dtype: int, device="cuda:0") -> torch.Tensor:
    """fp32 numpy array holding representable values -> device tensor of the pool's element type."""
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32))
    return t.to(torch_dtype(dtype)).to(device)


class PooledInstance:
    """An instance's adapters resident in a pool, plus its segment arrays in slot terms."""

    def __init__(self, inst, n_layers: Optional[int] = None, fill_layers: Optional[Iterable[int]] = None,
                 adapters: Optional[Iterable[int]] = None, extra_tokens: int = 0, n_plans: int = 2,
                 mfma_min_tokens: int = 0, class_rank: Sequence[int] = CLASS_RANKS, flags: int = 0):
        self.inst = inst
        self.dtype = B.LORA_BF16 if inst.dtype == "bf16" else B.LORA_F32
        self.n_layers = int(n_layers or inst.n_layers)
        self.class_slots, self.slot_of = slot_layout(inst.ranks, class_rank)
        self.pool = LoraPool([(p.h_in, p.h_out) for p in inst.projs], self.n_layers, class_rank, self.class_slots, self.dtype,
                             max_tokens=max(1, inst.T + extra_tokens), max_segments=max(1, inst.n_seg + 8), n_plans=n_plans,
                             mfma_min_tokens=mfma_min_tokens, flags=flags)
        self.seg_slot = np.where(inst.seg_adapter >= 0, self.slot_of[np.maximum(inst.seg_adapter, 0)], -1).astype(np.int32)
        self.seg_rank = inst.seg_rank
        self.filled: Dict[int, bool] = {}
        layers = list(range(self.n_layers)) if fill_layers is None else list(fill_layers)
        self.fill(inst.used_adapters() if adapters is None else adapters, layers)

    def fill(self, adapters: Iterable[int], layers: Sequence[int], stream=None, sync: bool = True) -> int:
        """Fill the (layer, projection) parts of the given pool adapters; the same weights go
        into every layer copy (values do not matter for layer copies, residency does)."""
        n_bytes = 0
        for a in adapters:
            a = int(a)
            for p in range(len(self.inst.projs)):
                A, Bm = self.inst.adapter_weights(a, p)
                ta = torch.from_numpy(A).to(torch_dtype(self.dtype)).pin_memory()
                tb = torch.from_numpy(Bm).to(torch_dtype(self.dtype)).pin_memory()
                for l in layers:
                    self.pool.fill(int(self.slot_of[a]), int(self.inst.adapter_ids[a]), int(self.inst.ranks[a]),
                                   float(self.inst.alpha[a]), l, p, ta, tb, stream=stream, pin=False)
                    n_bytes += ta.numel() * ta.element_size() + tb.numel() * tb.element_size()
            if sync:
                (stream.synchronize() if stream is not None else torch.cuda.current_stream().synchronize())
                self.pool.fills_done()
            self.filled[a] = True
        return n_bytes

    def apply(self, layer: int, p: int, x: torch.Tensor, y: torch.Tensor, stream=None) -> None:
        self.pool.apply(layer, p, x, y, self.inst.seg_offsets, self.seg_slot, self.seg_rank, self.inst.scale, stream)

    def close(self) -> None:
        self.pool.close()


def error_metrics(y_gpu: np.ndarray, y_ref: np.ndarray, base: np.ndarray, out_dtype: str = "bf16") -> Dict[str, float]:
    """Relative Frobenius error and worst element error (in units of RMS(y_ref)) on y, and the
    error measured against the adapter delta y - base alone (a kernel that does nothing nearly
    passes the first two).  The delta figure takes out what no kernel can avoid, the one rounding of
    the stored output: e_round = |round_to_out_dtype(y_ref) - y_ref|_F is computed from the reference
    itself (not a worst-case bound), and since the rounding of a result and the arithmetic error before
    it are independent they add in quadrature:
        delta_rel_fro = sqrt(max(0, |y_gpu - y_ref|_F^2 - e_round^2)) / |y_ref - base|_F
    """
    y_gpu, y_ref, base = (np.asarray(v, np.float64) for v in (y_gpu, y_ref, base))
    d = y_gpu - y_ref
    err = np.linalg.norm(d)
    fro = np.linalg.norm(y_ref)
    rms = np.sqrt(np.mean(y_ref**2)) if y_ref.size else 0.0
    dn = np.linalg.norm(y_ref - base)
    t = torch.from_numpy(np.ascontiguousarray(y_ref))
    rounded = t.to(torch.bfloat16 if out_dtype == "bf16" else torch.float32).to(torch.float64).numpy()
    e_round = np.linalg.norm(rounded - y_ref)
    excess = float(np.sqrt(max(0.0, err * err - e_round * e_round)))
    return {
        "rel_fro": float(err / fro) if fro > 0 else float(err),
        "max_abs_over_rms": float(np.max(np.abs(d)) / rms) if rms > 0 and d.size else 0.0,
        "delta_rel_fro": excess / float(dn) if dn > 0 else excess,
    }
