"""Seeded synthetic inputs for the rehearsal-buffer path.

This module only manufactures inputs (sample tensors and labels of the shapes,
value distributions and label structure of the five benchmark workloads).  It
holds none of the method's arithmetic: no candidate selection, no slot
assignment, no sampling.  Both the GPU tests / bench and the CPU oracle's tests
draw their inputs from here so that they see identical bytes.

The paper trains on ImageNet-1K (1000 classes, about 1300 images per class,
crops of 3x224x224; Sec. VI-A) with b=56, c=14, r=7 (Sec. VI-C).  That dataset
is not available here; the workloads below keep its shapes and class count and
replace pixel values by seeded random numbers.  Stored bytes are never
interpreted by the path, so the value distribution only has to make rows
distinguishable.
"""
from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    wid: int                  # 1-based index of the workload; seeds the data generator
    K: int                    # classes
    S: int                    # slots per class
    shape: Tuple[int, ...]    # shape of one sample
    dtype: str                # "f32" or "bf16"
    b: int                    # mini-batch size
    c: int                    # candidates per mini-batch
    r: int                    # representatives per augmented mini-batch
    steps: int
    values: str               # "normal" (N(0,1)) or "uniform" (U(0,1))
    labels: str               # "uniform", "zipf" (P(k) ~ (k+1)^-1.1), "active50" (50 classes drawn afresh every step)
                              # or "fixed50" (one set of 50 classes for the whole run)
    lib_seed: int = 0         # seed handed to rb_update / rb_sample_augment

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def row_elems(self) -> int:
        return int(np.prod(self.shape))

    @property
    def row_bytes(self) -> int:
        return self.row_elems * self.elem_bytes

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def buffer_bytes(self) -> int:
        return self.K * self.S * self.row_bytes

    def bytes_per_step(self) -> int:
        """Bytes the method itself has to move in one update+sample step:
        every inserted row and every representative row is read once and
        written once."""
        return 2 * (self.c + self.r) * self.row_bytes


C1 = Workload("C1-tiny-10x20-f32-3x32x32", 1, 10, 20, (3, 32, 32), "f32", 16, 4, 4, 100, "normal", "uniform")
C2 = Workload("C2-100x500-f32-3x32x32", 2, 100, 500, (3, 32, 32), "f32", 128, 16, 16, 1000, "normal", "uniform")
C3 = Workload("C3-1000x130-f32-3x224x224", 3, 1000, 130, (3, 224, 224), "f32", 64, 8, 8, 2000, "uniform", "uniform")
C4 = Workload("C4-1000x300-bf16-3x224x224-zipf", 4, 1000, 300, (3, 224, 224), "bf16", 512, 64, 64, 2000, "uniform", "zipf")
C5 = Workload("C5-10000x1000-f32-2048-active50", 5, 10000, 1000, (2048,), "f32", 4096, 1024, 1024, 500, "normal", "active50")
CONFIGS = (C1, C2, C3, C4, C5)
# C5 with ONE set of 50 active classes for the whole run (the configured C5 draws a fresh set every step, so its
# classes never fill): 1024 candidates per step into 50 classes of 1000 slots, which are all full after about 50
# steps; from then on every step overwrites about 20 slots per class and several candidates share a slot.
C5F = Workload("C5F-10000x1000-f32-2048-fixed50", 5, 10000, 1000, (2048,), "f32", 4096, 1024, 1024, 500, "normal", "fixed50")
EXTRA = (C5F,)


def by_name(name: str) -> Workload:
    for w in CONFIGS + EXTRA:
        if w.name == name or w.name.split("-")[0] == name:
            return w
    raise KeyError(name)


def variant(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields changed (stress variants for parity tests)."""
    return replace(w, **kw)


def _generator(w: Workload, step: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((1000 + w.wid) * 1_000_003 + int(step))
    return g


_ZIPF_CDF = {}


def _zipf_cdf(K: int, device) -> torch.Tensor:
    key = (K, str(device))
    if key not in _ZIPF_CDF:
        p = 1.0 / np.arange(1, K + 1, dtype=np.float64) ** 1.1
        cdf = np.cumsum(p / p.sum())
        cdf[-1] = 1.0
        _ZIPF_CDF[key] = torch.from_numpy(cdf).to(device)
    return _ZIPF_CDF[key]


def make_labels(w: Workload, step: int, device="cpu") -> torch.Tensor:
    """int64 labels of the mini-batch of one step."""
    g = _generator(w, step, device)
    if w.labels == "uniform":
        return torch.randint(0, w.K, (w.b,), generator=g, device=device, dtype=torch.int64)
    if w.labels == "zipf":
        u = torch.rand((w.b,), generator=g, device=device, dtype=torch.float64)
        k = torch.searchsorted(_zipf_cdf(w.K, device), u)
        return k.clamp_(max=w.K - 1).to(torch.int64)
    if w.labels == "active50":
        n_active = min(50, w.K)
        active = torch.randperm(w.K, generator=g, device=device)[:n_active]
        pick = torch.randint(0, n_active, (w.b,), generator=g, device=device)
        return active[pick].to(torch.int64)
    if w.labels == "fixed50":
        n_active = min(50, w.K)
        g0 = torch.Generator(device=device)
        g0.manual_seed((1000 + w.wid) * 1_000_003 + 999_983)      # the same set in every step
        active = torch.randperm(w.K, generator=g0, device=device)[:n_active]
        pick = torch.randint(0, n_active, (w.b,), generator=g, device=device)
        return active[pick].to(torch.int64)
    raise ValueError(w.labels)


def make_samples(w: Workload, step: int, device="cpu", rows: int = None) -> torch.Tensor:
    """Sample tensors [rows or b, *shape] of the mini-batch of one step."""
    g = _generator(w, 1_000_000 + step, device)
    n = w.b if rows is None else rows
    if w.values == "normal":
        x = torch.randn((n, *w.shape), generator=g, device=device, dtype=torch.float32)
        return x.to(w.torch_dtype)
    if w.values == "uniform":
        return torch.rand((n, *w.shape), generator=g, device=device, dtype=w.torch_dtype)
    raise ValueError(w.values)


def make_batch(w: Workload, step: int, device="cpu"):
    """(batch_x [b,*shape], batch_y [b] int64) of one step."""
    return make_samples(w, step, device), make_labels(w, step, device)


def as_row_bytes(x: torch.Tensor) -> np.ndarray:
    """Host uint8 view [rows, row_bytes] of a batch of samples (copies to the host if needed)."""
    t = x.detach().contiguous().cpu()
    return t.view(torch.uint8).reshape(t.shape[0], -1).numpy()
