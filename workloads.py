"""Seeded synthetic inputs for the five reduce workloads.

This module only *generates inputs* (object buffers, ready orders, failure
masks).  It holds none of the reduce method's arithmetic and is the one piece
of code that both the CPU oracle's tests and the GPU library's tests import.

The workloads stand in for the applications the paper evaluates (section 5):
  1  small all-ready reduce            (collective microbenchmark, 1 MB objects)
  2  asynchronous-SGD gradient reduce  (reduce over the first workers to finish)
  3  RL policy allreduce               (reduce + broadcast of a policy)
  4  large model, one participant fails mid-stream (section 5.4)
  5  ensemble serving, many sub-64-KB objects (appendix A sizes)
Only sizes, dtypes, value distributions and arrival structure matter to a
streaming reduce, so no model weights or datasets are involved.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

SEED_BASE = 200205814
ELEM_BYTES = {"f32": 4, "bf16": 2, "i32": 4}
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}


@dataclass(frozen=True)
class Workload:
    name: str
    n: int                      # source objects
    dtype: str                  # "f32" | "bf16" | "i32"
    object_bytes: int
    chunk_bytes: int
    k: int                      # objects to reduce (first k ready survivors)
    tree_degree: int            # 0 = library picks
    ops: Tuple[str, ...]        # "sum" | "min" | "max"
    dist: str                   # value recipe, see _fill
    order_seed: Optional[int]   # None = identity ready order
    data_seed: int
    fail: Dict[int, int] = field(default_factory=dict)   # object -> chunks delivered before failing
    n_dst: int = 0              # broadcast destinations (allreduce workloads)

    @property
    def n_elems(self) -> int:
        return self.object_bytes // ELEM_BYTES[self.dtype]

    @property
    def n_chunks(self) -> int:
        return max(1, -(-self.object_bytes // self.chunk_bytes))

    def scaled(self, object_bytes: int, chunk_bytes: Optional[int] = None, **kw) -> "Workload":
        """Same structure at another object size (for cases the oracle finishes in seconds)."""
        cb = chunk_bytes if chunk_bytes is not None else self.chunk_bytes
        return dataclasses.replace(self, object_bytes=object_bytes, chunk_bytes=cb, **kw)

    def ready_order(self) -> np.ndarray:
        if self.order_seed is None:
            return np.arange(self.n, dtype=np.int32)
        return np.random.default_rng(self.order_seed).permutation(self.n).astype(np.int32)

    def fail_mask(self) -> Optional[np.ndarray]:
        if not self.fail:
            return None
        m = np.full(self.n, -1, dtype=np.int64)
        for obj, chunks in self.fail.items():
            m[obj] = chunks
        return m


MiB = 1 << 20
KiB = 1 << 10

WORKLOADS: Dict[int, Workload] = {
    1: Workload("cfg1_small_allready", n=8, dtype="f32", object_bytes=1 * MiB, chunk_bytes=64 * KiB,
                k=8, tree_degree=2, ops=("sum",), dist="uniform_pm1", order_seed=None,
                data_seed=SEED_BASE + 1),
    2: Workload("cfg2_async_sgd", n=16, dtype="f32", object_bytes=64 * MiB, chunk_bytes=4 * MiB,
                k=12, tree_degree=4, ops=("sum",), dist="normal_std0.01", order_seed=58140002,
                data_seed=SEED_BASE + 2),
    3: Workload("cfg3_rl_allreduce", n=64, dtype="i32", object_bytes=16 * MiB, chunk_bytes=1 * MiB,
                k=64, tree_degree=0, ops=("sum",), dist="randint_pm2p20", order_seed=58140003,
                data_seed=SEED_BASE + 3, n_dst=64),
    4: Workload("cfg4_large_fault", n=32, dtype="bf16", object_bytes=256 * MiB, chunk_bytes=8 * MiB,
                k=32, tree_degree=8, ops=("sum",), dist="normal_std1", order_seed=58140004,
                data_seed=SEED_BASE + 4, fail={7: 10}),
    5: Workload("cfg5_ensemble_small", n=1024, dtype="f32", object_bytes=4 * KiB, chunk_bytes=4 * KiB,
                k=1000, tree_degree=16, ops=("max", "sum"), dist="softmax_normal", order_seed=58140005,
                data_seed=SEED_BASE + 5),
}


# Not one of the five: a deep bf16 tree for the degree ablation (64 inputs of 32 MiB; a binary tree over
# them needs 5 accumulator levels, a chain or a star one).
EXTRA_WORKLOADS: Dict[int, Workload] = {
    6: Workload("sweep_bf16_64x32MiB", n=64, dtype="bf16", object_bytes=32 * MiB, chunk_bytes=2 * MiB,
                k=64, tree_degree=0, ops=("sum",), dist="normal_std1", order_seed=58140006,
                data_seed=SEED_BASE + 6),
}


def _fill(w: Workload, n_elems: int, gen: torch.Generator, device) -> torch.Tensor:
    """One object's values, drawn from the workload's recipe."""
    if w.dist == "uniform_pm1":
        return torch.rand(n_elems, generator=gen, device=device, dtype=torch.float32) * 2.0 - 1.0
    if w.dist == "normal_std0.01":
        return torch.randn(n_elems, generator=gen, device=device, dtype=torch.float32) * 0.01
    if w.dist == "normal_std1":
        x = torch.randn(n_elems, generator=gen, device=device, dtype=torch.float32)
        return x.to(TORCH_DTYPE[w.dtype])
    if w.dist == "randint_pm2p20":
        return torch.randint(-(1 << 20), (1 << 20) + 1, (n_elems,), generator=gen, device=device,
                             dtype=torch.int32)
    if w.dist == "softmax_normal":
        logits = torch.randn(n_elems, generator=gen, device=device, dtype=torch.float32)
        return torch.softmax(logits, dim=0)
    raise ValueError(w.dist)


def make_objects(w: Workload, device="cpu", n_objects: Optional[int] = None) -> List[torch.Tensor]:
    """The workload's n source objects as 1-D tensors of w.dtype on `device`."""
    gen = torch.Generator(device=device)
    gen.manual_seed(w.data_seed)
    out = []
    for _ in range(w.n if n_objects is None else n_objects):
        t = _fill(w, w.n_elems, gen, device).to(TORCH_DTYPE[w.dtype]).contiguous()
        out.append(t)
    return out


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy for the oracle; bfloat16 comes back as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def from_numpy(a: np.ndarray, dtype: str, device="cpu") -> torch.Tensor:
    """Inverse of to_numpy."""
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)
