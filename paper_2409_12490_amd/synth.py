"""Seeded synthetic Q/K/V for the prefill-attention path (input recipe only).

This module draws the inputs that both the HIP path and the CPU checker are fed.
It holds none of the method's arithmetic: no pooling, scoring, selection or
attention happens here.  It needs numpy and torch (CPU) only and never touches
the GPU library or the checker.

Recipe (stands in for real Llama3-8B / Yi-9B activations, which the paper's
experiments section uses but which are not available offline):

* every (tensor, layer, batch, head) slice ``[n, d]`` has its own Philox
  stream keyed by ``(seed, tensor, layer, batch, head)``;
* per channel a random walk over positions, ``w[t] = w[t-1] + 0.1 * N(0,1)``
  with ``w[-1] = 0`` (0.1 is the standard deviation of a step), accumulated in
  float64, plus iid ``N(0,1)`` noise per token: ``x[t] = w[t] + e[t]``;
  adjacent tokens are therefore correlated, the locality the paper's
  "Locality Pattern of Query Criticality" section reports;
* ``unit_variance``: each whole tensor is divided by its own empirical
  standard deviation;
* ``hot_fraction`` > 0: every key position is "hot" independently with that
  probability (per batch and KV head) and hot keys get ``+3 * u`` added after
  scaling, ``u`` a random direction with ``||u|| = sqrt(d)`` (one per KV head),
  an attention-sink-like hotspot;
* finally values are rounded to the storage dtype (bf16 or fp32).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

_TENSOR_ID = {"q": 0, "k": 1, "v": 2, "hot": 3}


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and hyper-parameters of one attention layer workload."""

    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    segment_size: int
    block_size: int
    budget_blocks: int
    local_blocks: int
    dtype: str = "bf16"            # "bf16" | "fp32"
    unit_variance: bool = True
    hot_fraction: float = 0.0
    alpha: float = 1.0             # layer-fusion weight on the current layer
    layers: int = 1
    seed: int = 1234

    @property
    def n_segments(self) -> int:
        return -(-self.seq_len // self.segment_size)

    @property
    def n_blocks(self) -> int:
        return -(-self.seq_len // self.block_size)

    @property
    def blocks_per_segment(self) -> int:
        return self.segment_size // self.block_size

    @property
    def list_len(self) -> int:
        return self.budget_blocks + self.local_blocks + self.blocks_per_segment

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (shapes of Llama3-8B / Yi-9B attention).
WORKLOADS = {
    "c1_fp32_2k": Workload("c1_fp32_2k", 1, 1, 1, 128, 2048, 128, 32, 8, 0,
                           dtype="fp32", unit_variance=False, seed=1235),
    "c2_llama3_8b_16k": Workload("c2_llama3_8b_16k", 1, 32, 8, 128, 16384, 512, 64, 16, 1, seed=1236),
    "c3_llama3_8b_128k": Workload("c3_llama3_8b_128k", 1, 32, 8, 128, 131072, 512, 64, 32, 1, seed=1237),
    "c4_yi_9b_128k": Workload("c4_yi_9b_128k", 1, 32, 4, 128, 131072, 512, 64, 32, 1,
                              hot_fraction=0.05, seed=1238),
    "c5_llama3_8b_64k_x4": Workload("c5_llama3_8b_64k_x4", 2, 32, 8, 128, 65536, 256, 32, 32, 0,
                                    alpha=0.5, layers=4, seed=1239),
}


def _rng(seed: int, tensor: str, layer: int, batch: int, head: int) -> np.random.Generator:
    key = np.array([np.uint64(seed), (np.uint64(_TENSOR_ID[tensor]) << np.uint64(48))
                    | (np.uint64(layer) << np.uint64(32)) | (np.uint64(batch) << np.uint64(16))
                    | np.uint64(head)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def walk_slice(seed: int, tensor: str, layer: int, batch: int, head: int, n: int, d: int) -> np.ndarray:
    """One ``[n, d]`` float32 slice: per-channel random walk plus unit noise."""
    g = _rng(seed, tensor, layer, batch, head)
    out = np.empty((n, d), dtype=np.float32)
    chunk = 1 << 15
    carry = np.zeros(d, dtype=np.float64)
    for t0 in range(0, n, chunk):
        t1 = min(n, t0 + chunk)
        steps = g.standard_normal((t1 - t0, d), dtype=np.float32).astype(np.float64) * 0.1
        w = np.cumsum(steps, axis=0)
        w += carry
        carry = w[-1].copy()
        e = g.standard_normal((t1 - t0, d), dtype=np.float32)
        out[t0:t1] = (w + e).astype(np.float32)
    return out


def _tensor(w: Workload, tensor: str, heads: int, layer: int, threads: int) -> np.ndarray:
    x = np.empty((w.batch, heads, w.seq_len, w.head_dim), dtype=np.float32)

    def fill(bh):
        b, h = bh
        x[b, h] = walk_slice(w.seed, tensor, layer, b, h, w.seq_len, w.head_dim)

    jobs = [(b, h) for b in range(w.batch) for h in range(heads)]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    if w.unit_variance:
        # two-pass std over the whole tensor, accumulated per slice in float64
        cnt = x.size
        mean = sum(float(x[b, h].sum(dtype=np.float64)) for b, h in jobs) / cnt
        var = sum(float(((x[b, h].astype(np.float64) - mean) ** 2).sum()) for b, h in jobs) / cnt
        x *= np.float32(1.0 / np.sqrt(var))
    return x


def _add_hot_keys(w: Workload, k: np.ndarray, layer: int) -> None:
    d = w.head_dim
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            g = _rng(w.seed, "hot", layer, b, h)
            u = g.standard_normal(d)
            u *= np.sqrt(d) / np.linalg.norm(u)
            hot = g.random(w.seq_len) < w.hot_fraction
            k[b, h, hot] += (3.0 * u).astype(np.float32)


def _store(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(x)
    if dtype == "bf16":
        return t.to(torch.bfloat16)
    if dtype == "fp32":
        return t
    raise ValueError(f"unknown dtype {dtype!r}")


def make_qkv(w: Workload, layer: int = 0, threads: int = 8):
    """Return CPU tensors ``q [B,Hq,n,d]``, ``k, v [B,Hkv,n,d]`` in the storage dtype."""
    q = _tensor(w, "q", w.n_q_heads, layer, threads)
    k = _tensor(w, "k", w.n_kv_heads, layer, threads)
    v = _tensor(w, "v", w.n_kv_heads, layer, threads)
    if w.hot_fraction > 0.0:
        _add_hot_keys(w, k, layer)
    return _store(q, w.dtype), _store(k, w.dtype), _store(v, w.dtype)


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Widen a stored tensor (bf16/fp32, any device) to a float64 numpy array, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()
