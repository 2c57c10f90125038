"""Seeded synthetic inputs for the AdapShot KV-reuse hot path.

This module only *draws* inputs (shot lengths, selections, K/V/Q values, logits).
It contains none of the method's arithmetic (no rotation, no softmax, no entropy)
so that the CPU oracle and the HIP library can both be fed from it without
sharing any code of the method itself.

The five workloads are stand-ins for the paper's many-shot in-context-learning
runs (Experiments section: Qwen2.5-7B / LLaMA-3.2-3B with 64..1024 cached shots
per query); the paper's datasets and weights are not used.  Shapes follow the
model families named there: shot lengths are uniform in a closed range, K/V/Q are
N(0,1) (rounded to bf16 where the storage type is bf16) and logits are N(0, var 2).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np
import torch

SEED_BASE = 0xADA50000


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # 1-based config index
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_theta: float
    dtype: str                      # "f32" | "bf16"
    n_shots: int                    # pool size N
    len_lo: int                     # closed range of shot lengths
    len_hi: int
    m_select: int                   # shots assembled per query
    t_q: int                        # query tokens
    n_queries: int = 1              # independent queries (cfg 3: 8, cfg 5: 32)
    prefixes: Tuple[int, ...] = ()  # nested probe prefixes (cfg 3)
    decode_steps: int = 0           # single-token decode steps (cfg 5)
    entropy_rows: int = 0
    vocab: int = 0

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def kv_bytes_per_token_layer(self) -> int:
        """K row + V row of one token in one layer."""
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes


WORKLOADS = {
    "tiny_fp32": Workload("tiny_fp32", 1, 1, 4, 2, 64, 1.0e4, "f32", 16, 24, 40, 8, 16,
                          entropy_rows=16, vocab=1000),
    "llama8b_1layer": Workload("llama8b_1layer", 2, 1, 32, 8, 128, 5.0e5, "bf16", 2000, 48, 160, 256, 128,
                               entropy_rows=128, vocab=128256),
    "llama8b_sweep": Workload("llama8b_sweep", 3, 32, 32, 8, 128, 5.0e5, "bf16", 2000, 48, 160, 512, 64,
                              n_queries=8, prefixes=(16, 32, 64, 128, 256, 512),
                              entropy_rows=48, vocab=128256),
    "llama70b_128k": Workload("llama70b_128k", 4, 80, 64, 8, 128, 5.0e5, "bf16", 4000, 64, 192, 1000, 256,
                              entropy_rows=256, vocab=128256),
    "qwen7b_decode": Workload("qwen7b_decode", 5, 28, 28, 4, 128, 1.0e6, "bf16", 3000, 32, 128, 200, 1,
                              n_queries=32, decode_steps=64, entropy_rows=32, vocab=152064),
}


def shot_lengths(w: Workload) -> np.ndarray:
    """int64[N] shot lengths, uniform in [len_lo, len_hi]."""
    rng = np.random.default_rng(w.seed)
    return rng.integers(w.len_lo, w.len_hi, size=w.n_shots, endpoint=True).astype(np.int64)


def shot_offsets(w: Workload) -> np.ndarray:
    """int64[N+1] exclusive prefix sum of the shot lengths (token offsets in the pool)."""
    off = np.zeros(w.n_shots + 1, dtype=np.int64)
    np.cumsum(shot_lengths(w), out=off[1:])
    return off


def selection(w: Workload, query: int = 0, variant: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """(shot_ids int32[m], order int32[m]) for one query.

    shot_ids is a seeded m-subset of the pool in increasing id order; order is a
    seeded permutation of 0..m-1, so that slot j of the assembled context holds
    shot_ids[order[j]].  `variant` gives further independent draws for the same
    query (used to cycle distinct selections when timing).
    """
    rng = np.random.default_rng([w.seed, 1 + query, variant])
    ids = np.sort(rng.permutation(w.n_shots)[: w.m_select]).astype(np.int32)
    order = rng.permutation(w.m_select).astype(np.int32)
    return ids, order


def _torch_gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed & 0x7FFFFFFFFFFFFFFF)
    return g


def normal_tensor(shape, dtype: torch.dtype, device, seed: int, std: float = 1.0,
                  chunk_elems: int = 1 << 27) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 and rounded to `dtype`, generated in chunks along dim 0."""
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    g = _torch_gen(device, seed)
    n = flat.numel()
    for s in range(0, n, chunk_elems):
        e = min(n, s + chunk_elems)
        blk = torch.randn(e - s, dtype=torch.float32, device=device, generator=g)
        if std != 1.0:
            blk.mul_(std)
        flat[s:e].copy_(blk)
    return out


def make_pool(w: Workload, device, n_layers: Optional[int] = None) -> Tuple[torch.Tensor, torch.Tensor, np.ndarray]:
    """K_pool, V_pool of shape [L, pool_tokens, H_kv, d] (un-rotated keys) and the offsets."""
    off = shot_offsets(w)
    layers = w.n_layers if n_layers is None else n_layers
    shape = (layers, int(off[-1]), w.n_kv_heads, w.head_dim)
    k = normal_tensor(shape, w.torch_dtype, device, w.seed * 7 + 1)
    v = normal_tensor(shape, w.torch_dtype, device, w.seed * 7 + 2)
    return k, v, off


def make_query(w: Workload, device, query: int = 0, layer: int = 0, t_q: Optional[int] = None):
    """(Q [T_q,H_q,d], K_self [T_q,H_kv,d], V_self [T_q,H_kv,d]), all un-rotated."""
    t = w.t_q if t_q is None else t_q
    base = w.seed * 7 + 100 + 3 * (query * 1009 + layer)
    q = normal_tensor((t, w.n_q_heads, w.head_dim), w.torch_dtype, device, base)
    ks = normal_tensor((t, w.n_kv_heads, w.head_dim), w.torch_dtype, device, base + 1)
    vs = normal_tensor((t, w.n_kv_heads, w.head_dim), w.torch_dtype, device, base + 2)
    return q, ks, vs


def make_logits(w: Workload, device, n_rows: Optional[int] = None, variant: int = 0) -> torch.Tensor:
    """fp32 logits [rows, vocab] ~ N(0, variance 2)."""
    rows = w.entropy_rows if n_rows is None else n_rows
    return normal_tensor((rows, w.vocab), torch.float32, device, w.seed * 7 + 50 + variant, std=2.0 ** 0.5)


def as_numpy_storage(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor as the oracle's storage type: float32, or uint16 bit patterns for bf16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def from_numpy_storage(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    if dtype == torch.bfloat16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a))
