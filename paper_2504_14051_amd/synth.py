"""Seeded synthetic KV caches for the CAOTE score / select / compact path.

This module is the single source of inputs for the HIP path, the CPU oracle and the
benchmark.  It holds none of the method's arithmetic (no softmax, no scores): it only
draws random tensors with the structure of a real cache -- an attention sink, a few
heavy-hitter keys aligned with the mean window query, log-normal value norms -- in the
shapes of Llama-3 / Qwen2.5 layers, and rounds them to the storage dtype.  They stand
in for the long-context task inputs of the paper's Sec. 4 (1.5k-32k token prompts,
budgets 2k-8k), which need datasets and trained weights that are not available.

Everything is generated on the host with numpy's counter-based Philox generator, keyed
by (seed, tensor id, sequence), so any sequence can be regenerated independently.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_NONE, BASE_H2O, BASE_SNAPKV = 0, 1, 2
_BASE_NAMES = {"none": BASE_NONE, "h2o": BASE_H2O, "snapkv": BASE_SNAPKV}


@dataclass(frozen=True)
class Workload:
    """Shape of one scoring/eviction call (one layer)."""
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "bf16" | "f32"
    context: int          # N (capacity of the cache; ragged batches use seq_lens <= context)
    window: int           # W
    budget: int           # b
    base: int             # BASE_*
    pool_kernel: int = 1
    n_protect_head: int = 0
    n_protect_tail: int = 0
    window_in_cache: int = 1
    seed: int = 20250414
    n_heavy: int = 16

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def tiny() -> Workload:
    return Workload("tiny", 1, 1, 1, 64, "f32", 512, 8, 128, BASE_H2O, seed=20250414)


def llama3_8b_4k() -> Workload:
    return Workload("llama3-8b-4k", 1, 32, 8, 128, "bf16", 4096, 32, 1024, BASE_H2O,
                    seed=20250415)


def llama3_8b_32k() -> Workload:
    return Workload("llama3-8b-32k", 1, 32, 8, 128, "bf16", 32768, 64, 2048, BASE_SNAPKV,
                    pool_kernel=7, n_protect_tail=64, seed=20250416)


def qwen25_7b_128k() -> Workload:
    return Workload("qwen2.5-7b-128k", 1, 28, 4, 128, "bf16", 131072, 32, 4096, BASE_SNAPKV,
                    pool_kernel=7, n_protect_tail=32, seed=20250417)


def decode_step(batch: int = 16) -> Workload:
    """One layer of the decode-time stream: caches at budget 2048 plus the appended token,
    one query position, evict one token per head."""
    return Workload("llama3-8b-decode", batch, 32, 8, 128, "bf16", 2049, 1, 2048, BASE_H2O,
                    seed=20250418)


def prefill_block(batch: int = 1) -> Workload:
    """One step of block-wise prefill with eviction (Sec. 2, block-wise prefill; Sec. 4 set-up):
    the cache holds its budget of 2048 tokens plus the block of 128 just appended, the block's
    128 query positions form the window, and 128 tokens are evicted."""
    return Workload("llama3-8b-prefill-block", batch, 32, 8, 128, "bf16", 2048 + 128, 128, 2048,
                    BASE_H2O, seed=20250419)


WORKLOADS = {
    "tiny": tiny,
    "llama3-8b-4k": llama3_8b_4k,
    "llama3-8b-32k": llama3_8b_32k,
    "qwen2.5-7b-128k": qwen25_7b_128k,
    "llama3-8b-decode": decode_step,
    "llama3-8b-prefill-block": prefill_block,
}


def _rng(seed: int, tensor_id: int, seq: int, layer: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 20) ^ (layer << 8) ^ tensor_id, seq]))


def prefill_lengths(seed: int, batch: int, lo: int = 8192, hi: int = 32768) -> np.ndarray:
    """Ragged prefill lengths, uniform in [lo, hi]."""
    return _rng(seed, 99, 0).integers(lo, hi + 1, size=batch).astype(np.int32)


@dataclass
class Cache:
    """Host tensors of one layer.  q [B,Hq,W,d], K/V [B,Hkv,cap,d] in the storage dtype;
    base [B,Hkv,cap] fp32 (H2O accumulator, zeros for a first call); seq_lens [B] int32 or
    None (all sequences hold `context` tokens).  Rows at or beyond a sequence's length are
    NaN so that any read past the end shows up in the result."""
    wl: Workload
    q: torch.Tensor
    K: torch.Tensor
    V: torch.Tensor
    base: torch.Tensor
    seq_lens: torch.Tensor | None


def make_cache(wl: Workload, seq_lens=None, layer: int = 0, base_init: str = "zeros") -> Cache:
    B, Hq, Hkv, d, W, cap = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.context
    G = wl.group
    q = np.empty((B, Hq, W, d), dtype=np.float32)
    K = np.full((B, Hkv, cap, d), np.nan, dtype=np.float32)
    V = np.full((B, Hkv, cap, d), np.nan, dtype=np.float32)
    base = np.zeros((B, Hkv, cap), dtype=np.float32)
    for b in range(B):
        N = cap if seq_lens is None else int(seq_lens[b])
        assert W <= N <= cap
        rq, rk, rv, rm = (_rng(wl.seed, t, b, layer) for t in (1, 2, 3, 4))
        mu = rm.standard_normal((Hkv, 1, 1, d), dtype=np.float32)          # shared per group
        qb = rq.standard_normal((Hkv, G, W, d), dtype=np.float32) + mu
        q[b] = qb.reshape(Hq, W, d)
        k = rk.standard_normal((Hkv, N, d), dtype=np.float32)
        v = rv.standard_normal((Hkv, N, d), dtype=np.float32)
        k[:, 0, :] *= 8.0                                                    # attention sink
        n_free = N - W - 1
        n_heavy = min(wl.n_heavy, max(n_free, 0))
        for hk in range(Hkv):
            if n_heavy > 0:
                qbar = qb[hk].reshape(G * W, d).mean(axis=0).astype(np.float64)
                qhat = qbar / np.linalg.norm(qbar)
                heavy = 1 + rm.choice(n_free, size=n_heavy, replace=False)
                for j in heavy:
                    kj = k[hk, j].astype(np.float64)
                    norm = np.linalg.norm(kj)
                    orth = kj - (kj @ qhat) * qhat
                    orth /= np.linalg.norm(orth)
                    k[hk, j] = (norm * (0.6 * qhat + 0.8 * orth)).astype(np.float32)
        g = rv.standard_normal((Hkv, N, 1), dtype=np.float32)
        v *= np.exp(0.5 * g)                                                 # log-normal norms
        K[b, :, :N] = k
        V[b, :, :N] = v
        if base_init == "random":                                            # a carried accumulator
            base[b, :, :N] = rm.random((Hkv, N), dtype=np.float32) * (4.0 * G * W / N)
    dt = wl.torch_dtype
    return Cache(
        wl=wl,
        q=torch.from_numpy(q).to(dt),
        K=torch.from_numpy(K).to(dt),
        V=torch.from_numpy(V).to(dt),
        base=torch.from_numpy(base),
        seq_lens=None if seq_lens is None else torch.as_tensor(np.asarray(seq_lens), dtype=torch.int32),
    )


def decode_append(wl: Workload, step: int, layer: int = 0):
    """What one generation step brings: a fresh query position per head and one new (k, v) row
    per (sequence, KV head), with the statistics of `make_cache` (queries share the group's
    component mu_g of sequence b, which stays the same over the steps; log-normal value norm).
    Returns (q [B,Hq,1,d], k_new [B,Hkv,1,d], v_new [B,Hkv,1,d]) in the storage dtype."""
    B, Hq, Hkv, d, G = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.group
    q = np.empty((B, Hq, 1, d), dtype=np.float32)
    k = np.empty((B, Hkv, 1, d), dtype=np.float32)
    v = np.empty((B, Hkv, 1, d), dtype=np.float32)
    for b in range(B):
        mu = _rng(wl.seed, 4, b, layer).standard_normal((Hkv, 1, 1, d), dtype=np.float32)
        r = _rng(wl.seed, 5, b * 65536 + step, layer)
        q[b] = (r.standard_normal((Hkv, G, 1, d), dtype=np.float32) + mu).reshape(Hq, 1, d)
        k[b] = r.standard_normal((Hkv, 1, d), dtype=np.float32)
        v[b] = r.standard_normal((Hkv, 1, d), dtype=np.float32) * np.exp(
            0.5 * r.standard_normal((Hkv, 1, 1), dtype=np.float32))
    dt = wl.torch_dtype
    return torch.from_numpy(q).to(dt), torch.from_numpy(k).to(dt), torch.from_numpy(v).to(dt)
