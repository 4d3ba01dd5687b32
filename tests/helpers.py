"""Shared pieces of the parity tests: device staging, oracle calls, comparison rules.

Comparison rules (bf16/fp32 inputs, fp32 accumulation on the GPU, fp64 oracle):
  scores   |gpu - orc| <= rtol*|orc| + 1e-6*max(orc), rtol 2e-3 (bf16) / 2e-4 (fp32);
           +INF (protected rows) must match exactly; tokens whose oracle weight is
           within 1e-3 of 1 (1 - w_j cancels in fp32) are only required to be kept.
  kept     with theta = the budget-th largest oracle score: every token above
           theta*(1+band) is kept, none below theta*(1-band), band = 2*rtol; exactly
           `budget` ascending unique indices.  No oracle score inside the band =>
           the sets are identical.
  compact  the oracle's gather applied to the GPU's own (validated) kept list,
           compared byte for byte.
"""
from __future__ import annotations

import os
from dataclasses import replace

import numpy as np
import torch

RTOL = {"bf16": 2e-3, "f32": 2e-4}


def host_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def to_device(cache, device="cuda"):
    return replace(
        cache,
        q=cache.q.to(device), K=cache.K.to(device), V=cache.V.to(device),
        base=cache.base.to(device),
        seq_lens=None if cache.seq_lens is None else cache.seq_lens.to(device))


def oracle_row_lse(oracle, cache):
    """What the caller's attention pass would hand over: natural-log normaliser of every
    window query row, [B, Hq, W] fp64, from the oracle's definition."""
    wl = cache.wl
    q = cache.q.cpu().double().numpy()
    K = cache.K.cpu().double().numpy()
    G = wl.n_q_heads // wl.n_kv_heads
    out = np.zeros((q.shape[0], wl.n_q_heads, wl.window))
    for b, N in enumerate(lengths(cache)):
        for hk in range(wl.n_kv_heads):
            if N <= 0:
                continue
            qg = q[b, hk * G:(hk + 1) * G].reshape(G * wl.window, -1)
            out[b, hk * G:(hk + 1) * G] = oracle.row_lse(
                qg, K[b, hk, :N], G, wl.window, float(np.float32(wl.softmax_scale)),
                wl.window_in_cache).reshape(G, wl.window)
    return out


def oracle_scores(oracle, cache, variant=0, threads=None, lse=None):
    """Oracle on the exact stored values.  Returns (c, h, a) as fp64 [B,Hkv,cap].
    lse: row normalisers [B,Hq,W] to use instead of the oracle's own softmax."""
    wl = cache.wl
    lens = None if cache.seq_lens is None else cache.seq_lens.cpu().numpy()
    return oracle.score_batched(
        cache.q.cpu().double().numpy(), cache.K.cpu().double().numpy(),
        cache.V.cpu().double().numpy(),
        cache.base.cpu().double().numpy() if wl.base == 1 else None, lens,
        n_kv_heads=wl.n_kv_heads, window=wl.window, scale=float(np.float32(wl.softmax_scale)),
        window_in_cache=wl.window_in_cache, base=wl.base, pool_kernel=wl.pool_kernel,
        n_protect_head=wl.n_protect_head, n_protect_tail=wl.n_protect_tail, fast=bool(variant),
        threads=threads or host_threads(), lse=lse)


def lengths(cache):
    B = cache.K.shape[0]
    if cache.seq_lens is None:
        return [cache.K.shape[2]] * B
    return [int(x) for x in cache.seq_lens.cpu()]


def check_scores(gpu, orc_c, orc_h, cache, rtol):
    """gpu: float32 [B,Hkv,cap] numpy; orc_*: fp64.  Returns the worst relative error."""
    worst = 0.0
    wl = cache.wl
    for b, N in enumerate(lengths(cache)):
        lo, hi = min(wl.n_protect_head, N), max(min(wl.n_protect_head, N), N - wl.n_protect_tail)
        for hk in range(gpu.shape[1]):
            g = gpu[b, hk, :N].astype(np.float64)
            o = orc_c[b, hk, :N]
            assert not np.isnan(g).any(), f"NaN score at b={b} head={hk}"
            inf_o = np.isinf(o)
            assert np.array_equal(np.isinf(g), inf_o), f"+INF pattern differs at b={b} head={hk}"
            fin = ~inf_o
            if not fin.any():
                continue
            h = orc_h[b, hk, :N]
            w = h / h[lo:hi].sum()
            near_one = fin & (1.0 - w < 1e-3)
            cmp = fin & ~near_one
            atol = 1e-6 * o[fin].max()
            err = np.abs(g[cmp] - o[cmp])
            bad = err > rtol * np.abs(o[cmp]) + atol
            if bad.any():
                j = np.nonzero(cmp)[0][np.argmax(err - rtol * np.abs(o[cmp]))]
                raise AssertionError(
                    f"score mismatch b={b} head={hk} token={j}: gpu={g[j]!r} oracle={o[j]!r} "
                    f"({bad.sum()} of {cmp.sum()} outside rtol={rtol})")
            rel = err / np.maximum(np.abs(o[cmp]), atol / rtol)
            worst = max(worst, float(rel.max()) if rel.size else 0.0)
    return worst


def check_kept(kept, orc_c, cache, budget, rtol, gpu_scores=None):
    """kept: int32 [B,Hkv,budget] from the GPU; orc_c fp64 oracle scores."""
    band = 2 * rtol
    n_exact = 0
    for b, N in enumerate(lengths(cache)):
        for hk in range(kept.shape[1]):
            idx = kept[b, hk]
            n_keep = min(N, budget)
            assert (idx[n_keep:] == -1).all(), "tail of kept_idx must be -1"
            idx = idx[:n_keep]
            assert (idx >= 0).all() and (idx < N).all()
            assert (np.diff(idx) > 0).all(), "kept_idx must be ascending and unique"
            if N <= budget:
                assert np.array_equal(idx, np.arange(N))
                continue
            o = orc_c[b, hk, :N]
            srt = np.sort(o)[::-1]
            theta = srt[budget - 1]
            in_set = np.zeros(N, bool)
            in_set[idx] = True
            if np.isinf(theta):          # budget filled by protected rows: lowest indices win
                ref = np.sort(np.lexsort((np.arange(N), -o))[:budget])
                assert np.array_equal(idx, ref)
                continue
            must = o > theta * (1 + band)
            must_not = o < theta * (1 - band)
            assert in_set[must].all(), f"b={b} head={hk}: a token clearly above the threshold was evicted"
            assert not in_set[must_not].any(), f"b={b} head={hk}: a token clearly below the threshold was kept"
            if not (~must & ~must_not).sum() > 1:
                ref = np.sort(np.lexsort((np.arange(N), -o))[:budget])
                assert np.array_equal(idx, ref)
                n_exact += 1
            if gpu_scores is not None:   # exact top-k of the GPU's own scores, ties to low index
                g = gpu_scores[b, hk, :N].astype(np.float64)
                ref = np.sort(np.lexsort((np.arange(N), -g))[:budget])
                assert np.array_equal(idx, ref), f"b={b} head={hk}: not the exact top-k of the scores given"
    return n_exact


def check_compaction(oracle, K_before, V_before, base_before, K_after, V_after, base_after, kept,
                     cache, budget, mode="stable"):
    """All tensors on the host.  K/V compared as raw bytes."""
    def raw(t):
        return t.contiguous().view(torch.uint8).numpy() if t.dtype != torch.bfloat16 else \
            t.contiguous().view(torch.int16).numpy()
    for b, N in enumerate(lengths(cache)):
        for hk in range(kept.shape[1]):
            n_keep = min(N, budget)
            m = mode
            if mode == "swap_last" and N - n_keep != 1:
                m = "stable"             # sequences that do not evict exactly one token
            for before, after in ((K_before, K_after), (V_before, V_after)):
                ref, n_new = oracle.compact_one(raw(before[b, hk, :N]), kept[b, hk], m)
                assert n_new == n_keep
                got = raw(after[b, hk, :n_keep])
                assert np.array_equal(got, ref[:n_keep]), f"compacted rows differ at b={b} head={hk}"
            if base_before is not None:
                ref, _ = oracle.compact_one(base_before[b, hk, :N].numpy().view(np.uint32), kept[b, hk], m)
                got = base_after[b, hk, :n_keep].numpy().view(np.uint32)
                assert np.array_equal(got, ref[:n_keep]), f"compacted accumulator differs at b={b} head={hk}"
