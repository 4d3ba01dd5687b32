"""CAOTE oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes front end to ``caote_oracle.c`` (plain scalar fp64 C written from the
paper's definitions).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP path never
does, and this package never imports the HIP path.

The batched helpers below only loop the single-instance C routines over
(sequence, KV head) and widen inputs to fp64; they contain no arithmetic of the
method.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "caote_oracle.c")
_LIB = os.path.join(_HERE, "libcaote_oracle.so")

BASE_NONE, BASE_H2O, BASE_SNAPKV = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no intrinsics, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = f"{_LIB}.{os.getpid()}.tmp"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)
_bp = ctypes.POINTER(ctypes.c_ubyte)


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i, dbl, sz = ctypes.c_int, ctypes.c_double, ctypes.c_size_t
        L.oracle_window_attention.argtypes = [_dp, _dp, i, i, i, i, dbl, i, _dp]
        L.oracle_window_attention.restype = i
        L.oracle_column_sums.argtypes = [_dp, i, i, _dp]
        L.oracle_column_sums.restype = None
        L.oracle_base_score.argtypes = [_dp, _dp, i, i, i, i, i, _dp]
        L.oracle_base_score.restype = None
        L.oracle_caote_scores.argtypes = [_dp, _dp, i, i, i, i, i, _dp, _dp, _dp]
        L.oracle_caote_scores.restype = None
        L.oracle_score.argtypes = [_dp, _dp, _dp, _dp, i, i, i, i, dbl, i, i, i, i, i, i, _dp, _dp]
        L.oracle_score_given_lse.restype = ctypes.c_int
        L.oracle_score_given_lse.argtypes = [_dp, _dp, _dp, _dp, i, i, i, i, dbl, i, i, i, i, i, i,
                                             _dp, _dp, _dp]
        L.oracle_window_attention_given_lse.restype = ctypes.c_int
        L.oracle_window_attention_given_lse.argtypes = [_dp, _dp, i, i, i, i, dbl, i, _dp, _dp]
        L.oracle_row_lse.restype = ctypes.c_int
        L.oracle_row_lse.argtypes = [_dp, _dp, i, i, i, i, dbl, i, _dp]
        L.oracle_score.restype = i
        L.oracle_select.argtypes = [_dp, i, i, _ip]
        L.oracle_select.restype = None
        L.oracle_compact_stable.argtypes = [_bp, i, sz, _ip, i]
        L.oracle_compact_stable.restype = i
        L.oracle_compact_swap_last.argtypes = [_bp, i, sz, _ip, i]
        L.oracle_compact_swap_last.restype = i
        L.oracle_compact_fill.argtypes = [_bp, i, sz, _ip, i]
        L.oracle_compact_fill.restype = i
        L.oracle_bruteforce_eviction_error.argtypes = [_dp, _dp, i, i, _dp]
        L.oracle_bruteforce_eviction_error.restype = None
        L.oracle_bruteforce_delete_token.argtypes = [_dp, _dp, _dp, i, i, dbl, _dp]
        L.oracle_bruteforce_delete_token.restype = None
        L.oracle_joint_eviction_error.argtypes = [_dp, _dp, i, i, _ip, i]
        L.oracle_joint_eviction_error.restype = dbl
        L.oracle_joint_candidates.argtypes = [_dp, _dp, i, i, i, i, _ip, i, _dp]
        L.oracle_joint_candidates.restype = None
        L.oracle_greedy_joint_evict.argtypes = [_dp, _dp, i, i, i, i, i, _ip, _dp]
        L.oracle_greedy_joint_evict.restype = i
        _lib = L
    return _lib


def _d(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    return x, x.ctypes.data_as(_dp)


# ---- single-instance wrappers (one sequence, one KV head) --------------------

def window_attention(q, k, G, W, scale, window_in_cache):
    """q [G*W, d], k [N, d] -> A [G*W, N]."""
    q, qp = _d(q)
    k, kp = _d(k)
    N, d = k.shape
    A = np.empty((G * W, N), dtype=np.float64)
    rc = lib().oracle_window_attention(qp, kp, G, W, N, d, float(scale), int(window_in_cache),
                                       A.ctypes.data_as(_dp))
    if rc != 0:
        raise ValueError("oracle_window_attention: a query row has no visible key")
    return A


def row_lse(q, k, G, W, scale, window_in_cache):
    """q [G*W, d], k [N, d] -> natural-log normaliser of every query row, [G*W]."""
    q, qp = _d(q)
    k, kp = _d(k)
    N, d = k.shape
    out = np.empty(G * W, dtype=np.float64)
    rc = lib().oracle_row_lse(qp, kp, G, W, N, d, float(scale), int(window_in_cache),
                              out.ctypes.data_as(_dp))
    if rc != 0:
        raise ValueError("oracle_row_lse: a query row has no visible key")
    return out


def window_attention_given_lse(q, k, G, W, scale, window_in_cache, lse):
    """A_rj = exp(scale q_r.k_j - lse_r) for the visible keys, 0 elsewhere."""
    q, qp = _d(q)
    k, kp = _d(k)
    lse, lp = _d(lse)
    N, d = k.shape
    A = np.empty((G * W, N), dtype=np.float64)
    rc = lib().oracle_window_attention_given_lse(qp, kp, G, W, N, d, float(scale),
                                                 int(window_in_cache), lp, A.ctypes.data_as(_dp))
    if rc != 0:
        raise ValueError("oracle_window_attention_given_lse: a query row has no visible key")
    return A


def column_sums(A):
    A, Ap = _d(A)
    R, N = A.shape
    a = np.empty(N, dtype=np.float64)
    lib().oracle_column_sums(Ap, R, N, a.ctypes.data_as(_dp))
    return a


def base_score(a, h_in, base, pool_kernel, lo, hi):
    a, ap = _d(a)
    N = a.shape[0]
    h = np.empty(N, dtype=np.float64)
    if h_in is not None:
        h_in, hp = _d(h_in)
    else:
        hp = None
    lib().oracle_base_score(ap, hp, N, base, pool_kernel, lo, hi, h.ctypes.data_as(_dp))
    return h


def caote_scores(h, v, lo=0, hi=None, fast=False):
    """h [N], v [N, d] -> (c [N], w [N], o [d])."""
    h, hp = _d(h)
    v, vp = _d(v)
    N, d = v.shape
    hi = N if hi is None else hi
    c = np.empty(N, dtype=np.float64)
    w = np.empty(N, dtype=np.float64)
    o = np.empty(d, dtype=np.float64)
    lib().oracle_caote_scores(hp, vp, N, d, lo, hi, int(fast), c.ctypes.data_as(_dp),
                              w.ctypes.data_as(_dp), o.ctypes.data_as(_dp))
    return c, w, o


def score_one(q, k, v, h_in, G, W, scale, window_in_cache, base, pool_kernel=1,
              n_protect_head=0, n_protect_tail=0, fast=False, lse=None):
    """One (sequence, KV head).  Returns (c [N], h [N], a [N]).  lse: the caller's row
    normalisers [G*W] (natural log) or None."""
    q, qp = _d(q)
    k, kp = _d(k)
    v, vp = _d(v)
    N, d = k.shape
    h = np.zeros(N, dtype=np.float64) if h_in is None else np.array(h_in, dtype=np.float64)
    c = np.empty(N, dtype=np.float64)
    a = np.empty(N, dtype=np.float64)
    if lse is not None:
        lse, lp = _d(lse)
        assert lse.shape == (G * W,)
    else:
        lp = None
    rc = lib().oracle_score_given_lse(qp, kp, vp, h.ctypes.data_as(_dp), G, W, N, d,
                                      float(scale), int(window_in_cache), base, pool_kernel,
                                      n_protect_head, n_protect_tail, int(fast), lp,
                                      c.ctypes.data_as(_dp), a.ctypes.data_as(_dp))
    if rc != 0:
        raise ValueError(f"oracle_score failed rc={rc}")
    return c, h, a


def select_one(c, budget):
    c, cp = _d(c)
    idx = np.empty(budget, dtype=np.int32)
    lib().oracle_select(cp, c.shape[0], budget, idx.ctypes.data_as(_ip))
    return idx


def compact_one(rows, idx, mode="stable"):
    """rows: numpy array [N, ...] of any dtype (modified copy returned), idx int32 [budget].
    Returns (rows_after, new_len)."""
    rows = np.ascontiguousarray(rows).copy()
    N = rows.shape[0]
    row_bytes = rows.nbytes // max(N, 1)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    fn = {"stable": lib().oracle_compact_stable, "swap_last": lib().oracle_compact_swap_last,
          "fill": lib().oracle_compact_fill}[mode]
    n = fn(rows.ctypes.data_as(_bp), N, row_bytes, idx.ctypes.data_as(_ip), idx.shape[0])
    if n < 0:
        raise ValueError("oracle compact: swap_last needs exactly one evicted token")
    return rows, n


def bruteforce_eviction_error(w, v):
    w, wp = _d(w)
    v, vp = _d(v)
    N, d = v.shape
    e = np.empty(N, dtype=np.float64)
    lib().oracle_bruteforce_eviction_error(wp, vp, N, d, e.ctypes.data_as(_dp))
    return e


def bruteforce_delete_token(q, k, v, scale):
    q, qp = _d(q)
    k, kp = _d(k)
    v, vp = _d(v)
    N, d = k.shape
    e = np.empty(N, dtype=np.float64)
    lib().oracle_bruteforce_delete_token(qp, kp, vp, N, d, float(scale), e.ctypes.data_as(_dp))
    return e


def joint_eviction_error(w, v, token_set):
    w, wp = _d(w)
    v, vp = _d(v)
    N, d = v.shape
    s = np.ascontiguousarray(token_set, dtype=np.int32)
    return lib().oracle_joint_eviction_error(wp, vp, N, d, s.ctypes.data_as(_ip), s.shape[0])


def joint_candidates(w, v, gone, lo=0, hi=None):
    """Joint error of evicting token j on top of the tokens in `gone`, for every scored j
    not in `gone`; NaN elsewhere.  w [N] (sums to 1 over [lo,hi)), v [N, d] -> c [N]."""
    w, wp = _d(w)
    v, vp = _d(v)
    N, d = v.shape
    hi = N if hi is None else hi
    s = np.ascontiguousarray(gone, dtype=np.int32)
    c = np.empty(N, dtype=np.float64)
    lib().oracle_joint_candidates(wp, vp, N, d, lo, hi, s.ctypes.data_as(_ip), s.shape[0],
                                  c.ctypes.data_as(_dp))
    return c


def greedy_joint_evict(w, v, m, lo=0, hi=None):
    """Greedy eviction of m tokens by the joint error.  w [N] (sums to 1 over [lo,hi)),
    v [N, d] -> (order [m] int32, err [m]): the token evicted at each step and the joint
    error of everything evicted up to and including it."""
    w, wp = _d(w)
    v, vp = _d(v)
    N, d = v.shape
    hi = N if hi is None else hi
    order = np.empty(m, dtype=np.int32)
    err = np.empty(m, dtype=np.float64)
    rc = lib().oracle_greedy_joint_evict(wp, vp, N, d, lo, hi, m, order.ctypes.data_as(_ip),
                                         err.ctypes.data_as(_dp))
    if rc != 0:
        raise ValueError("oracle_greedy_joint_evict: bad arguments")
    return order, err


# ---- batched loops over (sequence, KV head) ----------------------------------

def score_batched(q, K, V, h_in, seq_lens, *, n_kv_heads, window, scale, window_in_cache,
                  base, pool_kernel=1, n_protect_head=0, n_protect_tail=0, fast=False,
                  threads=1, lse=None):
    """q [B, Hq, W, d], K/V [B, Hkv, cap, d], h_in [B, Hkv, cap] or None,
    seq_lens [B] or None.  Returns (scores, h, a), each [B, Hkv, cap] fp64; entries at
    or beyond a sequence's length are NaN.  The ctypes calls release the GIL, so
    `threads` > 1 runs instances on several cores.  lse: [B, Hq, W] row normalisers handed
    over by the caller (natural log) or None."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, Hq, W, d = q.shape
    cap = K.shape[2]
    G = Hq // n_kv_heads
    assert W == window
    out_c = np.full((B, n_kv_heads, cap), np.nan)
    out_h = np.full((B, n_kv_heads, cap), np.nan)
    out_a = np.full((B, n_kv_heads, cap), np.nan)

    def one(bh):
        b, hk = bh
        N = cap if seq_lens is None else int(seq_lens[b])
        if N <= 0:
            return
        qg = q[b, hk * G:(hk + 1) * G].reshape(G * W, d)
        hin = None if h_in is None else np.asarray(h_in[b, hk, :N], dtype=np.float64)
        lg = None if lse is None else np.asarray(lse[b, hk * G:(hk + 1) * G], dtype=np.float64).reshape(G * W)
        c, h, a = score_one(qg, K[b, hk, :N], V[b, hk, :N], hin, G, W, scale, window_in_cache,
                            base, pool_kernel, n_protect_head, n_protect_tail, fast, lg)
        out_c[b, hk, :N], out_h[b, hk, :N], out_a[b, hk, :N] = c, h, a

    work = [(b, hk) for b in range(B) for hk in range(n_kv_heads)]
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, work))
    else:
        for bh in work:
            one(bh)
    return out_c, out_h, out_a


def select_batched(scores, seq_lens, budget):
    """scores [B, Hkv, cap] -> kept_idx [B, Hkv, budget] int32 (ascending, -1 padded)."""
    scores = np.asarray(scores, dtype=np.float64)
    B, H, cap = scores.shape
    out = np.empty((B, H, budget), dtype=np.int32)
    for b in range(B):
        N = cap if seq_lens is None else int(seq_lens[b])
        for hk in range(H):
            out[b, hk] = select_one(scores[b, hk, :N], budget)
    return out
