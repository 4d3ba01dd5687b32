"""ctypes binding of the C ABI in ``include/caote.h``.

Argument marshalling only: every step of the path runs in the HIP kernels of
``libcaote_hip.so``.  torch tensors are used as device memory (``data_ptr()``) and for
the current HIP stream; nothing here computes.  If the library has not been built the
calls raise -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcaote_hip.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EDEVICE = 0, -1, -2, -3, -4
BF16, F32 = 0, 1
BASE_NONE, BASE_H2O, BASE_SNAPKV = 0, 1, 2
EXACT, FAST = 0, 1
COMPACT_STABLE, COMPACT_SWAP_LAST, COMPACT_FILL = 0, 1, 2
FILL_MAX_BUDGET = 16384

EXPORTS = ("caote_workspace_bytes", "caote_score", "caote_select", "caote_compact",
           "caote_append", "caote_evict", "caote_evict_static", "caote_evict_joint", "caote_evict_prefix", "caote_read_stream", "caote_issue_probe", "caote_phase_name", "caote_last_error",
           "caote_version")
MAX_PHASES = 16
JOINT_MAX_CAPACITY = 8192
STATIC_SCRATCH_BYTES = 32 << 20


class CaoteError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"caote status {status}: {message}")
        self.status = status


class Layout(ctypes.Structure):
    """Mirror of ``struct caote_layout``."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("window", ctypes.c_int32), ("capacity", ctypes.c_int32),
        ("seq_lens", ctypes.c_void_p),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_n", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_n", ctypes.c_int64),
        ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64), ("q_stride_w", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("base", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("pool_kernel", ctypes.c_int32), ("window_in_cache", ctypes.c_int32),
        ("n_protect_head", ctypes.c_int32), ("n_protect_tail", ctypes.c_int32),
        ("variant", ctypes.c_int32),
        ("row_lse", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_14051_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lp = ctypes.POINTER(Layout)
        L.caote_workspace_bytes.argtypes = [lp, i32]
        L.caote_workspace_bytes.restype = sz
        L.caote_score.argtypes = [vp, vp, vp, vp, lp, vp, vp, sz, vp]
        L.caote_score.restype = ctypes.c_int
        L.caote_select.argtypes = [vp, lp, i32, vp, vp, sz, vp]
        L.caote_select.restype = ctypes.c_int
        L.caote_compact.argtypes = [vp, vp, vp, vp, lp, i32, i32, vp, sz, vp]
        L.caote_compact.restype = ctypes.c_int
        L.caote_append.argtypes = [vp, vp, vp, vp, vp, lp, i32, i32, vp]
        L.caote_append.restype = ctypes.c_int
        L.caote_evict.argtypes = [vp, vp, vp, vp, lp, i32, i32, vp, vp, vp, sz, vp]
        L.caote_evict.restype = ctypes.c_int
        L.caote_evict_static.argtypes = [vp, vp, vp, vp, lp, i32, i32, vp, vp, vp]
        L.caote_evict_static.restype = ctypes.c_int
        L.caote_evict_joint.argtypes = [vp, vp, vp, vp, lp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.caote_evict_joint.restype = ctypes.c_int
        L.caote_evict_prefix.argtypes = [vp, vp, vp, vp, lp, i32, i32, vp, vp, vp, sz, vp, i32,
                                         ctypes.POINTER(i32)]
        L.caote_evict_prefix.restype = ctypes.c_int
        L.caote_read_stream.argtypes = [vp, sz, vp, vp]
        L.caote_read_stream.restype = ctypes.c_int
        L.caote_issue_probe.argtypes = [i32, i32, vp, vp]
        L.caote_issue_probe.restype = ctypes.c_int
        L.caote_phase_name.argtypes = [i32]
        L.caote_phase_name.restype = ctypes.c_char_p
        L.caote_last_error.argtypes = []
        L.caote_last_error.restype = ctypes.c_char_p
        L.caote_version.argtypes = []
        L.caote_version.restype = i32
        _lib = L
    return _lib


def _check(st: int) -> None:
    if st != OK:
        raise CaoteError(st, lib().caote_last_error().decode())


def _ptr(t) -> int | None:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def make_layout(q, K, V, *, base, softmax_scale, window_in_cache=1, pool_kernel=1,
                n_protect_head=0, n_protect_tail=0, variant=EXACT, seq_lens=None,
                row_lse=None) -> Layout:
    """Layout of q [B,Hq,W,d], K/V [B,Hkv,cap,d] (innermost dimension contiguous).
    row_lse: optional fp32 device tensor [B,Hq,W], the caller's softmax normalisers."""
    B, Hq, W, d = q.shape
    _, Hkv, cap, _ = K.shape
    assert q.stride(3) == 1 and K.stride(3) == 1 and V.stride(3) == 1
    assert q.dtype == K.dtype == V.dtype and q.dtype in (torch.bfloat16, torch.float32)
    if row_lse is not None:
        assert row_lse.dtype == torch.float32 and row_lse.is_contiguous() and tuple(row_lse.shape) == (B, Hq, W)
    return Layout(
        batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, window=W, capacity=cap,
        seq_lens=_ptr(seq_lens),
        k_stride_b=K.stride(0), k_stride_h=K.stride(1), k_stride_n=K.stride(2),
        v_stride_b=V.stride(0), v_stride_h=V.stride(1), v_stride_n=V.stride(2),
        q_stride_b=q.stride(0), q_stride_h=q.stride(1), q_stride_w=q.stride(2),
        dtype=BF16 if q.dtype == torch.bfloat16 else F32, base=base,
        softmax_scale=softmax_scale, pool_kernel=pool_kernel, window_in_cache=window_in_cache,
        n_protect_head=n_protect_head, n_protect_tail=n_protect_tail, variant=variant,
        row_lse=_ptr(row_lse))


def caote_version() -> int:
    return lib().caote_version()


def caote_last_error() -> str:
    return lib().caote_last_error().decode()


def caote_workspace_bytes(layout: Layout, budget: int) -> int:
    n = lib().caote_workspace_bytes(ctypes.byref(layout), budget)
    if n == 0:
        raise CaoteError(EINVAL, caote_last_error())
    return n


def caote_score(q_window, K, V, base_score, layout: Layout, scores, workspace, stream=None,
                workspace_bytes=None) -> None:
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().caote_score(_ptr(q_window), _ptr(K), _ptr(V), _ptr(base_score), ctypes.byref(layout),
                             _ptr(scores), _ptr(workspace), wb, _stream(stream)))


def caote_select(scores, layout: Layout, budget: int, kept_idx, workspace, stream=None,
                 workspace_bytes=None) -> None:
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().caote_select(_ptr(scores), ctypes.byref(layout), budget, _ptr(kept_idx),
                              _ptr(workspace), wb, _stream(stream)))


def caote_compact(K, V, base_score, kept_idx, layout: Layout, budget: int, mode, workspace,
                  stream=None, workspace_bytes=None) -> None:
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().caote_compact(_ptr(K), _ptr(V), _ptr(base_score), _ptr(kept_idx),
                               ctypes.byref(layout), budget, mode, _ptr(workspace), wb,
                               _stream(stream)))


def caote_append(K, V, base_score, k_new, v_new, layout: Layout, n_at: int, n_new: int,
                 stream=None) -> None:
    _check(lib().caote_append(_ptr(K), _ptr(V), _ptr(base_score), _ptr(k_new), _ptr(v_new),
                              ctypes.byref(layout), n_at, n_new, _stream(stream)))


def caote_evict(q_window, K, V, base_score, layout: Layout, budget: int, mode, scores, kept_idx,
                workspace, stream=None, workspace_bytes=None) -> None:
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().caote_evict(_ptr(q_window), _ptr(K), _ptr(V), _ptr(base_score),
                             ctypes.byref(layout), budget, mode, _ptr(scores), _ptr(kept_idx),
                             _ptr(workspace), wb, _stream(stream)))


def caote_evict_static(q_window, K, V, base_score, layout: Layout, budget: int, mode, scores, kept_idx,
                       stream=None) -> None:
    """caote_evict on the library's own fixed scratch array (no workspace, no allocation)."""
    _check(lib().caote_evict_static(_ptr(q_window), _ptr(K), _ptr(V), _ptr(base_score),
                                    ctypes.byref(layout), budget, mode, _ptr(scores), _ptr(kept_idx),
                                    _stream(stream)))


def caote_evict_joint(q_window, K, V, base_score, layout: Layout, budget: int, mode, scores, kept_idx,
                      evicted, joint_error, workspace, stream=None, workspace_bytes=None) -> None:
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().caote_evict_joint(_ptr(q_window), _ptr(K), _ptr(V), _ptr(base_score),
                                   ctypes.byref(layout), budget, mode, _ptr(scores), _ptr(kept_idx),
                                   _ptr(evicted), _ptr(joint_error), _ptr(workspace), wb,
                                   _stream(stream)))


def caote_evict_prefix(q_window, K, V, base_score, layout: Layout, budget: int, mode, scores,
                       kept_idx, workspace, n_kernels: int, stream=None, workspace_bytes=None):
    """Measurement aid: only the first `n_kernels` kernels of the caote_evict call (all if
    negative).  Returns the names of the kernels that were enqueued."""
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    n = ctypes.c_int32(0)
    _check(lib().caote_evict_prefix(_ptr(q_window), _ptr(K), _ptr(V), _ptr(base_score),
                                    ctypes.byref(layout), budget, mode, _ptr(scores),
                                    _ptr(kept_idx), _ptr(workspace), wb, _stream(stream), n_kernels,
                                    ctypes.byref(n)))
    return [lib().caote_phase_name(i).decode() for i in range(min(n.value, MAX_PHASES))]


def caote_read_stream(buf, nbytes: int, sink, stream=None) -> None:
    """Measurement aid: one plain streaming read of `nbytes` at `buf`."""
    _check(lib().caote_read_stream(_ptr(buf), nbytes, _ptr(sink), _stream(stream)))


ISSUE_PROBE_VARIANTS = ("mfma_16", "vector_block", "mfma_then_vector", "mfma_fma_interleaved", "fma_128",
                        "intervals_opposite_halves", "intervals_same_order", "intervals_opposite_parity")
ISSUE_PROBE_OUT_BYTES = 256 * 512 * 4


def caote_issue_probe(variant: int, iters: int, out, stream=None) -> None:
    """Measurement aid: one launch of the issue-rate probe (see caote.h)."""
    _check(lib().caote_issue_probe(variant, iters, _ptr(out), _stream(stream)))


def layout_for(wl, cache_dev, row_lse=None) -> Layout:
    """Layout of a `synth.Cache` whose tensors live on the device, for workload `wl`."""
    return make_layout(cache_dev.q, cache_dev.K, cache_dev.V, base=wl.base,
                       softmax_scale=wl.softmax_scale, window_in_cache=wl.window_in_cache,
                       pool_kernel=wl.pool_kernel, n_protect_head=wl.n_protect_head,
                       n_protect_tail=wl.n_protect_tail, seq_lens=cache_dev.seq_lens,
                       row_lse=row_lse)
