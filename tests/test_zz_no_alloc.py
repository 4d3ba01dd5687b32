"""caote_evict_static (the entry point that allocates nothing: its scratch is a fixed array in
the library's device image) against caote_evict with a caller-owned workspace, through the C
ABI: same bits on two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared array must not matter."""
import numpy as np
import pytest
import torch

import helpers as H
from paper_2504_14051_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2504_14051_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _evict(B, cache, budget, mode, static):
    wl = cache.wl
    dev = H.to_device(cache)
    L = B.layout_for(wl, dev)
    Bn, Hkv, cap = dev.K.shape[:3]
    scores = torch.full((Bn, Hkv, cap), float("nan"), device="cuda")
    kept = torch.full((Bn, Hkv, budget), -7, dtype=torch.int32, device="cuda")
    base = dev.base if wl.base == synth.BASE_H2O else None
    if static:
        B.caote_evict_static(dev.q, dev.K, dev.V, base, L, budget, mode, scores, kept)
    else:
        nb = B.caote_workspace_bytes(L, budget)
        assert nb <= B.STATIC_SCRATCH_BYTES
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        B.caote_evict(dev.q, dev.K, dev.V, base, L, budget, mode, scores, kept, ws)
    torch.cuda.synchronize()
    return dict(scores=scores.cpu(), kept=kept.cpu(), K=dev.K.cpu(), V=dev.V.cpu(),
                base=None if base is None else base.cpu())


def _same(a, b, cache, budget):
    assert torch.equal(a["kept"], b["kept"]), "kept_idx differs"
    sa, sb = a["scores"].numpy(), b["scores"].numpy()
    assert np.array_equal(sa, sb, equal_nan=True), "scores differ"
    for bi, N in enumerate(H.lengths(cache)):
        n = min(N, budget)
        for key in ("K", "V"):
            x, y = a[key][bi, :, :n], b[key][bi, :, :n]
            it = torch.int16 if x.dtype == torch.bfloat16 else torch.int32
            assert torch.equal(x.view(it), y.view(it)), f"compacted {key} differs"
        if a["base"] is not None:
            assert torch.equal(a["base"][bi, :, :n], b["base"][bi, :, :n]), "compacted accumulator differs"


def test_static_scratch_matches_workspace_call_twice_in_a_row(B):
    # first call: the 32k SnapKV layer (matrix-core sweeps, multi-workgroup selection, staged
    # compaction: every part of the scratch array is written)
    wl1 = synth.llama3_8b_32k()
    c1 = synth.make_cache(wl1)
    ref1 = _evict(B, c1, wl1.budget, 0, static=False)
    # second call, smaller: ragged H2O batch on the vector and few-row paths
    wl2 = synth.Workload("small-after-large", 2, 8, 2, 128, "bf16", 700, 8, 200, synth.BASE_H2O, seed=31)
    c2 = synth.make_cache(wl2, seq_lens=np.array([700, 333], dtype=np.int32), base_init="random")
    ref2 = _evict(B, c2, wl2.budget, 0, static=False)
    wl3 = synth.decode_step(batch=2)
    c3 = synth.make_cache(wl3, base_init="random")
    ref3 = _evict(B, c3, wl3.budget, 1, static=False)

    got1 = _evict(B, c1, wl1.budget, 0, static=True)
    got2 = _evict(B, c2, wl2.budget, 0, static=True)
    got3 = _evict(B, c3, wl3.budget, 1, static=True)
    _same(got1, ref1, c1, wl1.budget)
    _same(got2, ref2, c2, wl2.budget)
    _same(got3, ref3, c3, wl3.budget)


def test_static_scratch_rejects_what_does_not_fit(B):
    wl = synth.decode_step(batch=16)                 # its staging area alone exceeds the array
    dev = H.to_device(synth.make_cache(wl.with_(context=65, budget=64)))   # small tensors, big layout
    L = B.layout_for(wl.with_(context=65, budget=64), dev)
    L.capacity = wl.context
    L.k_stride_h = L.v_stride_h = wl.context * wl.head_dim
    L.k_stride_b = L.v_stride_b = wl.n_kv_heads * wl.context * wl.head_dim
    assert B.caote_workspace_bytes(L, wl.budget) > B.STATIC_SCRATCH_BYTES
    scores = torch.empty(1, device="cuda")
    kept = torch.empty(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.CaoteError) as e:           # rejected on the host: nothing is launched
        B.caote_evict_static(dev.q, dev.K, dev.V, dev.base, L, wl.budget, 1, scores, kept)
    assert e.value.status == B.EWORKSPACE and "static" in str(e.value)
