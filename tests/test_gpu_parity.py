"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on
the same seeded inputs.  Comparison rules are in tests/helpers.py."""
import numpy as np
import pytest
import torch

import helpers as H
from paper_2504_14051_amd import synth

pytestmark = pytest.mark.gpu


CAP_JOINT = 8192      # CAOTE_JOINT_MAX_CAPACITY


@pytest.fixture(scope="module")
def B():
    from paper_2504_14051_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def run_path(B, cache, budget, mode=0, variant=0, fused=False, row_lse=None):
    """Runs score -> select -> compact on the device.  Returns host copies of every stage.
    row_lse: fp32 host tensor [B,Hq,W] handed over as the caller's softmax normalisers."""
    wl = cache.wl
    dev = H.to_device(cache)
    lse_dev = None if row_lse is None else row_lse.cuda()
    L = B.layout_for(wl, dev, row_lse=lse_dev)
    L.variant = variant
    nb = B.caote_workspace_bytes(L, budget)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    Bn, Hkv, cap = dev.K.shape[:3]
    scores = torch.full((Bn, Hkv, cap), float("nan"), device="cuda")
    kept = torch.full((Bn, Hkv, budget), -7, dtype=torch.int32, device="cuda")
    base = dev.base if wl.base == synth.BASE_H2O else None
    out = {}
    if fused:
        B.caote_evict(dev.q, dev.K, dev.V, base, L, budget, mode, scores, kept, ws)
    else:
        B.caote_score(dev.q, dev.K, dev.V, base, L, scores, ws)
        B.caote_select(scores, L, budget, kept, ws)
        torch.cuda.synchronize()
        out["K_before"], out["V_before"] = dev.K.cpu(), dev.V.cpu()
        out["base_before"] = None if base is None else base.cpu()
        B.caote_compact(dev.K, dev.V, base, kept, L, budget, mode, ws)
    torch.cuda.synchronize()
    out.update(scores=scores.cpu().numpy(), kept=kept.cpu().numpy(), K_after=dev.K.cpu(),
               V_after=dev.V.cpu(), base_after=None if base is None else base.cpu())
    return out


def full_check(B, oracle, cache, budget, mode=0, variant=0, row_lse=None):
    """row_lse: fp32 [B,Hq,W] normalisers that both sides take as given."""
    wl = cache.wl
    rtol = H.RTOL[wl.dtype]
    res = run_path(B, cache, budget, mode, variant, row_lse=row_lse)
    oc, oh, oa = H.oracle_scores(oracle, cache, variant,
                                 lse=None if row_lse is None else row_lse.double().numpy())
    worst = H.check_scores(res["scores"], oc, oh, cache, rtol)
    H.check_kept(res["kept"], oc, cache, budget, rtol, gpu_scores=res["scores"])
    if wl.base == synth.BASE_H2O:        # the accumulator now holds h for every row
        for b, N in enumerate(H.lengths(cache)):
            np.testing.assert_allclose(res["base_before"][b, :, :N].numpy(), oh[b, :, :N],
                                       rtol=rtol, atol=1e-7)
    H.check_compaction(oracle, res["K_before"], res["V_before"], res["base_before"],
                       res["K_after"], res["V_after"], res["base_after"], res["kept"], cache,
                       budget, ("stable", "swap_last", "fill")[mode])
    # rows past each sequence's length are never written
    for b, N in enumerate(H.lengths(cache)):
        assert np.isnan(res["scores"][b, :, N:]).all()
    # the fused entry point gives the same bits
    fz = run_path(B, cache, budget, mode, variant, fused=True, row_lse=row_lse)
    for key in ("scores", "kept"):
        assert np.array_equal(res[key], fz[key], equal_nan=True), f"caote_evict differs in {key}"
    for b, N in enumerate(H.lengths(cache)):
        n_keep = min(N, budget)
        for key in ("K_after", "V_after"):
            assert torch.equal(res[key][b, :, :n_keep].view(torch.int16 if wl.dtype == "bf16" else torch.int32),
                               fz[key][b, :, :n_keep].view(torch.int16 if wl.dtype == "bf16" else torch.int32))
        if wl.base == synth.BASE_H2O:    # the fused call moves the accumulator in code of its own
            assert torch.equal(res["base_after"][b, :, :n_keep].view(torch.int32),
                               fz["base_after"][b, :, :n_keep].view(torch.int32)), \
                "caote_evict differs in the compacted accumulator"
    return worst


def small(**kw):
    base = dict(name="small", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16",
                context=700, window=8, budget=200, base=synth.BASE_H2O, seed=77)
    base.update(kw)
    return synth.Workload(**base)


# ---- the named configurations ------------------------------------------------------

def test_tiny_fp32_h2o(B, oracle):
    wl = synth.tiny()
    worst = full_check(B, oracle, synth.make_cache(wl), wl.budget)
    assert worst < 2e-4


def test_llama3_8b_4k_h2o(B, oracle):
    wl = synth.llama3_8b_4k()
    full_check(B, oracle, synth.make_cache(wl), wl.budget)


def test_llama3_8b_32k_snapkv(B, oracle):
    wl = synth.llama3_8b_32k()
    full_check(B, oracle, synth.make_cache(wl), wl.budget)


def test_llama3_8b_32k_snapkv_given_row_normalisers(B, oracle):
    """The benchmark's second figure: the 32k layer with layout.row_lse set."""
    wl = synth.llama3_8b_32k()
    cache = synth.make_cache(wl)
    lse = torch.from_numpy(H.oracle_row_lse(oracle, cache)).float()
    full_check(B, oracle, cache, wl.budget, row_lse=lse)


@pytest.mark.parametrize("wl_fn,batch", [(synth.llama3_8b_32k, 8), (synth.llama3_8b_4k, 8)], ids=["32k", "4k"])
def test_eight_layers_as_one_call(B, oracle, wl_fn, batch):
    """The launch configuration of the benchmark's `layers_one_call` figure: eight caches of the
    named layer as the batch of one call (64 heads: longer key splits than the one-layer call)."""
    wl = wl_fn().with_(batch=batch)
    full_check(B, oracle, synth.make_cache(wl), wl.budget)


def test_qwen25_7b_128k_snapkv(B, oracle):
    wl = synth.qwen25_7b_128k()
    full_check(B, oracle, synth.make_cache(wl), wl.budget)


def test_decode_stream_steps(B, oracle):
    """Decode-time eviction: caches at budget+1, one query, evict one token per head with the
    last row dropping into the hole; several steps, the oracle restarted from the GPU's
    state at every step so that rounding does not pile up."""
    wl = synth.decode_step(batch=3)
    cache = synth.make_cache(wl, base_init="random")
    for step in range(4):
        full_check(B, oracle, cache, wl.budget, mode=1)
        res = run_path(B, cache, wl.budget, mode=1)
        fresh = synth.make_cache(wl, layer=step + 1, base_init="random")
        K, V, base = res["K_after"].clone(), res["V_after"].clone(), res["base_after"].clone()
        K[:, :, -1], V[:, :, -1] = fresh.K[:, :, -1], fresh.V[:, :, -1]     # appended token
        base[:, :, -1] = 0.0
        cache = synth.Cache(wl, fresh.q, K, V, base, None)


def test_append_rows_behind_each_sequence(B):
    """caote_append against plain tensor assignment: ragged lengths, a strided cache, rows that
    do not fit are dropped, the accumulator of the new rows is zero."""
    torch.manual_seed(5)
    Bn, Hkv, cap, d, n_new = 3, 2, 40, 128, 6
    big = torch.randn(Bn, Hkv, cap, 2 * d, device="cuda").to(torch.bfloat16)
    K, V = big[..., :d], big[..., d:]                      # row stride 2 d: strided views
    base = torch.rand(Bn, Hkv, cap, device="cuda")
    k_new = torch.randn(Bn, Hkv, n_new, d, device="cuda").to(torch.bfloat16)
    v_new = torch.randn(Bn, Hkv, n_new, d, device="cuda").to(torch.bfloat16)
    q = torch.zeros(Bn, Hkv, 1, d, device="cuda", dtype=torch.bfloat16)
    lens = torch.tensor([10, 34, 37], dtype=torch.int32, device="cuda")   # the last one overflows
    Kr, Vr, br = K.clone(), V.clone(), base.clone()
    for b, n in enumerate(lens.tolist()):
        m = min(n_new, cap - n)
        Kr[b, :, n:n + m], Vr[b, :, n:n + m], br[b, :, n:n + m] = k_new[b, :, :m], v_new[b, :, :m], 0.0
    L = B.make_layout(q, K, V, base=synth.BASE_H2O, softmax_scale=0.1, seq_lens=lens)
    B.caote_append(K, V, base, k_new, v_new, L, 0, n_new)
    torch.cuda.synchronize()
    assert torch.equal(K.view(torch.int16), Kr.view(torch.int16)) and torch.equal(V.view(torch.int16), Vr.view(torch.int16))
    assert torch.equal(base, br)
    # uniform position, no accumulator
    L2 = B.make_layout(q, K, V, base=synth.BASE_NONE, softmax_scale=0.1)
    B.caote_append(K, V, None, k_new, v_new, L2, 20, n_new)
    torch.cuda.synchronize()
    Kr[:, :, 20:26], Vr[:, :, 20:26] = k_new, v_new
    assert torch.equal(K.view(torch.int16), Kr.view(torch.int16)) and torch.equal(V.view(torch.int16), Vr.view(torch.int16))
    assert torch.equal(base, br)


def test_blockwise_prefill_stream(B, oracle):
    """Block-wise prefill with eviction (Sec. 2; Sec. 4 set-up, scaled down): blocks of 32 new
    tokens join a cache held at a budget of 256, the block's queries are the window, the H2O
    accumulator is carried, 32 tokens are evicted per block.  Each block is checked against
    the oracle started from the GPU's state, so rounding does not pile up."""
    wl = small(batch=2, context=256 + 32, window=32, budget=256, base=synth.BASE_H2O)
    cache = synth.make_cache(wl, base_init="random")
    dev = H.to_device(cache)
    ws = scores = kept = None
    for block in range(4):
        fresh = synth.make_cache(wl, layer=block + 1)
        k_new = fresh.K[:, :, -wl.window:].contiguous().cuda()
        v_new = fresh.V[:, :, -wl.window:].contiguous().cuda()
        L = B.layout_for(wl, dev)
        # append on the device, and the same by assignment for the oracle's input
        B.caote_append(dev.K, dev.V, dev.base, k_new, v_new, L, wl.budget, wl.window)
        torch.cuda.synchronize()
        host = synth.Cache(wl, fresh.q, dev.K.cpu(), dev.V.cpu(), dev.base.cpu(), None)
        assert torch.equal(host.K[:, :, wl.budget:].view(torch.int16), fresh.K[:, :, -wl.window:].view(torch.int16))
        assert (host.base[:, :, wl.budget:] == 0).all()
        full_check(B, oracle, host, wl.budget)
        # carry the GPU's own state on: evict on the device tensors
        dev = synth.Cache(wl, fresh.q.cuda(), dev.K, dev.V, dev.base, None)
        L = B.layout_for(wl, dev)
        if ws is None:
            ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
            scores = torch.empty(wl.batch, wl.n_kv_heads, wl.context, device="cuda")
            kept = torch.empty(wl.batch, wl.n_kv_heads, wl.budget, dtype=torch.int32, device="cuda")
        base_in = host.base.clone()
        B.caote_evict(dev.q, dev.K, dev.V, dev.base, L, wl.budget, 0, scores, kept, ws)
        torch.cuda.synchronize()
        # the state that the next block starts from: the accumulator h = h_in + a of the kept
        # rows (oracle), moved to the front as the GPU's own kept list says
        _, oh, _ = H.oracle_scores(oracle, host)
        kept_h = kept.cpu().numpy()
        got = dev.base.cpu()
        for b in range(wl.batch):
            for hk in range(wl.n_kv_heads):
                ref = oh[b, hk][kept_h[b, hk]]
                np.testing.assert_allclose(got[b, hk, :wl.budget].numpy(), ref, rtol=H.RTOL[wl.dtype], atol=1e-7)
        assert torch.equal(base_in, host.base)


# ---- configs[4] at its stated size: ragged batch-16 prefill eviction, then the decode stream ----

def test_cfg5_ragged_prefill_eviction_batch16_at_size(B, oracle):
    """The set-up of the decode stream as the workload states it: 16 sequences with prefill
    lengths uniform in 8k..32k, each cut to the budget of 2048 per KV head in ONE call with
    seq_lens (SnapKV base, window 64, pool 7): BH = 128, so the planner's key splits are the
    ones the benchmark's ragged call runs with, not those of a single layer."""
    wl = synth.llama3_8b_32k().with_(batch=16, name="llama3-8b-prefill-ragged16")
    lens = synth.prefill_lengths(wl.seed, wl.batch)
    assert lens.min() >= 8192 and lens.max() <= 32768 and len(set(lens.tolist())) > 8
    cache = synth.make_cache(wl, seq_lens=lens)
    full_check(B, oracle, cache, wl.budget)


def test_cfg5_decode_stream_batch16_256_steps(B, oracle):
    """The stream itself at the stated batch: 16 caches of 2048 + 1 rows per KV head, one query
    position per head, H2O accumulator carried, evict one per head, last row into the hole;
    256 steps on each of 2 layers.  The GPU runs all 16 sequences (BH = 128: the timed
    geometry); the oracle follows sequences 0 and 1, restarted from the GPU's own state at
    every step, and checks scores, accumulator, kept lists and the moved rows."""
    wl = synth.decode_step(batch=16)
    sub = wl.with_(batch=2)
    rtol = H.RTOL[wl.dtype]
    n_steps = 256
    for layer in range(2):
        dev = H.to_device(synth.make_cache(wl, layer=layer, base_init="random"))
        L = B.layout_for(wl, dev)
        ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
        scores = torch.empty(wl.batch, wl.n_kv_heads, wl.context, device="cuda")
        kept = torch.empty(wl.batch, wl.n_kv_heads, wl.budget, dtype=torch.int32, device="cuda")
        q = dev.q
        worst = 0.0
        for step in range(n_steps):
            before = synth.Cache(sub, q[:2].cpu(), dev.K[:2].cpu(), dev.V[:2].cpu(), dev.base[:2].cpu(), None)
            Lq = B.make_layout(q, dev.K, dev.V, base=wl.base, softmax_scale=wl.softmax_scale)
            B.caote_evict(q, dev.K, dev.V, dev.base, Lq, wl.budget, B.COMPACT_SWAP_LAST, scores, kept, ws)
            torch.cuda.synchronize()
            oc, oh, _ = H.oracle_scores(oracle, before, threads=16)
            sc, kp = scores[:2].cpu().numpy(), kept[:2].cpu().numpy()
            worst = max(worst, H.check_scores(sc, oc, oh, before, rtol))
            H.check_kept(kp, oc, before, wl.budget, rtol, gpu_scores=sc)
            # the accumulator after the step: h of every kept row, the last row in the hole
            got_base = dev.base[:2].cpu()
            K_after, V_after = dev.K[:2].cpu(), dev.V[:2].cpu()
            for b in range(2):
                for hk in range(wl.n_kv_heads):
                    ref, _ = oracle.compact_one(oh[b, hk], kp[b, hk], "swap_last")
                    np.testing.assert_allclose(got_base[b, hk, :wl.budget].numpy(), ref[:wl.budget],
                                               rtol=rtol, atol=1e-7)
            H.check_compaction(oracle, before.K, before.V, None, K_after, V_after, None, kp, before,
                               wl.budget, "swap_last")
            # the next token joins every cache
            q_h, k_new, v_new = synth.decode_append(wl, step, layer)
            q = q_h.cuda()
            B.caote_append(dev.K, dev.V, dev.base, k_new.cuda(), v_new.cuda(), L, wl.budget, 1)
        assert worst < rtol


# ---- shapes, modes, edges -------------------------------------------------------------

@pytest.mark.parametrize("kw", [
    dict(),                                                       # H2O, ragged below
    dict(base=synth.BASE_NONE),
    dict(base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=8),
    dict(base=synth.BASE_SNAPKV, pool_kernel=5, n_protect_tail=8, n_protect_head=4),
    dict(base=synth.BASE_H2O, n_protect_head=3, n_protect_tail=2),
    dict(head_dim=64),
    dict(head_dim=64, dtype="f32", base=synth.BASE_SNAPKV, pool_kernel=3, n_protect_tail=8),
    dict(dtype="f32"),
    dict(n_q_heads=14, n_kv_heads=2, window=5),                   # G = 7, R = 35
    dict(window=1, n_q_heads=2, n_kv_heads=2, base=synth.BASE_NONE),   # TOVA
    dict(window_in_cache=0),
    dict(window=40),                                              # R = 160: padded row blocks
    dict(window=80, base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=80),   # R = 320: two row groups
    dict(window=16, n_q_heads=2, n_kv_heads=2),                   # R = 16: vector-ALU path, bf16
    dict(window=17, n_q_heads=2, n_kv_heads=2),                   # R = 17: smallest matrix-core case
], ids=lambda kw: "-".join(f"{k}={v}" for k, v in kw.items()) or "h2o")
def test_small_shapes_ragged(B, oracle, kw):
    wl = small(**kw)
    lens = np.array([wl.context, 333], dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    full_check(B, oracle, cache, wl.budget)


@pytest.mark.parametrize("ragged", [False, True], ids=["dense", "ragged"])
def test_many_heads_short_caches(B, oracle, ragged):
    """12 sequences x 8 KV heads x 256 query rows on caches of a few hundred tokens: the row
    statistics are merged with one thread per row (batches of many heads), the splits are a
    tile or two long, and in the ragged case a workgroup's share of tiles spans several heads."""
    wl = small(batch=12, n_q_heads=32, n_kv_heads=8, window=64, context=520, budget=130,
               base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=64)
    lens = np.array([520, 64, 519, 130, 321, 65, 520, 448, 131, 200, 64, 385], dtype=np.int32) if ragged else None
    full_check(B, oracle, synth.make_cache(wl, seq_lens=lens), wl.budget)


@pytest.mark.parametrize("kw", [
    dict(window=64),                                   # R = 256: eight-wave matrix-core sweep
    dict(window=32, base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=32),   # R = 128
    dict(window=8),                                    # R = 32
    dict(window=1, budget=699),                        # R = 4: few-row path, evict one
    dict(window=3, n_q_heads=8, n_kv_heads=2),         # R = 12: vector-ALU sweeps
    dict(dtype="f32", head_dim=64, window=4),          # fp32
], ids=["r256", "r128-snapkv", "r32", "r4", "r12", "f32"])
@pytest.mark.parametrize("shift", [0.0, 0.6931471805599453], ids=["exact", "shifted"])
def test_row_normalisers_from_the_caller(B, oracle, kw, shift):
    """The first key sweep is skipped when the layout carries row_lse.  Both sides take the
    same fp32 normalisers as given: the oracle's own, or those shifted by ln 2 (which halves
    every attention mass: nothing is renormalised behind the caller's back)."""
    wl = small(**kw)
    lens = np.array([wl.context, 333], dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    lse = torch.from_numpy(H.oracle_row_lse(oracle, cache) + shift).float()
    mode = 1 if wl.window == 1 else 0
    full_check(B, oracle, cache, wl.budget, mode=mode, row_lse=lse)


@pytest.mark.parametrize("pool", [1, 33, 127, 129, 131, 301])
@pytest.mark.parametrize("window", [8, 64])
def test_snapkv_pool_widths(B, oracle, pool, window):
    """Pooling half-widths up to and beyond what the fused second sweep carries (64 keys), with
    splits shorter than the window they pool over; the widest ones fall back to the separate
    value-sum kernel."""
    wl = small(base=synth.BASE_SNAPKV, pool_kernel=pool, window=window, n_protect_tail=window,
               n_protect_head=3, context=1500, budget=400)
    lens = np.array([wl.context, 1500 - 257], dtype=np.int32)
    full_check(B, oracle, synth.make_cache(wl, seq_lens=lens), wl.budget)


@pytest.mark.parametrize("seed", range(16))
def test_random_layouts(B, oracle, seed):
    """Seeded random shapes across every key-sweep variant, base mode, dtype, window mode,
    budget and ragged lengths: whatever path the planner picks has to match the oracle."""
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 7]))
    d = int(rng.choice([64, 128]))
    dtype = "f32" if rng.random() < 0.25 else "bf16"
    W = int(rng.choice([1, 2, 5, 16, 33, 64]))
    batch = int(rng.integers(1, 4))
    context = int(rng.integers(W + 2, 3000))
    budget = int(rng.integers(1, context))
    base = int(rng.choice([synth.BASE_NONE, synth.BASE_H2O, synth.BASE_SNAPKV]))
    pool = int(rng.choice([1, 3, 7, 15])) if base == synth.BASE_SNAPKV else 1
    wic = int(rng.random() < 0.7)
    tail = int(rng.choice([0, 0, W, 3]))
    head = int(rng.choice([0, 0, 1, 4]))
    wl = synth.Workload(f"rand{seed}", batch, hkv * G, hkv, d, dtype, context, W, budget, base,
                        pool_kernel=pool, n_protect_head=head, n_protect_tail=tail,
                        window_in_cache=wic, seed=4242 + seed)
    lens = rng.integers(W + 1, context + 1, size=batch).astype(np.int32)
    lens[0] = context
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    mode = int(rng.random() < 0.3)
    full_check(B, oracle, cache, budget, mode=mode, variant=int(rng.random() < 0.3))


def joint_check(B, oracle, cache, budget, mode=0):
    """caote_evict_joint against the oracle's greedy (App. B).  A greedy choice is an argmin
    over floats and one different choice changes every later step, so the GPU's sequence is
    replayed: at step t, with the GPU's own first t evictions as S, the oracle's table of
    c_{S+j} says how good the GPU's next choice was.  It has to be the oracle's best within
    the rounding of the two candidates, |c| error <= 2 rtol (||u|| + w_j ||o - v_j||) / rest
    (the terms of the sum before they cancel); the reported error has the same bound."""
    wl = cache.wl
    rtol = H.RTOL[wl.dtype]
    ref = run_path(B, cache, budget, mode)              # scores and the state before compaction
    dev = H.to_device(cache)
    L = B.layout_for(wl, dev)
    ws = torch.empty(B.caote_workspace_bytes(L, budget), dtype=torch.uint8, device="cuda")
    Bn, Hkv, cap = dev.K.shape[:3]
    n_ev = cap - budget
    scores = torch.full((Bn, Hkv, cap), float("nan"), device="cuda")
    kept = torch.full((Bn, Hkv, budget), -7, dtype=torch.int32, device="cuda")
    evicted = torch.full((Bn, Hkv, n_ev), -7, dtype=torch.int32, device="cuda")
    jerr = torch.full((Bn, Hkv, n_ev), -7.0, device="cuda")
    base = dev.base if wl.base == synth.BASE_H2O else None
    B.caote_evict_joint(dev.q, dev.K, dev.V, base, L, budget, mode, scores, kept, evicted, jerr, ws)
    torch.cuda.synchronize()
    assert np.array_equal(scores.cpu().numpy(), ref["scores"], equal_nan=True)
    kept, evicted, jerr = kept.cpu().numpy(), evicted.cpu().numpy(), jerr.cpu().numpy()
    _, oh, _ = H.oracle_scores(oracle, cache)
    V = cache.V.double().numpy()
    n_same = n_steps = 0
    worst_margin = 0.0                  # largest (c[GPU's choice] - c[oracle's argmin]) / allowed slack seen
    for b, N in enumerate(H.lengths(cache)):
        lo = min(wl.n_protect_head, N)
        hi = max(lo, N - wl.n_protect_tail)
        m = min(N - min(N, budget), hi - lo)
        for hk in range(Hkv):
            v = V[b, hk, :N]
            _, w, o = oracle.caote_scores(oh[b, hk, :N], v, lo, hi)
            order = evicted[b, hk]
            assert (order[m:] == -1).all() and np.isnan(jerr[b, hk, m:]).all()
            assert len(set(order[:m].tolist())) == m and ((order[:m] >= lo) & (order[:m] < hi)).all()
            gnorm = w * np.linalg.norm(o - v, axis=1)
            u = np.zeros_like(o)
            rest_all = 1.0
            for t in range(m):
                c = oracle.joint_candidates(w, v, order[:t], lo, hi)
                s = int(order[t])
                j_best = int(np.nanargmin(c))
                scale = (np.linalg.norm(u) + gnorm) / np.maximum(rest_all - w, 1e-300)
                slack = 2 * rtol * (scale[s] + scale[j_best])
                if np.isfinite(c[j_best]):
                    assert c[s] <= c[j_best] + slack, (b, hk, t, s, j_best, c[s], c[j_best])
                    if slack > 0:
                        worst_margin = max(worst_margin, float((c[s] - c[j_best]) / slack))
                    if rest_all - w[s] > 1e-3:
                        assert abs(jerr[b, hk, t] - c[s]) <= 2 * rtol * scale[s] + 1e-30, (b, hk, t)
                n_same += s == j_best
                n_steps += 1
                u += w[s] * (o - v[s])
                rest_all -= w[s]
            want = np.setdiff1d(np.arange(N), order[:m])
            n_keep = min(N, budget)
            assert np.array_equal(kept[b, hk, :n_keep], want) and (kept[b, hk, n_keep:] == -1).all()
    H.check_compaction(oracle, ref["K_before"], ref["V_before"], ref["base_before"], dev.K.cpu(), dev.V.cpu(),
                       None if base is None else base.cpu(), kept, cache, budget,
                       ("stable", "swap_last", "fill")[mode])
    # how much of the replay bound the run used: a regression shows here long before it fails
    print(f"greedy replay: {n_same}/{n_steps} choices equal the oracle's argmin, "
          f"worst excess over the argmin = {worst_margin:.3f} of the allowed slack")
    return n_same, n_steps


@pytest.mark.parametrize("kw,budget", [
    (dict(context=700, window=8), 650),
    (dict(context=700, window=8, base=synth.BASE_NONE, n_protect_head=4, n_protect_tail=8), 600),
    (dict(context=1500, window=32, base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=32), 1400),
    (dict(context=300, window=4, head_dim=64, dtype="f32", n_q_heads=4, n_kv_heads=4), 250),
    (dict(context=513, window=1, head_dim=64, batch=3), 500),
    (dict(context=257, window=1), 256),
], ids=["h2o", "plain-protected", "snapkv", "f32-d64", "bf16-d64", "evict-one"])
def test_greedy_joint_eviction(B, oracle, kw, budget):
    wl = small(**kw)
    lens = None
    if wl.batch > 1 and wl.context > 400:
        lens = np.array([wl.context] + [wl.context - 37 * (i + 1) for i in range(wl.batch - 1)], dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    n_same, n_steps = joint_check(B, oracle, cache, budget, mode=1 if kw.get("context") == 257 else 0)
    assert n_same >= 0.9 * n_steps        # near-ties aside, the very sequence of the oracle's greedy


def test_greedy_joint_eviction_prefill_block(B, oracle):
    """The block-wise prefill step (2048 cached + 128 new rows, 128 leave), joint selection."""
    wl = synth.prefill_block()
    cache = synth.make_cache(wl, base_init="random")
    joint_check(B, oracle, cache, wl.budget)


def test_greedy_joint_eviction_with_fill_compaction(B, oracle):
    """The joint selection followed by the hole-filling compaction (ragged batch, 40 tokens leave)."""
    wl = small(context=600, window=8)
    cache = synth.make_cache(wl, seq_lens=np.array([600, 575], dtype=np.int32), base_init="random")
    joint_check(B, oracle, cache, 560, mode=2)


def test_greedy_joint_eviction_limits(B):
    wl = small(context=CAP_JOINT + 64, window=8)
    dev = H.to_device(synth.make_cache(wl))
    L = B.layout_for(wl, dev)
    ws = torch.empty(B.caote_workspace_bytes(L, 100), dtype=torch.uint8, device="cuda")
    args = lambda: (dev.q, dev.K, dev.V, dev.base, L, 100, 0, torch.empty(2, 2, wl.context, device="cuda"),
                    torch.empty(2, 2, 100, dtype=torch.int32, device="cuda"),
                    torch.empty(2, 2, wl.context - 100, dtype=torch.int32, device="cuda"),
                    torch.empty(2, 2, wl.context - 100, device="cuda"), ws)
    with pytest.raises(B.CaoteError) as e:
        B.caote_evict_joint(*args())
    assert e.value.status == B.EUNSUPPORTED


@pytest.mark.parametrize("factor", [8.0, 1.0 / 64], ids=["sharp", "flat"])
@pytest.mark.parametrize("kw", [
    dict(window=8),                                                   # matrix-core sweeps
    dict(window=1, context=1500, budget=1400),                        # few rows, matrix cores
    dict(window=2, head_dim=64, dtype="f32"),                         # few rows, vector ALUs
    dict(window=8, head_dim=64, dtype="f32"),                         # two-sweep vector path
    dict(window=16, base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=16),
], ids=["mfma", "few-mfma", "few-valu", "generic", "snapkv"])
def test_sharp_and_flat_softmax(B, oracle, kw, factor):
    """Logits scaled by 8 (attention collapses onto a few keys, exponents far apart) and by
    1/64 (nearly uniform attention): the queries carry the factor, a power of two, so the
    stored values stay exact."""
    wl = small(**kw)
    cache = synth.make_cache(wl, base_init="random")
    cache.q.mul_(factor)
    full_check(B, oracle, cache, wl.budget)


@pytest.mark.parametrize("kw", [
    dict(window=1, context=2176, budget=2100),                          # register-resident value rows, full
    dict(window=1, context=2177, budget=2000),                          # one row more: the streaming value kernels
    dict(window=2, context=4352, budget=4000, batch=1),
    dict(window=1, context=5000, budget=4999, batch=1),
    dict(window=1, context=8704, budget=8000, batch=1, base=synth.BASE_NONE),
    dict(window=1, context=8705, budget=8000, batch=1),
    dict(window=4, context=3000, budget=2500, batch=1),                 # 16 query rows: two vector-ALU key sweeps
    dict(window=4, context=3000, budget=2500, batch=1, base=synth.BASE_SNAPKV, pool_kernel=9, n_protect_tail=4),
    dict(window=1, context=2500, budget=2400, base=synth.BASE_SNAPKV, pool_kernel=301, n_protect_head=3),
], ids=["resident-full", "streaming-2177", "streaming-4352", "streaming-5000", "streaming-8704", "streaming-8705",
        "generic-h2o", "generic-snapkv", "wide-pool"])
@pytest.mark.parametrize("variant", [0, 1], ids=["exact", "fast"])
def test_value_side_column_splits(B, oracle, kw, variant):
    """Short caches keep a head's value rows in registers (a head cut by columns into two
    workgroups), longer ones stream V twice: both sides of the limit, both variants, every
    base mode."""
    wl = small(**kw)
    lens = None
    if wl.batch > 1:
        lens = np.array([wl.context, wl.context - 129], dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    full_check(B, oracle, cache, wl.budget, mode=1 if wl.budget == wl.context - 1 else 0, variant=variant)


def test_fastcaote_variant(B, oracle):
    wl = small(base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=8)
    full_check(B, oracle, synth.make_cache(wl), wl.budget, variant=1)
    wl = small()
    full_check(B, oracle, synth.make_cache(wl, base_init="random"), wl.budget, variant=1)


@pytest.mark.parametrize("lens,budget", [
    ([700, 8], 200),        # second sequence: only the window, shorter than the budget
    ([300, 0], 200),        # an empty sequence is skipped
    ([201, 200], 200),      # evict exactly one / evict none
    ([700, 699], 1),        # budget of one
    ([700, 700], 699),      # budget N-1
    ([512, 256], 256),      # tile-aligned lengths
    ([513, 257], 250),
])
def test_length_and_budget_edges(B, oracle, lens, budget):
    wl = small(budget=budget)
    lens = np.array(lens, dtype=np.int32)
    host_lens = np.maximum(lens, wl.window)       # the generator needs N >= W
    cache = synth.make_cache(wl, seq_lens=host_lens, base_init="random")
    cache.seq_lens = torch.as_tensor(lens)
    if (lens < wl.window).any():
        # a sequence shorter than the window breaks the caller's contract for
        # window_in_cache; run it with every key visible instead
        cache = synth.Cache(wl.with_(window_in_cache=0), cache.q, cache.K, cache.V, cache.base,
                            cache.seq_lens)
    full_check(B, oracle, cache, budget)


@pytest.mark.parametrize("lens,budget", [
    ([700, 1], 200),        # a cache of one token
    ([300, 0], 200),        # an empty sequence is skipped
    ([201, 200], 200),      # evict exactly one / evict none
    ([700, 2], 1),          # budget of one
    ([700, 700], 699),      # evict one everywhere
    ([512, 511], 100),
])
@pytest.mark.parametrize("mode", [0, 1], ids=["stable", "swap-last"])
def test_length_and_budget_edges_one_query_row(B, oracle, lens, budget, mode):
    """The same edges on the generation path (one query position per head: few-row key sweep,
    register-resident value kernel, evict-one fast path in the selection)."""
    wl = small(budget=budget, window=1)
    lens = np.array(lens, dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=np.maximum(lens, 1), base_init="random")
    cache.seq_lens = torch.as_tensor(lens)
    full_check(B, oracle, cache, budget, mode=mode)


def test_all_rows_protected_and_single_scored_token_one_query_row(B, oracle):
    for tail in (34, 33, 0):
        wl = small(context=64, budget=40, window=1, n_protect_head=30, n_protect_tail=tail, batch=1)
        full_check(B, oracle, synth.make_cache(wl), wl.budget)
    wl = small(context=64, budget=63, window=1, n_protect_head=0, n_protect_tail=64, batch=1)
    full_check(B, oracle, synth.make_cache(wl), wl.budget, mode=1)     # evict one, every row protected


def test_all_rows_protected_and_single_scored_token(B, oracle):
    wl = small(context=64, budget=40, n_protect_head=30, n_protect_tail=34, batch=1)
    full_check(B, oracle, synth.make_cache(wl), wl.budget)
    wl = small(context=64, budget=40, n_protect_head=30, n_protect_tail=33, batch=1)
    full_check(B, oracle, synth.make_cache(wl), wl.budget)


@pytest.mark.parametrize("window", [8, 1], ids=["window8", "one-query-row"])
def test_strided_views(B, oracle, window):
    """K and V as slices of a larger allocation (row stride > head_dim), on the prefill and on
    the generation path."""
    wl = small(batch=1, window=window)
    cache = synth.make_cache(wl)
    padK = torch.zeros(1, 2, wl.context, 256, dtype=cache.K.dtype)
    padV = torch.zeros(1, 2, wl.context, 256, dtype=cache.K.dtype)
    padK[..., :128], padV[..., 128:] = cache.K, cache.V
    dev = H.to_device(cache)
    dK, dV = padK.cuda()[..., :128], padV.cuda()[..., 128:]
    assert dK.stride(2) == 256
    L = B.make_layout(dev.q, dK, dV, base=wl.base, softmax_scale=wl.softmax_scale)
    ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
    s1 = torch.empty(1, 2, wl.context, device="cuda")
    s2 = torch.empty_like(s1)
    b1, b2 = dev.base.clone(), dev.base.clone()
    B.caote_score(dev.q, dK, dV, b1, L, s1, ws)
    L2 = B.layout_for(wl, dev)
    B.caote_score(dev.q, dev.K, dev.V, b2, L2, s2, ws)
    torch.cuda.synchronize()
    assert torch.equal(s1, s2) and torch.equal(b1, b2)


def test_deterministic_bits(B):
    wl = synth.llama3_8b_4k()
    cache = synth.make_cache(wl)
    r1 = run_path(B, cache, wl.budget, fused=True)
    r2 = run_path(B, cache, wl.budget, fused=True)
    assert np.array_equal(r1["scores"], r2["scores"]) and np.array_equal(r1["kept"], r2["kept"])
    assert torch.equal(r1["K_after"].view(torch.int16), r2["K_after"].view(torch.int16))


# ---- select and compact on their own ------------------------------------------------------

def _layout_only(B, batch, hkv, cap, d=128, dtype=torch.bfloat16):
    q = torch.empty(batch, hkv, 1, d, dtype=dtype, device="cuda")
    K = torch.empty(batch, hkv, cap, d, dtype=dtype, device="cuda")
    return B.make_layout(q, K, K, base=B.BASE_NONE, softmax_scale=1.0), K


@pytest.mark.parametrize("cap,budget", [(1, 1), (63, 10), (1000, 999), (2049, 2048), (4096, 100), (4096, 4095),
                                        (4097, 2048), (4097, 4096), (5000, 1234), (8192, 8191), (8193, 8192), (16384, 16383), (12345, 6000), (16384, 3), (16385, 8000), (20000, 100), (32768, 2048),
                                        (32769, 2048), (40000, 2048), (131072, 4096),
                                        (300000, 100000)])
def test_select_exact_with_ties_and_infinities(B, oracle, cap, budget):
    rng = np.random.default_rng(cap)
    sc = rng.standard_normal((2, 3, cap)).astype(np.float32)
    sc[0, 0] = np.round(sc[0, 0], 1)                   # many ties (incl. +-0)
    sc[0, 1] = np.abs(sc[0, 1]) * 1e-30                # tiny positives, same exponent range
    sc[0, 2, :] = 1.5                                  # all equal
    sc[1, 0, rng.integers(0, cap, size=max(1, cap // 50))] = np.inf
    sc[1, 1, rng.integers(0, cap, size=max(1, cap // 3))] = 0.0
    sc[1, 2] = -np.abs(sc[1, 2])                       # negatives sort correctly too
    L, _ = _layout_only(B, 2, 3, cap)
    ws = torch.empty(B.caote_workspace_bytes(L, budget), dtype=torch.uint8, device="cuda")
    kept = torch.full((2, 3, budget), -7, dtype=torch.int32, device="cuda")
    B.caote_select(torch.from_numpy(sc).cuda(), L, budget, kept, ws)
    torch.cuda.synchronize()
    kept = kept.cpu().numpy()
    ref = oracle.select_batched(sc.astype(np.float64), None, budget)
    assert np.array_equal(kept, ref)


@pytest.mark.parametrize("pattern", ["identity", "tail", "every_other", "head_then_tail", "shift_one"])
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64), (torch.bfloat16, 64)])
@pytest.mark.parametrize("cmode", ["stable", "fill"])
def test_compact_hazard_patterns(B, oracle, pattern, dtype, d, cmode):
    cap, budget = 3000, 1400
    idx = {
        "identity": np.arange(budget),
        "tail": np.arange(cap - budget, cap),
        "every_other": np.arange(0, 2 * budget, 2),
        "head_then_tail": np.concatenate([np.arange(700), np.arange(cap - 700, cap)]),
        "shift_one": np.arange(1, budget + 1),
    }[pattern].astype(np.int32)
    L, _ = _layout_only(B, 1, 2, cap, d, dtype)
    g = torch.Generator().manual_seed(5)
    K = torch.randn(1, 2, cap, d, generator=g).to(dtype)
    V = torch.randn(1, 2, cap, d, generator=g).to(dtype)
    base = torch.rand(1, 2, cap, generator=g)
    kept = torch.from_numpy(np.tile(idx, (1, 2, 1)))
    dK, dV, db = K.cuda(), V.cuda(), base.cuda()
    L = B.make_layout(torch.empty(1, 2, 1, d, dtype=dtype, device="cuda"), dK, dV, base=B.BASE_NONE,
                      softmax_scale=1.0)
    ws = torch.empty(B.caote_workspace_bytes(L, budget), dtype=torch.uint8, device="cuda")
    B.caote_compact(dK, dV, db, kept.cuda(), L, budget, B.COMPACT_FILL if cmode == "fill" else B.COMPACT_STABLE, ws)
    torch.cuda.synchronize()
    cache = synth.Cache(None, None, K, V, base, None)
    H.check_compaction(oracle, K, V, base, dK.cpu(), dV.cpu(), db.cpu(), kept.numpy(), cache, budget, cmode)
    if cmode == "fill":          # rows at and beyond the new length are sources only: untouched
        assert torch.equal(dK.cpu()[:, :, budget:], K[:, :, budget:]) and torch.equal(dV.cpu()[:, :, budget:], V[:, :, budget:])


@pytest.mark.parametrize("kw,budget", [
    (dict(), 200),                                                      # H2O accumulator moves along
    (dict(base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=8), 650),    # few evictions
    (dict(window=64, context=5000), 1),                                 # budget 1
    (dict(window=64, context=5000, base=synth.BASE_SNAPKV, pool_kernel=7, n_protect_tail=64), 2048),
    (dict(window=1, n_q_heads=2, n_kv_heads=2, context=2049), 2048),    # evict one: the swap
    (dict(dtype="f32", head_dim=64), 300),
    (dict(context=20000, window=32), 16384),                            # the largest budget the mode takes
], ids=lambda x: "-".join(f"{k}={v}" for k, v in x.items()) if isinstance(x, dict) else str(x))
def test_fill_compaction_mode(B, oracle, kw, budget):
    """CAOTE_COMPACT_FILL through all three entry points (score/select/compact and the fused call):
    kept rows below the new length stay, the others fill the freed positions (ragged batch)."""
    wl = small(**kw)
    lens = np.array([wl.context, max(wl.window + 1, wl.context // 3)], dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    full_check(B, oracle, cache, budget, mode=2)


def test_fill_compaction_rejects_larger_budgets(B):
    wl = small(context=40000, window=32, budget=B.FILL_MAX_BUDGET + 1)
    c = synth.make_cache(wl)
    q, K, V = c.q.cuda(), c.K.cuda(), c.V.cuda()
    L = B.make_layout(q, K, V, base=wl.base, softmax_scale=wl.softmax_scale, window_in_cache=wl.window_in_cache)
    ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
    kept = torch.zeros(*K.shape[:2], wl.budget, dtype=torch.int32, device="cuda")
    with pytest.raises(B.CaoteError):
        B.caote_compact(K, V, None, kept, L, wl.budget, B.COMPACT_FILL, ws)


@pytest.mark.parametrize("cap", [2, 257, 5000, 20000])
def test_swap_last_finds_the_hole(B, oracle, cap):
    """caote_compact in swap-last mode on evict-one kept lists: the hole at the first rank, inside
    and at the ends of the search segments, at the last kept rank, and the last row itself evicted."""
    budget, d, dtype = cap - 1, 128, torch.bfloat16
    seg = (budget + 255) // 256
    holes = sorted({0, min(seg - 1, cap - 1), min(seg, cap - 1), cap // 2, max(cap - 2, 0), cap - 1})
    g = torch.Generator().manual_seed(cap)
    K = torch.randn(len(holes), 1, cap, d, generator=g).to(dtype)
    V = torch.randn(len(holes), 1, cap, d, generator=g).to(dtype)
    base = torch.rand(len(holes), 1, cap, generator=g)
    kept = np.stack([np.delete(np.arange(cap, dtype=np.int32), h) for h in holes])[:, None, :]
    dK, dV, db = K.cuda(), V.cuda(), base.cuda()
    L = B.make_layout(torch.empty(len(holes), 1, 1, d, dtype=dtype, device="cuda"), dK, dV, base=B.BASE_NONE,
                      softmax_scale=1.0)
    ws = torch.empty(B.caote_workspace_bytes(L, budget), dtype=torch.uint8, device="cuda")
    B.caote_compact(dK, dV, db, torch.from_numpy(kept).cuda(), L, budget, B.COMPACT_SWAP_LAST, ws)
    torch.cuda.synchronize()
    cache = synth.Cache(None, None, K, V, base, None)
    H.check_compaction(oracle, K, V, base, dK.cpu(), dV.cpu(), db.cpu(), kept, cache, budget, "swap_last")


def test_hip_graph_replays_match_eager(B):
    """The calls neither allocate nor synchronise, so they can be captured; every replay,
    with eager work and synchronisation in between, must give the eager bits."""
    wl = synth.llama3_8b_4k()
    cache = synth.make_cache(wl, base_init="random")
    dev = H.to_device(cache)
    L = B.layout_for(wl, dev)
    ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
    shape = dev.K.shape[:3]
    base0 = dev.base.clone()

    def run(scores, kept, base, stream=None):
        B.caote_score(dev.q, dev.K, dev.V, base, L, scores, ws, stream)
        B.caote_select(scores, L, wl.budget, kept, ws, stream)

    e_scores, e_kept, e_base = torch.empty(shape, device="cuda"), \
        torch.empty((*shape[:2], wl.budget), dtype=torch.int32, device="cuda"), base0.clone()
    run(e_scores, e_kept, e_base)
    torch.cuda.synchronize()

    g_scores, g_kept, g_base = torch.zeros_like(e_scores), torch.zeros_like(e_kept), base0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run(g_scores, g_kept, g_base, side)          # warm up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(g_scores, g_kept, g_base, side)
    torch.cuda.synchronize()
    for rep in range(4):
        g_base.copy_(base0)                          # eager work between the replays
        g_scores.zero_()
        g_kept.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_scores, e_scores), f"replay {rep}: scores differ from the eager call"
        assert torch.equal(g_kept, e_kept), f"replay {rep}: kept indices differ"
        assert torch.equal(g_base, e_base), f"replay {rep}: accumulator differs"


def test_hip_graph_replays_of_joint_eviction_match_eager(B):
    """caote_evict_joint enqueues one kernel per evicted token, with buffers that alternate
    between steps; captured once and replayed from restored inputs it must give the eager bits."""
    wl = small(context=600, window=8)
    budget = 560
    cache = synth.make_cache(wl, base_init="random")
    dev = H.to_device(cache)
    L = B.layout_for(wl, dev)
    ws = torch.empty(B.caote_workspace_bytes(L, budget), dtype=torch.uint8, device="cuda")
    Bn, Hkv, cap = dev.K.shape[:3]
    K0, V0, base0 = dev.K.clone(), dev.V.clone(), dev.base.clone()

    def outputs():
        return (torch.zeros(Bn, Hkv, cap, device="cuda"),
                torch.zeros(Bn, Hkv, budget, dtype=torch.int32, device="cuda"),
                torch.zeros(Bn, Hkv, cap - budget, dtype=torch.int32, device="cuda"),
                torch.zeros(Bn, Hkv, cap - budget, device="cuda"))

    def run(out, stream=None):
        B.caote_evict_joint(dev.q, dev.K, dev.V, dev.base, L, budget, 0, *out, ws, stream)

    eager = outputs()
    run(eager)
    torch.cuda.synchronize()
    eK, eV, eb = dev.K.clone(), dev.V.clone(), dev.base.clone()

    def restore():
        dev.K.copy_(K0)
        dev.V.copy_(V0)
        dev.base.copy_(base0)

    got = outputs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        restore()
        run(got, side)
        side.synchronize()
        restore()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(got, side)
    torch.cuda.synchronize()
    for rep in range(3):
        restore()
        for t in got:
            t.zero_()
        ws.random_(0, 255)                           # nothing may depend on what the workspace held
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("scores", "kept", "evicted", "joint_error"), got, eager):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager call"
        n = budget
        assert torch.equal(dev.K[:, :, :n], eK[:, :, :n]) and torch.equal(dev.V[:, :, :n], eV[:, :, :n])
        assert torch.equal(dev.base[:, :, :n], eb[:, :, :n])


def test_truncated_calls_are_prefixes_of_the_fused_call(B):
    """The measurement aid behind the benchmark's per-kernel times: cut after k kernels it enqueues
    exactly the first k of the fused call's kernels, and uncut it is the fused call, bit for bit."""
    for wl in (synth.llama3_8b_4k(), synth.decode_step(batch=2),
               synth.llama3_8b_32k().with_(context=20000, budget=1500)):
        cache = synth.make_cache(wl, base_init="random")
        mode = 1 if wl.budget == wl.context - 1 else 0
        ref = run_path(B, cache, wl.budget, mode, fused=True)
        dev = H.to_device(cache)
        L = B.layout_for(wl, dev)
        ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
        scores = torch.full(dev.K.shape[:3], float("nan"), device="cuda")
        kept = torch.full((*dev.K.shape[:2], wl.budget), -7, dtype=torch.int32, device="cuda")
        base = dev.base if wl.base == synth.BASE_H2O else None
        names = B.caote_evict_prefix(dev.q, dev.K, dev.V, base, L, wl.budget, mode, scores, kept, ws, -1)
        torch.cuda.synchronize()
        assert 3 <= len(names) <= B.MAX_PHASES and all(names)
        assert np.array_equal(scores.cpu().numpy(), ref["scores"], equal_nan=True)
        assert np.array_equal(kept.cpu().numpy(), ref["kept"])
        n = wl.budget
        assert torch.equal(dev.K.cpu()[:, :, :n].view(torch.int16), ref["K_after"][:, :, :n].view(torch.int16))
        dev2 = H.to_device(cache)
        base2 = dev2.base if wl.base == synth.BASE_H2O else None
        for k in range(len(names) + 2):
            got = B.caote_evict_prefix(dev2.q, dev2.K, dev2.V, base2, L, wl.budget, mode, scores, kept, ws, k)
            assert got == names[:k]
        torch.cuda.synchronize()


def test_read_stream_probe_runs_and_writes_nothing(B):
    """The measurement aid only reads: ragged sizes, the sink keeps its value."""
    buf = torch.arange(0, (1 << 20) + 48, dtype=torch.uint8, device="cuda")
    sink = torch.full((1,), 1234, dtype=torch.int32, device="cuda")
    for nbytes in (16, 4096, 32768 + 16, 1 << 20, (1 << 20) + 48):
        B.caote_read_stream(buf, nbytes, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 1234
    with pytest.raises(B.CaoteError):
        B.caote_read_stream(buf, 24, sink)
    with pytest.raises(B.CaoteError):
        B.caote_read_stream(buf.data_ptr() + 8, 16, sink)


def test_issue_probe_runs_every_variant(B):
    """The measurement aid behind the benchmark's arithmetic floor: every variant launches and ends."""
    out = torch.empty(B.ISSUE_PROBE_OUT_BYTES, dtype=torch.uint8, device="cuda")
    for v in range(len(B.ISSUE_PROBE_VARIANTS)):
        B.caote_issue_probe(v, 8, out)
    torch.cuda.synchronize()
    with pytest.raises(B.CaoteError):
        B.caote_issue_probe(len(B.ISSUE_PROBE_VARIANTS), 8, out)


def test_calls_in_flight_on_separate_streams_match_serial(B):
    """The library keeps no state of its own: calls on different caches, each with its own
    workspace and stream, may overlap and must give the bits of the same calls run alone."""
    wl = synth.llama3_8b_4k()
    caches = [synth.make_cache(wl.with_(seed=wl.seed + 100 * i), base_init="random") for i in range(3)]

    def run(devs, streams):
        outs = []
        for dev, st in zip(devs, streams):
            L = B.layout_for(wl, dev)
            ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
            Bn, Hkv, cap = dev.K.shape[:3]
            scores = torch.zeros(Bn, Hkv, cap, device="cuda")
            kept = torch.zeros(Bn, Hkv, wl.budget, dtype=torch.int32, device="cuda")
            outs.append((scores, kept, ws, L))
        torch.cuda.synchronize()
        for dev, st, (scores, kept, ws, L) in zip(devs, streams, outs):   # enqueued back to back
            B.caote_evict(dev.q, dev.K, dev.V, dev.base, L, wl.budget, 0, scores, kept, ws, st)
        torch.cuda.synchronize()
        return [(s.cpu(), k.cpu(), d.K.cpu(), d.V.cpu(), d.base.cpu()) for (s, k, _, _), d in zip(outs, devs)]

    serial = run([H.to_device(c) for c in caches], [None] * 3)
    streams = [torch.cuda.Stream() for _ in caches]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    overlapped = run([H.to_device(c) for c in caches], streams)
    for i, (a, b) in enumerate(zip(serial, overlapped)):
        for name, x, y in zip(("scores", "kept", "K", "V", "base"), a, b):
            n = wl.budget if name in ("K", "V", "base") else x.shape[2]
            assert torch.equal(x[:, :, :n], y[:, :, :n]), f"call {i}: {name} differs when the calls overlap"
