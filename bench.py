#!/usr/bin/env python3
"""Benchmark of the CAOTE hot path on one MI355X.

A step = one fused score + select + compact call (caote_evict) over one layer's KV
cache (all KV heads) of synthetic data already resident in HBM.  Steps rotate over
several independent layer buffers so that K and V come from HBM, not from the 256 MB
Infinity Cache.  Prints ONE JSON line:

  metric/value  cached tokens scored+evicted per second per layer (all heads)
  roofline      the slowest kernel of the path: its own compulsory HBM bytes / its duration
                against the 8 TB/s peak.  A kernel's duration is the replay time of the call
                cut after that kernel minus that of the call cut before it (caote_evict_prefix,
                same graph, same rotation of buffers): kernel time, not gaps between events
  path          the whole path's algorithmic bytes / step time against the same peak
  step_time_us  median / p10 / p90 of single steps (one graph replay each between two events)
  cpu_baseline  the fp64 oracle on the host, same workload, on all cores it can use and on one
                thread (a reported baseline, not a target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def swap_last(wl):
    """Evict-one calls (generation) move one row per head: the last row drops into the hole."""
    return wl.window == 1 and wl.budget == wl.context - 1


def algorithmic_bytes(wl, n_tokens=None):
    """HBM bytes the method must move for one layer (K and V once, window queries, three
    fp32 per-token vectors, gather read + write of the kept rows, or of the one row that an
    evict-one call in swap-last mode moves)."""
    N = wl.context if n_tokens is None else n_tokens
    esz = 2 if wl.dtype == "bf16" else 4
    bh = wl.batch * wl.n_kv_heads
    kv = 2 * bh * N * wl.head_dim * esz
    q = wl.batch * wl.n_q_heads * wl.window * wl.head_dim * esz
    vec = 3 * bh * N * 4
    rows_moved = 1 if swap_last(wl) else min(wl.budget, N)
    comp = 2 * 2 * bh * rows_moved * wl.head_dim * esz
    return {"kv": kv, "q": q, "vectors": vec, "compact": comp, "total": kv + q + vec + comp}


def phase_bytes(wl, name, fused_value_sum=False):
    """Compulsory HBM bytes of one kernel of the path, given that its inputs live in HBM.
    fused_value_sum: the second key sweep also streams V once (no separate value_sum kernel)."""
    N, d, esz = wl.context, wl.head_dim, (2 if wl.dtype == "bf16" else 4)
    bh = wl.batch * wl.n_kv_heads
    R = wl.group * wl.window
    k_bytes = bh * N * d * esz
    q_bytes = wl.batch * wl.n_q_heads * wl.window * d * esz
    vec = bh * N * 4
    rows = bh * min(wl.budget, N) * d * esz
    table = {
        "key_rowstats": k_bytes + q_bytes,
        "merge_stats": bh * R * 8,
        "key_colsum": k_bytes + q_bytes + vec + ((k_bytes + vec) if fused_value_sum else 0),
        "key_sweeps": k_bytes + q_bytes + vec,          # fused: K from HBM once
        "value_sum": k_bytes + 2 * vec,
        "value_score": k_bytes + 2 * vec,
        "value_sweeps": k_bytes + 3 * vec,
        "value_side": k_bytes + 3 * vec,                 # V once, logits / mass and accumulator in, partial distances out
        "value_combine": 4 * vec,
        "value_final": bh * (d + 1) * 4 * 2,              # at least: one partial sum in, the total out
        "select": vec + bh * wl.budget * 4,
        "select_hist": vec,
        "select_span": vec,
        "select_emit": vec + bh * wl.budget * 4,
        "compact_swap": bh * 2 * 2 * d * esz,            # one row of K and of V read and written per head
        "compact_gather": 2 * 2 * rows,
        "compact_scatter": 2 * 2 * rows,
        "compact": 2 * 2 * rows,
        "evict_fused": algorithmic_bytes(wl)["total"],
    }
    return table.get(name)


# Kernel(s) behind each phase name that caote_evict_prefix reports.
PHASE_KERNELS = {
    "key_rowstats": r"k_logits_\w+<.*, 0>$", "key_colsum": r"k_logits_\w+<.*, [12]>$",
    "merge_stats": r"k_merge_stats", "value_sum": r"k_vsum", "value_final": r"k_vfinal",
    "value_score": r"k_vscore", "value_side": r"k_vside", "value_combine": r"k_vcombine", "select_hist": r"k_select_hist", "select_span": r"k_select_span",
    "select_emit": r"k_select_emit", "compact_gather": r"k_move_rows<0>", "compact_scatter": r"k_move_rows<1>",
}


def measured_traffic(workload, phase):
    """HBM-side bytes per launch of the phase's kernel from the committed counter summary
    (profiles/traffic_<workload>.json, written from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs of this script), or None if there is none."""
    import re
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    pat = PHASE_KERNELS.get(phase)
    if not pat or not os.path.exists(path):
        return None
    with open(path) as f:
        kernels = json.load(f)["kernels"]
    hits = [v for k, v in kernels.items() if re.search(pat, k)]
    if not hits:
        return None
    return sum(v["fetch_bytes"] + v["write_bytes"] for v in hits)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed steps before the timed ones; when equal to --steps they are a first replay of "
                         "the timed graph itself (its one-time upload then falls into the warm-up)")
    ap.add_argument("--workload", default="llama3-8b-32k")
    ap.add_argument("--layers", type=int, default=0,
                    help="independent layer buffers to rotate over (default 16; 32 for the decode stream: its model's depth)")
    ap.add_argument("--ragged-prefill", action="store_true",
                    help="decode workload: also time the ragged batch-16 prefill eviction (8k-32k tokens to 2048) "
                         "that sets the stream up (generates 2 GiB of cache on the host first)")
    ap.add_argument("--batch", type=int, default=0, help="sequences per call (default: the workload's own)")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--calls-in-flight", type=int, default=4,
                    help="second figure: the same steps with this many calls (different layers) in flight "
                         "on streams of their own; 1 leaves it out")
    ap.add_argument("--no-issue-probe", action="store_true")
    ap.add_argument("--layers-per-call", type=int, default=8,
                    help="layers_one_call figure: this many layers' caches as the batch of one call")
    ap.add_argument("--no-batched-layers", action="store_true",
                    help="decode workload: leave out the all-layers-as-one-call figure (under a kernel trace "
                         "its batch-512 launches would be averaged into the per-layer kernels' durations)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (each (sequence, layer, KV head) is "
              "independent, so sharding by any of them needs no exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_14051_amd import binding as B
    from paper_2504_14051_amd import synth

    B.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]()
    if args.batch > 0:
        wl = wl.with_(batch=args.batch)
    host = synth.make_cache(wl)
    decode_stream = wl.name == "llama3-8b-decode"
    use_probe = wl.dtype == "bf16" and wl.head_dim == 128 and not args.no_issue_probe
    n_layers = args.layers if args.layers > 0 else (32 if decode_stream else 16)
    mode = B.COMPACT_SWAP_LAST if swap_last(wl) else B.COMPACT_STABLE

    # Layer 0 is the generator's output; the others are the same tensors with the KV heads
    # rotated (same statistics, different addresses), so each step streams fresh HBM lines.
    G = wl.group
    layers = []
    for l in range(n_layers):
        sh = l % wl.n_kv_heads
        K = torch.roll(host.K, sh, dims=1).cuda()
        V = torch.roll(host.V, sh, dims=1).cuda()
        q = torch.roll(host.q, sh * G, dims=1).cuda()
        base = torch.roll(host.base, sh, dims=1).cuda() if wl.base == synth.BASE_H2O else None
        layers.append((q, K, V, base))
    # Block-wise prefill: every step first appends the block (here: the rows the generator put
    # last, from a buffer of their own) behind the budget of kept rows, then evicts.
    blockwise = wl.name.endswith("prefill-block")
    blocks = [(K[:, :, -wl.window:].contiguous(), V[:, :, -wl.window:].contiguous())
              for (_, K, V, _) in layers] if blockwise else None
    q0, K0, V0, _ = layers[0]
    L = B.make_layout(q0, K0, V0, base=wl.base, softmax_scale=wl.softmax_scale,
                      window_in_cache=wl.window_in_cache, pool_kernel=wl.pool_kernel,
                      n_protect_head=wl.n_protect_head, n_protect_tail=wl.n_protect_tail)
    ws = torch.empty(B.caote_workspace_bytes(L, wl.budget), dtype=torch.uint8, device="cuda")
    scores = torch.empty(wl.batch, wl.n_kv_heads, wl.context, device="cuda")
    kept = torch.empty(wl.batch, wl.n_kv_heads, wl.budget, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()

    # A plain copy of known size (256 MiB read + 256 MiB written), so that a counter run
    # of this script (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) can be scaled to bytes.
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    def append(i):
        if blockwise:
            _, K, V, base = layers[i % n_layers]
            k_new, v_new = blocks[i % n_layers]
            B.caote_append(K, V, base, k_new, v_new, L, wl.budget, wl.window, stream)

    def step(i):
        q, K, V, base = layers[i % n_layers]
        append(i)
        B.caote_evict(q, K, V, base, L, wl.budget, mode, scores, kept, ws, stream)

    # The same path when the caller's attention pass hands its softmax normalisers over
    # (layout.row_lse): the first key sweep is skipped.  The normalisers are formed here with
    # plain torch ops, once, from the untouched caches (input preparation, outside any timing).
    lse_layouts = []
    if not args.no_graph:
        scale = float(torch.tensor(wl.softmax_scale, dtype=torch.float32))
        for (q, K, V, base) in layers:
            lse = torch.empty(wl.batch, wl.n_q_heads, wl.window, dtype=torch.float32, device="cuda")
            for b in range(wl.batch):
                for hk in range(wl.n_kv_heads):
                    qg = q[b, hk * G:(hk + 1) * G].float().reshape(G * wl.window, -1)
                    for r0 in range(0, qg.shape[0], 64):      # bounded temporaries
                        sl = (qg[r0:r0 + 64] @ K[b, hk].float().T) * scale
                        if wl.window_in_cache:
                            iw = (torch.arange(r0, r0 + sl.shape[0], device="cuda") % wl.window)[:, None]
                            col = torch.arange(wl.context, device="cuda")[None, :]
                            sl = sl.masked_fill(col > wl.context - wl.window + iw, float("-inf"))
                        lse[b, hk * G:(hk + 1) * G].view(-1)[r0:r0 + sl.shape[0]] = torch.logsumexp(sl, dim=1)
            lse_layouts.append((lse, B.make_layout(
                q, K, V, base=wl.base, softmax_scale=wl.softmax_scale,
                window_in_cache=wl.window_in_cache, pool_kernel=wl.pool_kernel,
                n_protect_head=wl.n_protect_head, n_protect_tail=wl.n_protect_tail, row_lse=lse)))
        torch.cuda.synchronize()

    def step_lse(i):
        q, K, V, base = layers[i % n_layers]
        append(i)
        B.caote_evict(q, K, V, base, lse_layouts[i % n_layers][1], wl.budget, mode, scores, kept, ws, stream)

    # Greedy selection under the joint error (caote_evict_joint), where the entry point takes
    # the workload: a second figure, as for row_lse.
    # (one launch per evicted token and step of the graph: only where few tokens leave)
    joint_ok = wl.context <= B.JOINT_MAX_CAPACITY and wl.context - wl.budget <= 256 and not args.no_graph
    if joint_ok:
        n_ev = wl.context - wl.budget
        evicted = torch.empty(wl.batch, wl.n_kv_heads, n_ev, dtype=torch.int32, device="cuda")
        joint_err = torch.empty(wl.batch, wl.n_kv_heads, n_ev, device="cuda")

    def step_joint(i):
        q, K, V, base = layers[i % n_layers]
        append(i)
        B.caote_evict_joint(q, K, V, base, L, wl.budget, mode, scores, kept, evicted, joint_err, ws, stream)

    replays = []       # per timed_replay call: ms per step of the extra replays

    def timed_replay(step_fn, n_again=0):
        """K steps captured once into a HIP graph (the library neither allocates nor
        synchronises; eager launches are launch-bound: three to nine short kernels per step)."""
        nonlocal stream
        outer = stream
        side = torch.cuda.Stream()
        side.wait_stream(outer)
        with torch.cuda.stream(side):
            stream = side
            for i in range(3):
                step_fn(i)
            side.synchronize()
            g_warm, g_timed = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
            if args.warmup and args.warmup != args.steps:
                with torch.cuda.graph(g_warm, stream=side):
                    for i in range(args.warmup):
                        step_fn(i)
            with torch.cuda.graph(g_timed, stream=side):
                for i in range(args.steps):
                    step_fn(args.warmup + i)
            if args.warmup == args.steps:
                g_timed.replay()         # W = K: the warm-up steps are a first replay of the same graph
            elif args.warmup:
                g_warm.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g_timed.replay()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            # the same graph a few more times: the spread of the per-step time between replays
            again = []
            for _ in range(n_again):
                t1 = time.perf_counter()
                g_timed.replay()
                torch.cuda.synchronize()
                again.append((time.perf_counter() - t1) / args.steps * 1e3)
            replays.append(again)
        stream = outer
        return dt

    dt_lse = None
    if args.no_graph:
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    else:
        dt = timed_replay(step, n_again=4)
        dt_lse = timed_replay(step_lse)
    dt_joint = timed_replay(step_joint) if joint_ok else None

    # FastCAOTE (Sec. 3.3): the same step with o = plain mean of the scored values, and the
    # rank correlation of its scores with the exact ones on this synthetic layer (the paper
    # reports Spearman >= 0.8 per layer on a real prompt: context, not a target).
    fast = None
    if not args.no_graph:
        Lf = B.make_layout(q0, K0, V0, base=wl.base, softmax_scale=wl.softmax_scale,
                           window_in_cache=wl.window_in_cache, pool_kernel=wl.pool_kernel,
                           n_protect_head=wl.n_protect_head, n_protect_tail=wl.n_protect_tail, variant=B.FAST)

        def step_fast(i):
            q, K, V, base = layers[i % n_layers]
            append(i)
            B.caote_evict(q, K, V, base, Lf, wl.budget, mode, scores, kept, ws, stream)

        def rank(x):
            r = torch.empty_like(x)
            r[x.argsort()] = torch.arange(x.numel(), device=x.device, dtype=x.dtype)
            return r

        # scores of both variants on an untouched copy of layer 0 (input preparation, not timed)
        fq, fK, fV = host.q.cuda(), host.K.cuda(), host.V.cuda()
        fb = host.base.cuda() if wl.base == synth.BASE_H2O else None
        s_ex, s_fa = torch.empty_like(scores), torch.empty_like(scores)
        B.caote_score(fq, fK, fV, None if fb is None else fb.clone(), L, s_ex, ws, stream)
        B.caote_score(fq, fK, fV, None if fb is None else fb.clone(), Lf, s_fa, ws, stream)
        torch.cuda.synchronize()
        rho = []
        for b in range(wl.batch):
            for hk in range(wl.n_kv_heads):
                m = torch.isfinite(s_ex[b, hk]) & torch.isfinite(s_fa[b, hk])
                x, y = rank(s_ex[b, hk][m].double()), rank(s_fa[b, hk][m].double())
                x, y = x - x.mean(), y - y.mean()
                rho.append(float((x * y).sum() / (x.norm() * y.norm()).clamp_min(1e-300)))
        del fq, fK, fV, fb, s_ex, s_fa
        dt_fast = timed_replay(step_fast)
        fast = {"ms_per_step": dt_fast / args.steps * 1e3,
                "value": wl.batch * wl.context / (dt_fast / args.steps), "unit": "tokens/s",
                "spearman_vs_exact": {"min": min(rho), "mean": sum(rho) / len(rho), "max": max(rho),
                                      "n_heads": len(rho)},
                "note": "variant = CAOTE_FAST; Spearman rank correlation of FastCAOTE and CAOTE scores per "
                        "(sequence, KV head) over the scored tokens of layer 0"}

    # The same step with the hole-filling compaction (CAOTE_COMPACT_FILL: kept rows below the new
    # length stay, the others drop into the freed positions; one kernel, fewest rows moved).
    fill = None
    if not args.no_graph and mode == B.COMPACT_STABLE and wl.budget <= B.FILL_MAX_BUDGET:
        def step_fill(i):
            q, K, V, base = layers[i % n_layers]
            append(i)
            B.caote_evict(q, K, V, base, L, wl.budget, B.COMPACT_FILL, scores, kept, ws, stream)
        dt_fill = timed_replay(step_fill, n_again=2)
        fill = {"ms_per_step": dt_fill / args.steps * 1e3, "ms_per_step_replays": replays.pop(),
                "value": wl.batch * wl.context / (dt_fill / args.steps), "unit": "tokens/s",
                "note": "mode = CAOTE_COMPACT_FILL instead of CAOTE_COMPACT_STABLE: same kept set, rows not in "
                        "ascending order afterwards"}

    # Every timed step above works on a cache that earlier steps have already compacted (the
    # layer buffers rotate and are not restored).  The same call on caches that no call has
    # touched: one buffer per step, all restored from pristine copies before every replay.
    fresh = None
    if not args.no_graph and not blockwise and not decode_stream:
        layer_bytes = 2 * K0.numel() * K0.element_size()
        nf = int(max(4, min(args.steps, 48, (16 << 30) // layer_bytes)))
        nm = min(n_layers, 8)
        masters = []
        for l in range(nm):
            sh = l % wl.n_kv_heads
            masters.append((torch.roll(host.q, sh * G, dims=1).cuda(), torch.roll(host.K, sh, dims=1).cuda(),
                            torch.roll(host.V, sh, dims=1).cuda(),
                            torch.roll(host.base, sh, dims=1).cuda() if wl.base == synth.BASE_H2O else None))
        work = [tuple(None if t is None else t.clone() for t in masters[i % nm][1:]) for i in range(nf)]

        def restore():
            for i, (K, V, base) in enumerate(work):
                _, mK, mV, mb = masters[i % nm]
                K.copy_(mK); V.copy_(mV)
                if base is not None:
                    base.copy_(mb)
            torch.cuda.synchronize()

        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for i in range(2):
                K, V, base = work[i]
                B.caote_evict(masters[i % nm][0], K, V, base, L, wl.budget, mode, scores, kept, ws, side)
            side.synchronize()
            gf = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gf, stream=side):
                for i in range(nf):
                    K, V, base = work[i]
                    B.caote_evict(masters[i % nm][0], K, V, base, L, wl.budget, mode, scores, kept, ws, side)
            ts = []
            for _ in range(5):
                restore()
                t0 = time.perf_counter()
                gf.replay()
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) / nf * 1e3)
        ts.sort()
        fresh = {"ms_per_step": ts[len(ts) // 2], "min": ts[0], "max": ts[-1], "steps": nf,
                 "value": wl.batch * wl.context / (ts[len(ts) // 2] * 1e-3), "unit": "tokens/s",
                 "note": "the same call on caches no earlier call has compacted: one buffer per step, restored "
                         "from pristine copies before each of five replays (median, min, max)"}
        del work, masters, gf

    # The three calls one after the other (same kernels minus what only the fused call can
    # merge), and a plain streaming read of the same K and V buffers: the empirical ceiling.
    def step_separate(i):
        q, K, V, base = layers[i % n_layers]
        append(i)
        B.caote_score(q, K, V, base, L, scores, ws, stream)
        B.caote_select(scores, L, wl.budget, kept, ws, stream)
        B.caote_compact(K, V, base, kept, L, wl.budget, mode, ws, stream)

    sink = torch.zeros(1, dtype=torch.int32, device="cuda")

    def step_read(i):
        _, K, V, _ = layers[i % n_layers]
        B.caote_read_stream(K, K.numel() * K.element_size(), sink, stream)
        B.caote_read_stream(V, V.numel() * V.element_size(), sink, stream)

    dt_sep = dt_read = None
    if not args.no_graph:
        dt_sep = timed_replay(step_separate)
        dt_read = timed_replay(step_read)

    # Several calls in flight: consecutive steps work on different layers and do not depend on
    # each other, so they may run on streams of their own (each with its own workspace and
    # outputs); the narrow kernels of one call (merges, selection, compaction) then share the
    # chip with the wide sweeps of another.  `value` stays the one-call-at-a-time figure, the one
    # the per-kernel durations and the committed profiles belong to.
    dt_two = dt_two_lse = None
    NL = max(1, min(args.calls_in_flight, n_layers))
    if not args.no_graph and NL >= 2:
        lanes_res = [(ws, scores, kept)] + [(torch.empty_like(ws), torch.empty_like(scores), torch.empty_like(kept)) for _ in range(NL - 1)]

        def two_lanes(lo, hi, main, with_lse=False):
            sts = [main] + [torch.cuda.Stream() for _ in range(NL - 1)]
            for st in sts[1:]:
                st.wait_stream(main)
            for i in range(lo, hi):
                q, K, V, base = layers[i % n_layers]
                st = sts[i % NL]
                w, sc, kp = lanes_res[i % NL]
                if blockwise:
                    k_new, v_new = blocks[i % n_layers]
                    B.caote_append(K, V, base, k_new, v_new, L, wl.budget, wl.window, st)
                B.caote_evict(q, K, V, base, lse_layouts[i % n_layers][1] if with_lse else L, wl.budget, mode,
                              sc, kp, w, st)
            for st in sts[1:]:
                main.wait_stream(st)

        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            two_lanes(0, 4, side)
            side.synchronize()
            g_two = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_two, stream=side):
                two_lanes(args.warmup, args.warmup + args.steps, side)
            g_two.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g_two.replay()
            torch.cuda.synchronize()
            dt_two = time.perf_counter() - t0
            # ... and with the caller's row normalisers handed over as well: the configuration a
            # serving loop that owns the attention pass would run
            two_lanes(0, 4, side, with_lse=True)
            side.synchronize()
            g_two_lse = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_two_lse, stream=side):
                two_lanes(args.warmup, args.warmup + args.steps, side, with_lse=True)
            g_two_lse.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g_two_lse.replay()
            torch.cuda.synchronize()
            dt_two_lse = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = wl.batch * wl.context / (dt / args.steps)

    # The other way to have several layers in flight: ONE call over several layers' caches (the
    # batch dimension; layers allocated at a constant stride, e.g. all layers of a prompt evicted
    # together after its prefill).  --layers-per-call layers per call, from copies of the rotating buffers.
    stacked = None
    if not args.no_graph and not blockwise and not decode_stream and n_layers >= 4 and wl.batch == 1 \
            and 2 * K0.numel() * K0.element_size() * n_layers <= (24 << 30):
        LPC = max(2, min(args.layers_per_call, n_layers))
        groups = []
        for g0 in range(0, n_layers - LPC + 1, LPC):
            grp = layers[g0:g0 + LPC]
            groups.append((torch.cat([x[0] for x in grp]), torch.cat([x[1] for x in grp]),
                           torch.cat([x[2] for x in grp]),
                           torch.cat([x[3] for x in grp]) if wl.base == synth.BASE_H2O else None))
        gq, gK, gV, _ = groups[0]
        Lg = B.make_layout(gq, gK, gV, base=wl.base, softmax_scale=wl.softmax_scale,
                           window_in_cache=wl.window_in_cache, pool_kernel=wl.pool_kernel,
                           n_protect_head=wl.n_protect_head, n_protect_tail=wl.n_protect_tail)
        wsg = torch.empty(B.caote_workspace_bytes(Lg, wl.budget), dtype=torch.uint8, device="cuda")
        scg = torch.empty(LPC, wl.n_kv_heads, wl.context, device="cuda")
        kpg = torch.empty(LPC, wl.n_kv_heads, wl.budget, dtype=torch.int32, device="cuda")

        def step_stacked(i):
            q, K, V, base = groups[i % len(groups)]
            B.caote_evict(q, K, V, base, Lg, wl.budget, mode, scg, kpg, wsg, stream)
        saved_steps, saved_warm = args.steps, args.warmup
        args.steps = max(4, args.steps // LPC)
        args.warmup = args.steps
        dt_g = timed_replay(step_stacked)
        stacked = {"layers_per_call": LPC, "ms_per_layer": dt_g / args.steps / LPC * 1e3,
                   "value": LPC * wl.context / (dt_g / args.steps), "unit": "tokens/s",
                   "note": f"one caote_evict call over {LPC} layers' caches (batch = {LPC}): the narrow kernels are "
                           f"paid once per call"}
        # ... and with the caller's row normalisers
        if lse_layouts:
            g_lse = []
            for gi, g0 in enumerate(range(0, n_layers - LPC + 1, LPC)):
                lse_g = torch.cat([lse_layouts[g0 + i][0] for i in range(LPC)])
                q, K, V, _ = groups[gi]
                g_lse.append((lse_g, B.make_layout(
                    q, K, V, base=wl.base, softmax_scale=wl.softmax_scale, window_in_cache=wl.window_in_cache,
                    pool_kernel=wl.pool_kernel, n_protect_head=wl.n_protect_head,
                    n_protect_tail=wl.n_protect_tail, row_lse=lse_g)))

            def step_stacked_lse(i):
                q, K, V, base = groups[i % len(groups)]
                B.caote_evict(q, K, V, base, g_lse[i % len(groups)][1], wl.budget, mode, scg, kpg, wsg, stream)
            dt_gl = timed_replay(step_stacked_lse)
            stacked["given_row_lse"] = {"ms_per_layer": dt_gl / args.steps / LPC * 1e3,
                                        "value": LPC * wl.context / (dt_gl / args.steps), "unit": "tokens/s"}
        args.steps, args.warmup = saved_steps, saved_warm
        del groups, wsg, scg, kpg

    # Per-kernel durations: the call cut after its k-th kernel, for every k, each as a graph of
    # the same steps over the same rotation of buffers; kernel k costs T(k) - T(k-1).
    q, K, V, base = layers[0]
    names = B.caote_evict_prefix(q, K, V, base, L, wl.budget, mode, scores, kept, ws, -1, stream)
    torch.cuda.synchronize()

    # Every truncated step ends with the same tiny kernel (a 64-element fill), so that whatever
    # kernel k is, the next step's first kernel follows the same predecessor: without it the gap
    # between the last kernel of a step and the first of the next moved up to 3 us between
    # neighbouring phases.  T(0) is the graph of the fills (and appends) alone.
    sep = torch.zeros(64, device="cuda")

    def prefix_time(k):
        def step_k(i):
            q, K, V, base = layers[i % n_layers]
            append(i)
            B.caote_evict_prefix(q, K, V, base, L, wl.budget, mode, scores, kept, ws, k, stream)
            sep.zero_()
        timed_replay(step_k, n_again=4)
        return min(replays.pop()) * 1e-3 * args.steps

    phases = {}
    if args.no_graph:
        phases = {"evict_fused": ms_per_step}
    else:
        t_prev = prefix_time(0)
        for k, name in enumerate(names, start=1):
            t_k = prefix_time(k)
            phases[name] = max(t_k - t_prev, 0.0) / args.steps * 1e3
            t_prev = t_k
    dom = max(phases, key=phases.get)
    dom_bytes = phase_bytes(wl, dom, fused_value_sum="key_colsum" in phases and "value_sum" not in phases)
    dom_gbs = dom_bytes / (phases[dom] * 1e-3) / 1e9
    alg = algorithmic_bytes(wl)
    path_gbs = alg["total"] / (ms_per_step * 1e-3) / 1e9

    # Single steps: one graph per layer buffer holding one step, replayed in rotation between two
    # events each (the queue stays ahead of the GPU, so an interval is one step plus the gap to the
    # next graph launch).
    dist = None
    if not args.no_graph:
        n_dist = max(200, args.steps)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        outer = stream
        with torch.cuda.stream(side):
            stream = side
            singles = []
            for l in range(n_layers):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(l)
                singles.append(g)
            for l in range(n_layers):
                singles[l].replay()
            side.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_dist)]
            for i, (e0, e1) in enumerate(evs):
                e0.record(side)
                singles[i % n_layers].replay()
                e1.record(side)
            side.synchronize()
            us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs)
            dist = {"n": n_dist, "median": us[n_dist // 2], "p10": us[n_dist // 10], "p90": us[(9 * n_dist) // 10],
                    "note": "single-step graph replays between two events each; ms_per_step is the K-step graph"}
        stream = outer

    out = {
        "metric": "cached tokens scored+evicted/sec per layer (all heads); % of HBM peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads,
                   "head_dim": wl.head_dim, "context": wl.context, "window": wl.window,
                   "budget": wl.budget, "base": {0: "none", 1: "h2o", 2: "snapkv"}[wl.base],
                   "pool_kernel": wl.pool_kernel, "batch": wl.batch, "layer_buffers": n_layers,
                   "entry_point": "caote_append + caote_evict" if blockwise else "caote_evict",
                   "launch": "stream" if args.no_graph else "hip_graph"},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": dom_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS,
                     "traffic": measured_traffic(wl.name, dom),
                     "bytes_per_launch": dom_bytes, "ms_per_launch": phases[dom]},
        "path": {"algorithmic_bytes": alg["total"], "achieved": path_gbs, "peak": HBM_PEAK_GBS,
                 "unit": "GB/s", "frac": path_gbs / HBM_PEAK_GBS},
        "phases_ms": phases,
        "phases_note": "kernel k = replay time of the call cut after k kernels minus cut after k-1 (caote_evict_prefix)",
    }
    if dist is not None:
        out["step_time_us"] = dist
    if dt_lse is not None:
        out["given_row_lse"] = {
            "ms_per_step": dt_lse / args.steps * 1e3,
            "value": wl.batch * wl.context / (dt_lse / args.steps), "unit": "tokens/s",
            "note": "same call with layout.row_lse set (the caller's attention pass supplies the "
                    "softmax normalisers): no first key sweep"}

    if replays and replays[0]:
        out["ms_per_step_replays"] = sorted(replays[0])
    if dt_sep is not None:
        out["separate_calls"] = {"ms_per_step": dt_sep / args.steps * 1e3,
                                 "note": "caote_score, caote_select, caote_compact one after the other"}
    if dt_read is not None:
        kv_bytes = 2 * layers[0][1].numel() * layers[0][1].element_size()
        out["read_stream"] = {"achieved": kv_bytes / (dt_read / args.steps) / 1e9, "unit": "GB/s",
                              "bytes_per_step": kv_bytes,
                              "note": "plain streaming read of the same K and V buffers, same rotation: "
                                      "the rate no sweep over them can exceed on this device"}
        out["path"]["frac_of_read_stream"] = out["path"]["achieved"] / out["read_stream"]["achieved"]
        out["roofline"]["frac_of_read_stream"] = out["roofline"]["achieved"] / out["read_stream"]["achieved"]
    if dt_two is not None:
        out["calls_in_flight"] = {
            "n": NL, "ms_per_step": dt_two / args.steps * 1e3,
            "value": wl.batch * wl.context / (dt_two / args.steps), "unit": "tokens/s",
            "note": "the same K steps, step i (layer i mod layers) on stream i mod n: independent "
                    "calls overlap, total time / K"}
        if dt_two_lse is not None:
            out["calls_in_flight"]["given_row_lse"] = {
                "ms_per_step": dt_two_lse / args.steps * 1e3,
                "value": wl.batch * wl.context / (dt_two_lse / args.steps), "unit": "tokens/s",
                "note": "the same with layout.row_lse set: no first key sweep"}
    # What bounds a key sweep's arithmetic on this device: the per-tile instruction mix on
    # registers only, matrix and vector work alone and together (caote_issue_probe).
    if use_probe:
        pb = torch.empty(B.ISSUE_PROBE_OUT_BYTES, dtype=torch.uint8, device="cuda")
        iters = 2048
        ns = {}
        for v, name in enumerate(B.ISSUE_PROBE_VARIANTS):
            B.caote_issue_probe(v, 64, pb, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            B.caote_issue_probe(v, iters, pb, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            ns[name] = e0.elapsed_time(e1) * 1e6 / iters
        out["issue_probe"] = {
            "ns_per_tile_two_waves_per_simd": ns,
            "note": "256 workgroups of 8 waves, one per compute unit: time of one tile's worth of instructions per "
                    "SIMD (two waves); mfma_then_vector lies between max(mfma_16, vector_block) (the two pipes overlap "
                    "fully) and their sum (not at all): the arithmetic floor of a key sweep's tile"}
    if fast is not None:
        out["fastcaote"] = fast
    if stacked is not None:
        out["layers_one_call"] = stacked
    if fresh is not None:
        out["fresh_caches"] = fresh
    if fill is not None:
        out["fill_compaction"] = fill
    if dt_joint is not None:
        out["joint_selection"] = {
            "ms_per_step": dt_joint / args.steps * 1e3,
            "value": wl.batch * wl.context / (dt_joint / args.steps), "unit": "tokens/s",
            "evicted_per_head": wl.context - wl.budget,
            "note": "caote_evict_joint: the same step with the greedy selection under the joint "
                    "error: one kernel per evicted token, each step needs the one before"}

    # The decode stream as the workload states it: one generation step is one evict-one call per
    # layer, 32 layers with caches of their own, each layer's call after the one before (the
    # model's own order).  Two more figures: the 32 calls of a step as ONE call over 32 x 16
    # sequences (the evictions of a step do not depend on each other, so they can be deferred to the
    # end of the token's forward pass and issued together), and, on request, the ragged
    # prefill eviction that brings the 16 prompts down to the budget.
    if decode_stream and not args.no_graph:
        step_ms = ms_per_step * n_layers
        out["decode_stream"] = {
            "layers": n_layers, "sequences": wl.batch, "ms_per_generation_step": step_ms,
            "tokens_per_s": wl.batch / (step_ms * 1e-3),
            "cached_tokens_per_s": wl.batch * wl.context * n_layers / (step_ms * 1e-3),
            "note": f"{n_layers} layers with independent caches, one call per layer in the model's order, "
                    f"inside one HIP graph; a generation step appends one token to each of {wl.batch} sequences"}
    if decode_stream and not args.no_graph and not args.no_batched_layers:
        Kb = torch.cat([K for (_, K, _, _) in layers], dim=0)
        Vb = torch.cat([V for (_, _, V, _) in layers], dim=0)
        qb = torch.cat([q for (q, _, _, _) in layers], dim=0)
        bb = torch.cat([b for (_, _, _, b) in layers], dim=0)
        Lb = B.make_layout(qb, Kb, Vb, base=wl.base, softmax_scale=wl.softmax_scale,
                           window_in_cache=wl.window_in_cache, pool_kernel=wl.pool_kernel)
        wsb = torch.empty(B.caote_workspace_bytes(Lb, wl.budget), dtype=torch.uint8, device="cuda")
        sb = torch.empty(Kb.shape[:3], device="cuda")
        kb = torch.empty((*Kb.shape[:2], wl.budget), dtype=torch.int32, device="cuda")
        saved_steps, saved_warm = args.steps, args.warmup
        args.steps = max(4, min(args.steps // n_layers, 20))
        args.warmup = args.steps
        dt_b = timed_replay(lambda i: B.caote_evict(qb, Kb, Vb, bb, Lb, wl.budget, mode, sb, kb, wsb, stream))
        out["decode_stream"]["all_layers_one_call"] = {
            "ms_per_generation_step": dt_b / args.steps * 1e3, "steps": args.steps,
            "note": f"the same step as one call over {Kb.shape[0]} sequences (all layers batched: the evictions of a "
                    f"generation step deferred to the end of the forward pass)"}
        args.steps, args.warmup = saved_steps, saved_warm
        del Kb, Vb, qb, bb, wsb, sb, kb
    if decode_stream and args.ragged_prefill:
        pw = synth.llama3_8b_32k().with_(batch=wl.batch, name="llama3-8b-prefill-ragged16")
        lens = synth.prefill_lengths(pw.seed, pw.batch)
        pc = synth.make_cache(pw, seq_lens=lens)
        pq, pK, pV, pl = pc.q.cuda(), pc.K.cuda(), pc.V.cuda(), pc.seq_lens.cuda()
        pL = B.make_layout(pq, pK, pV, base=pw.base, softmax_scale=pw.softmax_scale, pool_kernel=pw.pool_kernel,
                           n_protect_tail=pw.n_protect_tail, seq_lens=pl)
        pws = torch.empty(B.caote_workspace_bytes(pL, pw.budget), dtype=torch.uint8, device="cuda")
        ps = torch.empty(pK.shape[:3], device="cuda")
        pk = torch.empty((*pK.shape[:2], pw.budget), dtype=torch.int32, device="cuda")
        saved_steps, saved_warm = args.steps, args.warmup
        args.steps, args.warmup = 10, 10
        dt_p = timed_replay(lambda i: B.caote_evict(pq, pK, pV, None, pL, pw.budget, B.COMPACT_STABLE, ps, pk, pws, stream))
        out["ragged_prefill_eviction"] = {
            "tokens": int(lens.sum()), "sequences": pw.batch, "ms_per_call": dt_p / args.steps * 1e3,
            "value": float(lens.sum()) / (dt_p / args.steps), "unit": "tokens/s",
            "note": "16 prompts of 8k-32k tokens cut to 2048 per KV head in one call with seq_lens (SnapKV base, "
                    "window 64, pool 7); the caches are not restored between the timed calls"}
        args.steps, args.warmup = saved_steps, saved_warm
        del pq, pK, pV, pws, ps, pk, pc

    if not args.skip_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import helpers as H
        oracle.build()
        n_tasks = wl.batch * wl.n_kv_heads               # the oracle runs one (sequence, KV head) per thread
        host_cores = os.cpu_count() or 1

        def oracle_layer(threads):
            t0 = time.perf_counter()
            oc, oh, _ = H.oracle_scores(oracle, host, threads=threads)
            kept_o = oracle.select_batched(oc, None, wl.budget)
            for b in range(wl.batch):
                for hk in range(wl.n_kv_heads):
                    oracle.compact_one(host.K[b, hk].view(torch.uint8).numpy(), kept_o[b, hk])
                    oracle.compact_one(host.V[b, hk].view(torch.uint8).numpy(), kept_o[b, hk])
            return time.perf_counter() - t0

        used = max(1, min(host_cores, n_tasks))
        t_all = oracle_layer(used)
        # a bounded sample of about 10-30 s of CPU work: more passes over the layer when one is short
        n_pass = 1
        if t_all * used < 10.0:
            n_pass = int(min(16, -(-10.0 // (t_all * used))))
            t_all = sum(oracle_layer(used) for _ in range(n_pass)) / n_pass
        # one thread: the whole layer if the all-cores run says it fits in about 30 s, else one
        # (sequence, KV head) of it, scaled by the number of heads (stated in `sample`)
        whole = t_all * used <= 30.0
        if whole:
            t_one = oracle_layer(1)
            one_sample = "the same layer, one thread"
        else:
            sub = synth.Cache(wl.with_(batch=1, n_q_heads=wl.group, n_kv_heads=1), host.q[:1, :wl.group],
                              host.K[:1, :1], host.V[:1, :1], host.base[:1, :1], None)
            t0 = time.perf_counter()
            H.oracle_scores(oracle, sub, threads=1)
            t_one = (time.perf_counter() - t0) * n_tasks
            one_sample = f"one (sequence, KV head) of the layer on one thread, times {n_tasks} (extrapolated)"
        out["cpu_baseline"] = {
            "value": wl.batch * wl.context / t_all, "unit": "tokens/s", "cores": used,
            "host_cores": host_cores, "kind": "oracle", "seconds": t_all,
            "sample": f"one whole layer of the same workload (all {n_tasks} (sequence, KV head) pairs, one "
                      f"thread each): score + select + compact; mean of {n_pass} pass(es)",
            "single_thread": {"value": wl.batch * wl.context / t_one, "unit": "tokens/s", "cores": 1,
                              "seconds": t_one, "sample": one_sample}}
        if decode_stream:
            out["cpu_baseline"]["generation_step_seconds_extrapolated"] = t_all * n_layers
            out["cpu_baseline"]["sample"] += (f"; a generation step is {n_layers} such layers "
                                              f"(extrapolated: {n_layers} x the measured layer)")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
