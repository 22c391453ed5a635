#!/usr/bin/env python3
"""Benchmark of the Keyformer decode hot path on one MI355X.

A "step" is one generation step of the whole path over every (layer, batch,
head) unit of a workload: append + logits + attention + score accumulation
(one fused kernel) followed by top-(k-w) selection + window retention +
in-place KV compaction, issued as ONE library call (kf_decode_select_step,
ordered layout).  The state the timed steps start from is produced by the path
itself: kf_prefill_score over the synthetic prompt, then the first eviction
from n to k tokens.

With no --config the four bf16 workloads are timed one after the other in this
process.  The line's headline fields (`value`, `config`, `roofline`,
`cpu_baseline`, ...) belong to `batched`, the largest workload that fits one
GPU; `per_config` carries the same fields for the other three.

Protocol per workload: W warm-up steps, then the timed region of exactly K
steps (bracketed by torch.cuda.synchronize()) is run R times in a row, the
generation simply continuing; `value` is K over the MEDIAN region, `repeats_ms`
lists all of them.  Nothing but the step calls runs inside a timed region.
Per-kernel durations are taken afterwards, in a pass of their own, with HIP
events on the launch stream around the two calls of the same step
(kf_decode_step, kf_select_evict: the kernels the fused call launches):
`roofline` is the decode kernel's algorithmic HBM bytes per launch over its
mean duration there, against the 8 TB/s peak; `select_compact` likewise for
the selection/compaction kernel on the bytes it really moved.  `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same state.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak
HEADLINE = "batched"
ALL_CONFIGS = ["batched", "gptj", "mpt", "long"]   # headline first: a failure later cannot lose it


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--repeats", type=int, default=5, help="timed regions of --steps steps each; the median is reported")
    ap.add_argument("--config", default=None,
                    help="time one workload of kf_workloads.CONFIGS only (it then takes the headline fields)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU work budget of the oracle leg on the headline workload (a third of it on the others)")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip everything after the timed regions and the per-kernel event pass (used when "
                         "profiling, so that per-kernel statistics cover the headline step only)")
    ap.add_argument("--all-variants", action="store_true",
                    help="also time the graph replays, the other logit adjustments, the shared score function "
                         "and grouped-query decode on the headline workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of a known size (1 GiB, 10 times): the reference the "
                         "FETCH_SIZE / WRITE_SIZE counters are scaled by")
    return ap.parse_args()


def decode_bytes(wl, m):
    """Algorithmic HBM bytes of one fused decode launch: K and V rows read once,
    score read + written, pos read, plus the per-unit q/k_new/v_new/out vectors."""
    per_unit = m * (2 * wl.d * wl.elem_bytes + 12) + 3 * wl.d * wl.elem_bytes + 4 * wl.d
    return wl.units * per_unit


def copy_ceiling(torch):
    """What a plain device-to-device copy reaches on this machine (bytes read + written)."""
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(5):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    gbs = 5 * 2 * src.numel() * 4 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    return {"value": round(gbs, 1), "unit": "GB/s", "kind": "device copy of 1 GiB, bytes read + written"}


def bench_config(wl, args, headline):
    import numpy as np
    import torch

    import kf_workloads as kw
    import paper_2403_09054_amd as kf

    K_steps, W_steps, R = args.steps, args.warmup, max(1, args.repeats)
    dt = kf.F32 if wl.dtype == "f32" else kf.BF16
    seeds = torch.from_numpy(kw.noise_seeds(wl).view(np.int64).copy()).cuda()
    slopes_np = kw.alibi_slopes(wl)
    slopes = None if slopes_np is None else torch.from_numpy(slopes_np).cuda()
    noise = kf.NOISE_GUMBEL

    # ---------------- state: prompt scoring + first eviction, a few layers per call ----------------
    cache = kf.Cache.allocate(wl.L, wl.B, wl.H, wl.d, wl.k + 1, dt)
    ws = kf.new_workspace(cache)
    Ls = kw.staging_layers(wl)
    stage = kf.Cache.allocate(Ls, wl.B, wl.H, wl.d, wl.n, dt)
    Qs = torch.empty((Ls, wl.B, wl.H, wl.n, wl.d), dtype=wl.torch_dtype, device="cuda")
    ws_stage = kf.new_workspace(stage, wl.n)
    tau0 = kf.kf_tau(0, wl.T, wl.tau_init, wl.tau_end)
    prefill_ms = 0.0
    first_select_ms = 0.0
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for l0 in range(0, wl.L, Ls):
        nl = min(Ls, wl.L - l0)
        for i in range(nl):
            Q, K, V = kw.prompt_layer(wl, l0 + i, device="cuda")
            Qs[i].copy_(Q)
            stage.K[i].copy_(K)
            stage.V[i].copy_(V)
            del Q, K, V
        sub = stage if nl == Ls else kf.Cache(K=stage.K[:nl], V=stage.V[:nl], score=stage.score[:nl],
                                              pos=stage.pos[:nl], len=stage.len[:nl], L=nl, B=wl.B, H=wl.H,
                                              d=wl.d, cap=wl.n, dtype=dt)
        sub.layer0 = l0   # the staging cache plays layers l0 .. l0+nl-1 (noise key)
        ev[0].record()
        kf.kf_prefill_score(sub, Qs[:nl], wl.n, tau0, wl.scale, noise, seeds, slopes, ws_stage)
        ev[1].record()
        # first eviction n -> k, gathered straight into the generation cache (cap = k+1)
        kf.kf_select_evict_into(sub, cache, l0, wl.k, wl.w, None, ws_stage)
        ev[2].record()
        torch.cuda.synchronize()
        prefill_ms += ev[0].elapsed_time(ev[1])
        first_select_ms += ev[1].elapsed_time(ev[2])
    del Qs, stage, ws_stage, sub
    torch.cuda.empty_cache()
    assert int(cache.len.min()) == wl.k and int(cache.len.max()) == wl.k

    # ---------------- decode inputs, resident in HBM ----------------
    n_distinct = min(W_steps + K_steps * R, 32)
    steps_in = [kw.decode_inputs(wl, t + 1, device="cuda") for t in range(n_distinct)]
    out = torch.zeros((wl.L, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
    m = wl.k + 1
    clock = {"t": 0}   # decode steps taken so far: the generation continues through every phase below

    def tau_of(t):
        return kf.kf_tau(min(t, wl.T), wl.T, wl.tau_init, wl.tau_end)

    def fused_step(layout=kf.LAYOUT_ORDERED):
        clock["t"] += 1
        t = clock["t"]
        q, kn, vn = steps_in[(t - 1) % n_distinct]
        kf.kf_decode_select_step(cache, q, kn, vn, wl.n + t - 1, m, tau_of(t), wl.scale, noise, seeds, slopes, out,
                                 k=wl.k, w=wl.w, layout=layout, workspace=ws)

    def two_call_step(e=None, kept=None, mode=noise):
        clock["t"] += 1
        t = clock["t"]
        q, kn, vn = steps_in[(t - 1) % n_distinct]
        if e is not None:
            e[0].record()
        kf.kf_decode_step(cache, q, kn, vn, wl.n + t - 1, m, tau_of(t), wl.scale, mode, seeds, slopes, out, ws)
        if e is not None:
            e[1].record()
        kf.kf_select_evict(cache, wl.k, wl.w, kept, ws)
        if e is not None:
            e[2].record()

    def check_state():
        assert int(ws[:4].view(torch.int32)[0].item()) == 0, "a kernel skipped units"
        assert int(cache.len.min()) == wl.k and int(cache.len.max()) == wl.k

    def timed(step_fn, n_steps):
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(n_steps):
            step_fn()
        torch.cuda.synchronize()
        return time.perf_counter() - c0

    for _ in range(W_steps):
        fused_step()
    torch.cuda.synchronize()

    # snapshot for the CPU baseline (layer 0), taken before the timed regions
    snap, snap_t = None, clock["t"]
    if not args.no_cpu_baseline:
        snap = dict(K=cache.K[0:1].clone(), V=cache.V[0:1].clone(), score=cache.score[0:1].clone(),
                    pos=cache.pos[0:1].clone(), len=cache.len[0:1].clone())

    # ---------------- the timed regions: K fused steps each, nothing else inside ----------------
    regions = [timed(fused_step, K_steps) for _ in range(R)]
    check_state()
    med = statistics.median(regions)
    res = {
        "workload": "%s: L=%d B=%d H=%d d=%d n=%d k=%d w=%d T=%d %s" % (
            wl.name, wl.L, wl.B, wl.H, wl.d, wl.n, wl.k, wl.w, wl.T, wl.dtype),
        "units": wl.units,
        "value": round(K_steps / med, 2), "unit": "steps/s", "ms_per_step": round(med * 1e3 / K_steps, 4),
        "repeats_ms": [round(r * 1e3, 3) for r in regions],
        "spread": round((max(regions) - min(regions)) / med, 4),
        "step": "kf_decode_select_step, ordered layout (in-place order-preserving compaction)",
    }

    # ---------------- per-kernel pass: HIP events around the two calls of the same step ----------------
    n_ev = 16
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)]
    for _ in range(2):
        two_call_step()
    torch.cuda.synchronize()
    for e in evs:
        two_call_step(e)
    torch.cuda.synchronize()
    check_state()
    dec_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / n_ev
    sel_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / n_ev
    nbytes = decode_bytes(wl, m)
    achieved = nbytes / (dec_ms * 1e-3) / 1e9
    splits, chunk = kf.kf_decode_launch_shape(cache, m)
    roofline = {"bound": "hbm",
                "kernel": "decode_kernel" + (" + decode_merge_kernel" if splits > 1 else ""),
                "launch_shape": {"splits_per_unit": splits, "rows_per_split": chunk},
                "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": None, "traffic_source": None,
                "bytes_per_launch": nbytes, "avg_launch_us": round(dec_ms * 1e3, 2),
                "timing": "HIP events on the launch stream, %d launches after the timed regions" % n_ev}
    traffic_file = os.path.join(ROOT, "profiles", "traffic_%s.json" % wl.name)
    if os.path.exists(traffic_file):
        tj = json.load(open(traffic_file))
        roofline["traffic"] = tj.get("decode_kernel_bytes_per_launch", 0) + tj.get(
            "decode_merge_kernel_bytes_per_launch", 0)
        roofline["traffic_source"] = ("profiles/traffic_%s.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                                      "earlier run of this workload, not measured in this run)" % wl.name)
    res["roofline"] = roofline
    # bytes the in-place, order-preserving compaction really moves: every row behind the evicted
    # slot is read and written once (K and V), plus the score read of the selection
    kept = torch.zeros((wl.L, wl.B, wl.H, wl.k), dtype=torch.int32, device="cuda")
    ar = torch.arange(wl.k, device="cuda", dtype=torch.int32)
    moved, probes = 0.0, 4
    for _ in range(probes):
        two_call_step(kept=kept)
        moved += float((kept != ar).sum().item())
    del kept
    moved_rows = moved / probes
    sel_bytes = moved_rows * (2 * 2 * wl.d * wl.elem_bytes + 2 * 8) + wl.units * m * 4
    sel_gbs = sel_bytes / (sel_ms * 1e-3) / 1e9
    res["select_compact"] = {"kernel": "select_kernel", "avg_launch_us": round(sel_ms * 1e3, 2),
                             "moved_rows_per_step": round(moved_rows, 1), "bytes_per_launch": int(sel_bytes),
                             "achieved": round(sel_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(sel_gbs / HBM_PEAK_GBS, 4)}

    # prompt-phase scoring: dense causal QK^T twice (row statistics, column sums)
    prefill_flops = wl.units * 2 * (2.0 * wl.d * wl.n * (wl.n + 1) / 2)
    res["prefill_score"] = {"layers_per_call": Ls, "ms_total": round(prefill_ms, 3),
                            "tflops": round(prefill_flops / (prefill_ms * 1e-3) / 1e12, 2),
                            "logits_per_s": round(wl.units * wl.n * (wl.n + 1) / (prefill_ms * 1e-3), 0),
                            "first_select_ms_total": round(first_select_ms, 3)}

    # ---------------- variants of the same step (not the headline) ----------------
    def rate(dt_, n_steps):
        return {"steps_per_s": round(n_steps / dt_, 2), "ms_per_step": round(dt_ * 1e3 / n_steps, 4)}

    def graph_variant(layout):
        """A run of fused steps captured once in a HIP graph and replayed: no launch gaps, no host work.  The
        captured calls take the step number from device memory (kf_decode_select_step_at), so every replay
        continues the generation (q_pos and tau move on) instead of repeating the captured steps."""
        n_cap = min(n_distinct, K_steps)
        reps = max(1, K_steps // n_cap)
        step = torch.full((1,), clock["t"] + 1, dtype=torch.int32, device="cuda")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n_cap):
                q, kn, vn = steps_in[i]
                kf.kf_decode_select_step_at(cache, q, kn, vn, wl.n, wl.T, wl.tau_init, wl.tau_end, step, m, wl.scale,
                                            noise, seeds, slopes, out, k=wl.k, w=wl.w, layout=layout, workspace=ws)
        g.replay()                      # warm replay
        torch.cuda.synchronize()
        t_before = int(step.item())
        c0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        dt_ = time.perf_counter() - c0
        assert int(step.item()) == t_before + reps * n_cap
        clock["t"] = int(step.item()) - 1
        check_state()
        r = rate(dt_, reps * n_cap)
        r.update({"steps_per_graph": n_cap, "replays": reps})
        return r

    def noise_variant(mode):
        """The two-call step with another logit adjustment of the paper's ablation (same kernels)."""
        n_v = min(K_steps, 32)
        ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_v)]
        for _ in range(2):
            two_call_step(mode=mode)
        for e in ev2:
            two_call_step(e, mode=mode)
        torch.cuda.synchronize()
        dec = sum(e[0].elapsed_time(e[1]) for e in ev2) / n_v
        sel = sum(e[1].elapsed_time(e[2]) for e in ev2) / n_v
        return {"decode_us": round(dec * 1e3, 2), "select_us": round(sel * 1e3, 2),
                "decode_frac_of_peak": round(decode_bytes(wl, m) / (dec * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    def shared_variant():
        """One score function for all layers (the paper's "Shared" ablation): fused steps, ordered layout.
        All layers must hold the same tokens: layer 0's positions and scores are given to every layer."""
        cache.pos.copy_(cache.pos[0:1].expand_as(cache.pos).clone())
        cache.score.copy_(cache.score[0:1].expand_as(cache.score).clone())

        def step_fn():
            clock["t"] += 1
            t = clock["t"]
            q, kn, vn = steps_in[(t - 1) % n_distinct]
            kf.kf_decode_select_step(cache, q, kn, vn, wl.n + t - 1, m, tau_of(t), wl.scale, noise, seeds, slopes,
                                     out, k=wl.k, w=wl.w, layout=kf.LAYOUT_ORDERED, workspace=ws,
                                     score_mode=kf.SCORE_SHARED)
        for _ in range(4):
            step_fn()
        n_v = min(K_steps, 64)
        dt_ = timed(step_fn, n_v)
        check_state()
        assert bool((cache.pos[:, :, :, : wl.k] == cache.pos[0:1, :, :, : wl.k]).all()), "layers kept different tokens"
        return rate(dt_, n_v)

    def gqa_variant(G):
        """Decode call with G query heads per cached head (grouped-query attention): the workload's query
        heads on H/G cached heads, same per-unit shape, the batch raised to the largest with at most 1024
        cached heads (the workload's own batch would leave a launch of a few dozen units; a few more than
        the ~1024 workgroups the chip holds at once would time a nearly empty second round); K+V
        algorithmic bytes over the call's duration."""
        Hk = wl.H // G
        B2 = max(1, 1024 // (wl.L * Hk))
        c2 = kf.Cache.allocate(wl.L, B2, Hk, wl.d, wl.k + 1, dt, q_per_kv=G)
        c2.K.normal_()
        c2.V.normal_()
        c2.score.uniform_()
        c2.pos.copy_(torch.arange(wl.k + 1, device="cuda", dtype=torch.int32).expand_as(c2.pos))
        ws2 = kf.new_workspace(c2)
        tdt = steps_in[0][0].dtype
        q2 = torch.randn((wl.L, B2, wl.H, wl.d), device="cuda").to(tdt)
        kn2, vn2 = (torch.randn((wl.L, B2, Hk, wl.d), device="cuda").to(tdt) for _ in range(2))
        out2 = torch.zeros((wl.L, B2, wl.H, wl.d), dtype=torch.float32, device="cuda")
        seeds2 = torch.arange(B2, device="cuda", dtype=torch.int64) + 20240309
        n_v = 20
        ev2 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_v + 3)]
        for e0, e1 in ev2:              # back to back, no synchronisation in between: the chip stays busy
            c2.len.fill_(wl.k)
            e0.record()
            kf.kf_decode_step(c2, q2, kn2, vn2, wl.n + 7, m, 1.5, wl.scale, noise, seeds2, slopes, out2, ws2)
            e1.record()
        torch.cuda.synchronize()
        assert int(ws2[:4].view(torch.int32)[0].item()) == 0
        ms = sum(e0.elapsed_time(e1) for e0, e1 in ev2[3:]) / n_v
        byt = wl.L * B2 * Hk * (m * (2 * wl.d * wl.elem_bytes + 12))
        return {"batch": B2, "cached_heads": Hk, "decode_us": round(ms * 1e3, 2),
                "frac_of_peak": round(byt / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "query_head_rows_per_s": round(wl.L * B2 * wl.H * m / (ms * 1e-3), 0)}

    def one_layer_variant(layout):
        """The fused step on ONE layer's cache per call -- the shape an integration launches, a model running
        its layers one after the other: layer 0's units copied into a cache of their own, 32 calls captured
        in a HIP graph (step number in device memory) and replayed."""
        c1 = kf.Cache.allocate(1, wl.B, wl.H, wl.d, wl.k + 1, dt)
        for nm in ("K", "V", "score", "pos", "len"):
            getattr(c1, nm).copy_(getattr(cache, nm)[0:1])
        ws1 = kf.new_workspace(c1)
        out1 = torch.zeros((1, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
        ins = [tuple(t[0:1].contiguous() for t in steps_in[i % n_distinct]) for i in range(32)]
        step = torch.full((1,), clock["t"] + 1, dtype=torch.int32, device="cuda")

        def calls():
            for q, kn, vn in ins:
                kf.kf_decode_select_step_at(c1, q, kn, vn, wl.n, wl.T, wl.tau_init, wl.tau_end, step, m, wl.scale,
                                            noise, seeds, slopes, out1, k=wl.k, w=wl.w, layout=layout, workspace=ws1)
        calls()                         # eager warm-up
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            calls()
        g.replay()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(8):
            g.replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - c0) / (8 * len(ins)) * 1e6
        assert int(ws1[:4].view(torch.int32)[0].item()) == 0
        assert int(c1.len.min()) == wl.k and int(c1.len.max()) == wl.k
        splits1, chunk1 = kf.kf_decode_launch_shape(c1, m)
        byt = decode_bytes(wl, m) / wl.L
        return {"us_per_step": round(us, 2), "units": wl.B * wl.H, "splits_per_unit": splits1,
                "rows_per_split": chunk1, "GB_per_s": round(byt / us / 1e3, 1)}

    variants = None
    if not args.no_variants:
        n_v = min(K_steps, 32)
        for _ in range(2):
            two_call_step()
        variants = {"two_call_step_ordered_layout": rate(timed(two_call_step, n_v), n_v)}
        check_state()
        if args.all_variants and headline:
            variants["graph_fused_step_ordered_layout"] = graph_variant(kf.LAYOUT_ORDERED)
            # the paper's ablations of the logit adjustment (two-call step, ordered layout)
            variants["noise_none"] = noise_variant(kf.NOISE_NONE)
            variants["noise_constant"] = noise_variant(kf.NOISE_CONSTANT)
            variants["noise_gaussian"] = noise_variant(kf.NOISE_GAUSSIAN)
            if Ls >= wl.L:   # every layer was in one cache: the shared score function can be timed
                variants["shared_score_fused_step_ordered_layout"] = shared_variant()
        variants["one_layer_graph_fused_step_ordered_layout"] = one_layer_variant(kf.LAYOUT_ORDERED)
        # slot layout last: it unsorts the cache
        for _ in range(2):
            fused_step(kf.LAYOUT_SLOT)
        variants["fused_step_slot_layout"] = rate(timed(lambda: fused_step(kf.LAYOUT_SLOT), n_v), n_v)
        check_state()
        variants["one_layer_graph_fused_step_slot_layout"] = one_layer_variant(kf.LAYOUT_SLOT)
        if args.all_variants and headline:
            variants["graph_fused_step_slot_layout"] = graph_variant(kf.LAYOUT_SLOT)
            for G in (2, 4, 8):
                if wl.H % G == 0:
                    variants["grouped_query_decode_G%d" % G] = gqa_variant(G)
    res["variants"] = variants
    del cache, ws, out
    torch.cuda.empty_cache()

    # ---------------- CPU oracle on a bounded sample of the same state ----------------
    cpu = None
    if snap is not None:
        from oracle import kf_oracle as ko
        oc = ko.OracleCache(1, wl.B, wl.H, wl.d, wl.k + 1, ko.F32 if wl.dtype == "f32" else ko.BF16)
        oc.K[...] = kw.to_oracle(snap["K"])
        oc.V[...] = kw.to_oracle(snap["V"])
        oc.score[...] = kw.to_oracle(snap["score"])
        oc.pos[...] = kw.to_oracle(snap["pos"])
        oc.len[...] = kw.to_oracle(snap["len"])
        sl_units = wl.B * wl.H
        budget = args.cpu_seconds if headline else args.cpu_seconds / 3.0
        host_in = [tuple(kw.to_oracle(a[0:1]) for a in s) for s in steps_in]
        cpu_steps, cpu_time = 0, 0.0
        t = snap_t + 1
        while cpu_time < budget and cpu_steps < 1000000:   # a bounded sample: about `budget` seconds of oracle work
            q, kn, vn = host_in[(t - 1) % n_distinct]
            c0 = time.perf_counter()
            oc.decode_step(q, kn, vn, wl.n + t - 1, ko.tau(min(t, wl.T), wl.T, wl.tau_init, wl.tau_end),
                           wl.scale, ko.NOISE_GUMBEL, kw.noise_seeds(wl), slopes_np)
            oc.select_evict(wl.k, wl.w, want_idx=False)
            cpu_time += time.perf_counter() - c0
            cpu_steps += 1
            t += 1
        cpu_value = (cpu_steps / cpu_time) * (sl_units / wl.units)
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": round(cpu_value, 4), "unit": "steps/s", "cores": min(cores, sl_units), "kind": "oracle",
               "sample": "layer 0 of %d (%d of %d units), %d decode+evict steps in %.1f s, scaled by units" % (
                   wl.L, sl_units, wl.units, cpu_steps, cpu_time),
               "host_cpus": os.cpu_count()}
    res["cpu_baseline"] = cpu
    del steps_in, snap
    gc.collect()
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (units are independent: the path would shard by head, batch "
              "or layer without any exchange); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch

    import kf_workloads as kw

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": src.numel() * 4, "launches": 10}))
        return
    names = [args.config] if args.config else ALL_CONFIGS
    head_name = names[0]
    results = {}
    for name in names:
        t0 = time.perf_counter()
        print("bench.py: %s ..." % name, file=sys.stderr, flush=True)
        if name == head_name:
            results[name] = bench_config(kw.CONFIGS[name], args, True)
        else:
            try:
                results[name] = bench_config(kw.CONFIGS[name], args, False)
            except Exception as exc:   # the headline is already measured: report the failure, keep the line
                results[name] = {"workload": name, "error": "%s: %s" % (type(exc).__name__, exc)}
                torch.cuda.empty_cache()
        results[name]["bench_wall_s"] = round(time.perf_counter() - t0, 1)
        print("bench.py: %s done in %.1f s" % (name, results[name]["bench_wall_s"]), file=sys.stderr, flush=True)
    head = results[head_name]
    wl = kw.CONFIGS[head_name]
    line = {
        "metric": "decode steps/s + achieved HBM GB/s (fused attn+score+evict) at %d%% KV budget" % round(100 * wl.k / wl.n),
        "value": head["value"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": head["workload"], "units": wl.units, "noise": "gumbel", "tau": [wl.tau_init, wl.tau_end],
                   "layout": "ordered (in-place order-preserving compaction)", "step": head["step"]},
        "repeats": max(1, args.repeats), "repeats_ms": head["repeats_ms"], "spread": head["spread"],
        "roofline": head["roofline"], "select_compact": head["select_compact"], "prefill_score": head["prefill_score"],
        "variants": head["variants"], "copy_ceiling": copy_ceiling(torch), "cpu_baseline": head["cpu_baseline"],
        "per_config": [results[n] for n in names[1:]],
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
