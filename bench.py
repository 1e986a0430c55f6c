#!/usr/bin/env python3
"""Benchmark of the adaptive mixed-precision KV-cache hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input, all on one stream with no host
synchronisation inside: kvq_features (logits -> H, R, V, C) -> kvq_controller (bits for the new token of every
sequence) -> for every layer: kvq_append (quantize + append the new token's K/V) -> kvq_decode_attn (one query
per sequence and head over the whole mixed-precision cache).  Inputs are resident in HBM before timing starts.

Prints ONE JSON line.  `value` is microseconds per step (lower is better); the `roofline` object is for the
dominant kernel (decode attention), timed live with events on the launch stream; `cpu_baseline` times the CPU
oracle on a bounded sample of the same workload on the host cores of this machine.
"""
from __future__ import annotations

import argparse
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
STATIC_WIDTH = {"static2": 2, "static4": 4, "static8": 8, "fp16": 16}     # caches that store every token at one width
EVENT_STEPS = 5        # timed steps whose launches are bracketed by events (spread evenly over the run)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload index 1..5 (4 = SmolLM-1.7B-shaped, the metric's config)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (profiling runs only)")
    ap.add_argument("--variant", default="mixed", choices=["mixed", "static2", "static4", "static8", "fp16", "rule", "kchannel"],
                    help="cache the timed loops run on (profiling runs: the same config stored as static 4-bit, FP16, or with "
                         "per-channel keys); anything but 'mixed' is not the metric and is named in config.variant")
    ap.add_argument("--no-compare", action="store_true", help="skip the static-4-bit, FP16, rule-policy and per-channel-key caches")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-events", action="store_true", help="do not bracket attention launches with events")
    ap.add_argument("--no-fused", action="store_true", help="skip the second timed loop that uses kvq_append_decode_attn")
    ap.add_argument("--no-graph", action="store_true", help="skip the third timed loop that replays the fused step as a HIP graph")
    ap.add_argument("--no-prefill", action="store_true", help="skip the timing of the prefill-stage kernels (bulk controller, bulk append)")
    ap.add_argument("--no-rotate", action="store_true", help="small configs: skip the loop over rotating copies of the cache")
    ap.add_argument("--trace-steps", action="store_true", help="log the mean attention time per layer of every timed step")
    ap.add_argument("--cpu-seqs", type=int, default=0, help="sequences of one layer the CPU oracle is timed on (0 = the whole batch)")
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported (sequences and kv-heads are "
              "independent units, so a larger job shards over GPUs without any exchange inside this path)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    # ---------------- comparison caches built by the same library ------------------------------------
    # Each comparison cache (static 4-bit, FP16, the rule policy's, per-channel keys) is built and timed by a child process
    # of its own (this script with --variant), one after the other, BEFORE this process touches the device: a cache is
    # then measured exactly as the headline is, as the first cache of a process that has the GPU to itself.  Device memory
    # that is released (hipFree, torch emptying its cache when a graph is captured, a process that exits) is wiped by
    # the driver in the background, and until that is done every bandwidth-bound launch on the device runs 3-5 % slow
    # (launch-bound ones do not change; measured: 58 GB released -> the next process's first 50 ms of launches), so
    # this process waits a few seconds after every child before the next measurement starts.
    compare = {}
    if not args.no_compare:
        import subprocess
        import workloads as wl0
        variants = ("static4", "fp16") + (("rule",) if wl0.CONFIGS[args.config].bits_kind == "controller" else ()) + ("kchannel",)
        for variant in variants:
            cmd = [sys.executable, os.path.abspath(__file__), "--config", str(args.config), "--variant", variant,
                   "--steps", str(args.steps), "--warmup", str(args.warmup), "--layers", str(args.layers),
                   "--no-compare", "--no-cpu", "--no-fused", "--no-prefill", "--no-rotate"]
            try:
                r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
                sub = json.loads(r.stdout.strip().splitlines()[-1]) if r.returncode == 0 and r.stdout.strip() else None
            except (subprocess.TimeoutExpired, ValueError):
                sub = None
            time.sleep(3.0)
            if sub is None:
                compare[variant] = {"skipped": "the child run of this variant failed (a cache that does not fit the device, most likely)"}
                continue
            log("[bench] %s cache (child process): %.1f us per attention launch" % (variant, sub["stages_us"]["attn_per_layer"]))
            compare[variant] = {"us_per_step": sub["value"], "attn_us_per_layer": sub["stages_us"]["attn_per_layer"],
                                "attn_GBps": sub["roofline"]["achieved"], "attn_bytes_per_layer": sub["roofline"]["bytes_per_launch"],
                                "frac_of_hbm_peak": sub["roofline"]["frac"]}

    import numpy as np
    import torch

    from paper_2604_04722_amd import binding as kvq
    import benchprobe
    import workloads as wl

    kvq.load_library()                      # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    L = args.layers or cfg.n_layers
    B, Hq, Hkv = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads
    n_steps = args.warmup + args.steps
    lens0 = wl.ragged_lengths(cfg).astype(np.int64) - 1          # prefill so that the first step reaches the context
    max_ctx = int(cfg.context + 4 * n_steps + 16)                  # up to four timed loops run on the mixed cache

    # ---------------- controller + per-token precisions of the prefill -----------------------------
    if cfg.bits_kind == "controller":
        Ws, bs = wl.calibrated_mlp(cfg)
    else:
        Ws, bs = wl.xavier_mlp(cfg)
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(dev) for w in Ws], [torch.from_numpy(b).to(dev) for b in bs])
    rule = kvq.make_rule(*wl.calibrated_rule(cfg)) if cfg.bits_kind == "controller" else None

    def prefill_bits(variant):
        T = int(lens0.max())
        if variant in STATIC_WIDTH:
            return np.full((B, T), STATIC_WIDTH[variant], np.uint8)
        if variant == "rule":
            f = torch.from_numpy(np.concatenate([wl.bulk_features(cfg, T, chunk=100 + s) for s in range(B)])).to(dev)
            b = torch.empty(B * T, dtype=torch.uint8, device=dev)
            kvq.kvq_rule_policy(f, rule, b)
            return b.view(B, T).cpu().numpy()
        if cfg.bits_kind == "uniform":
            return wl.uniform_bits(cfg, B, T)
        if cfg.bits_kind == "runs":
            return np.stack([wl.run_bits(cfg, s, T) for s in range(B)])
        # one bulk controller launch on the seeded feature draws of all sequences (sequence s draws chunk 100 + s)
        f = torch.from_numpy(np.concatenate([wl.bulk_features(cfg, T, chunk=100 + s) for s in range(B)])).to(dev)
        b = torch.empty(B * T, dtype=torch.uint8, device=dev)
        kvq.kvq_controller(f, mlp, b)
        return b.view(B, T).cpu().numpy()

    def build_cache(variant):
        t0 = time.time()
        bits = prefill_bits(variant)
        pools = []
        for w in (2, 4, 8, 16):
            need = 0
            for s in range(B):
                need += math.ceil(((bits[s, :lens0[s]] == w).sum() + 4 * n_steps + 16) / 256) + 1
            pools.append(int(need))
        cache = kvq.Cache(L, B, Hq, Hkv, max_ctx, pool_pages=pools)
        if variant == "kchannel":
            # static per-channel key quantizer, calibrated offline as +-4 sigma of each channel of the synthetic keys
            sig = torch.stack([wl.channel_multipliers(cfg, l_, 0) for l_ in range(L)])
            cache.set_k_channel_quant((-4.0 * sig).to(torch.float16).to(dev), (8.0 * sig).to(torch.float16).to(dev))
        CH = 512
        Tmax = int(lens0.max())
        lens_d = torch.from_numpy(lens0).to(dev)
        for ci, t in enumerate(range(0, Tmax, CH)):
            tc = min(CH, Tmax - t)
            # ragged prefill: sequences shorter than this chunk's end take part with fewer tokens, so they are
            # appended in groups of equal remaining length
            rem = np.clip(lens0 - t, 0, tc)
            for r in sorted(set(rem.tolist())):
                if r == 0:
                    continue
                idx = np.where(rem == r)[0]
                ids = torch.from_numpy(idx.astype(np.int32)).to(dev)
                bt = torch.from_numpy(np.ascontiguousarray(bits[idx, t:t + r])).to(dev)
                for layer in range(L):
                    K, V = wl.kv_chunk_fast(cfg, layer, ci, B, tc, dev)
                    if len(idx) == B and r == tc:
                        kvq.kvq_append(cache, layer, K, V, bt if layer == 0 else None, None, B, tc)
                    else:
                        kvq.kvq_append(cache, layer, K[idx, :r].contiguous(), V[idx, :r].contiguous(),
                                       bt if layer == 0 else None, ids, len(idx), r)
                    del K, V
        del lens_d
        flags, free = cache.status()
        if flags:
            raise RuntimeError("cache build raised device flags %d (free pages %s)" % (flags, free))
        log("[bench] built %s cache: %d layers, %.2f GB arena, %.1f s" %
            (variant, L, kvq.Cache.arena_bytes(L, B, Hq, Hkv, max_ctx, pool_pages=pools) / 1e9, time.time() - t0))
        return cache

    # ---------------- per-step inputs, resident before timing ---------------------------------------
    counts_np, N, Vobs, probs_tab = wl.zipf_table(cfg)
    step_logits = [wl.logits(cfg, s, B, dev) for s in range(n_steps)]
    step_ids = [torch.from_numpy(wl.zipf_ids(cfg, probs_tab, s, B)).to(dev) for s in range(n_steps)]
    step_len = [torch.from_numpy((lens0 + s).astype(np.int32)).to(dev) for s in range(4 * n_steps + 16)]
    done_steps = {}                                          # cache id -> decode steps already run on it
    n_in = min(n_steps, 4)                                   # K/V/q of the new token: a few distinct sets, cycled
    step_k = [[wl.kv_chunk_fast(cfg, l, 5000 + s, B, 1, dev) for l in range(L)] for s in range(n_in)]
    step_q = [[wl.queries(cfg, l, s, B, dev) for l in range(L)] for s in range(n_in)]
    feats = torch.zeros((B, 4), dtype=torch.float32, device=dev)
    step_bits = torch.zeros((B, 1), dtype=torch.uint8, device=dev)
    out = torch.zeros((B, Hq, 64), dtype=torch.float32, device=dev)
    sum_p2 = torch.full((B, Hq), 1.0 / float(cfg.context), dtype=torch.float32, device=dev)
    fws = torch.empty(kvq.kvq_features_workspace(B, wl.VOCAB), dtype=torch.uint8, device=dev)

    def algorithmic_bytes(counts):
        """decode-attention bytes of ONE layer: codes + (scale, min) pairs of every cached token and kv-head, plus q in, out back"""
        per_class = counts[:B, :4].to(torch.float64).sum(dim=0).tolist()
        kv = sum(n * Hkv * wl.BYTES_PER_TOKEN_HEAD[w] for n, w in zip(per_class, (2, 4, 8, 16)))
        return kv + B * Hq * 64 * (2 + 4), per_class

    def run_variant(variant, timed_steps, warm_steps, events, fused=False, cache=None, graph=False, rotate=None):
        cache = cache or build_cache(variant)
        aws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev)
        counts_d = torch.from_numpy(counts_np).to(dev)
        totals_d = torch.tensor([N, Vobs], dtype=torch.int64, device=dev)
        fixed = None
        if variant in STATIC_WIDTH:
            fixed = torch.full((B, 1), STATIC_WIDTH[variant], dtype=torch.uint8, device=dev)
        ev_pairs, stage_ev = [], []
        base_step = done_steps.get(id(cache), 0)
        done_steps[id(cache)] = base_step + warm_steps + timed_steps + (1 if graph else 0)

        ring = [cache] + list(rotate or [])                     # rotating copies: step s works on copy s mod len(ring)
        main_cache = cache

        def step(s, record):
            cache = ring[s % len(ring)]
            if record:
                e0 = torch.cuda.Event(enable_timing=True); e0.record()
            if fused:
                # two launches: features, controller, count update and the cache's bucket bookkeeping for the new token
                kvq.kvq_features_controller(step_logits[s % n_steps], step_ids[s % n_steps], counts_d, totals_d, True, sum_p2,
                                            step_len[base_step + s], Hq, mlp, feats, step_bits.view(-1), fws,
                                            cache=cache if fixed is None else None)
                if record:
                    e2 = torch.cuda.Event(enable_timing=True); e2.record()
                    stage_ev.append((e0, e2, e2))
            else:
                kvq.kvq_features(step_logits[s % n_steps], step_ids[s % n_steps], counts_d, totals_d, True, step_len[base_step + s], Hq, feats, fws, sum_p2=sum_p2)
                if record:
                    e1 = torch.cuda.Event(enable_timing=True); e1.record()
                if variant == "rule":
                    kvq.kvq_rule_policy(feats, rule, step_bits.view(-1))
                else:
                    kvq.kvq_controller(feats, mlp, step_bits.view(-1))
                if record:
                    e2 = torch.cuda.Event(enable_timing=True); e2.record()
                    stage_ev.append((e0, e1, e2))
            bits_now = step_bits if fixed is None else fixed
            kin, qin = step_k[s % n_in], step_q[s % n_in]
            for l in range(L):
                if not fused:
                    kvq.kvq_append(cache, l, kin[l][0], kin[l][1], bits_now if l == 0 else None, None, B, 1)
                if record:
                    a0 = torch.cuda.Event(enable_timing=True); a0.record()
                if fused:
                    # layer 0 passes no bits when the front end has already advanced the cache
                    b0 = bits_now.view(-1) if (l == 0 and fixed is not None) else None
                    kvq.kvq_append_decode_attn(cache, l, kin[l][0], kin[l][1], b0, qin[l], None, B,
                                               out, aws, None, sum_p2 if l == L - 1 else None)
                else:
                    kvq.kvq_decode_attn(cache, l, qin[l], None, B, out, aws, None, sum_p2 if l == L - 1 else None)
                if record:
                    a1 = torch.cuda.Event(enable_timing=True); a1.record()
                    ev_pairs.append((a0, a1))

        # the device drops its clocks within a second of idling (the CPU-oracle leg, a cache build on the host side) and
        # takes ~15 ms of work to bring them back: read-only attention launches until 40 ms have passed, then the warm-up steps
        t_spin = time.perf_counter()
        while time.perf_counter() - t_spin < 0.040:
            for l in range(L):
                kvq.kvq_decode_attn(cache, l, step_q[0][l], None, B, out, aws)
            torch.cuda.synchronize()
        for s in range(warm_steps):
            step(s, False)
        torch.cuda.synchronize()
        c_before = cache.counts()
        # a collector pause on the host drains the launch queue and shows up as device idle time inside the event
        # brackets, so the cyclic collector is off while the steps are timed
        replay = None
        if graph:
            # one decode step captured as a HIP graph (kernel launches only) and replayed: the same input buffers every
            # time, one more token per sequence and layer each replay
            events = False
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(warm_steps, False)
            replay = g.replay
            torch.cuda.synchronize()
            c_before = cache.counts()
        gc.collect()
        gc.disable()
        t0 = time.perf_counter()
        for s in range(warm_steps, warm_steps + timed_steps):
            if replay is not None:
                replay()
            else:
                # event brackets on EVENT_STEPS of the timed steps only: an event record costs ~3 us of device time, and
                # bracketing every launch of every step would inflate the step by 5 %, every fourth by about 1 %
                every = max(1, timed_steps // EVENT_STEPS)
                step(s, events and (s - warm_steps) % every == every // 2)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        gc.enable()
        c_after = cache.counts()
        flags, _ = cache.status()
        if flags:
            raise RuntimeError("device flags %d raised during the timed steps" % flags)
        ms_per_step = (t1 - t0) * 1e3 / timed_steps
        bytes_b, mix_b = algorithmic_bytes(c_before)
        bytes_a, mix_a = algorithmic_bytes(c_after)
        abytes = 0.5 * (bytes_b + bytes_a)
        res = {"ms_per_step": ms_per_step, "attn_bytes_per_layer": abytes,
               "tokens_per_class": [0.5 * (x + y) for x, y in zip(mix_b, mix_a)]}
        if events:
            attn_us = [a0.elapsed_time(a1) * 1e3 for a0, a1 in ev_pairs]
            if args.trace_steps:
                per = np.array(attn_us).reshape(-1, L).mean(axis=1)
                log("[bench] attn us/layer by step: " + " ".join("%.0f" % x for x in per))
            if not fused and L > 1:
                # what lies between the end of one layer's attention and the start of the next one's: that layer's append
                # (layers >= 1: no bookkeeping), plus one event record (~3 us)
                gaps = [ev_pairs[i][1].elapsed_time(ev_pairs[i + 1][0]) * 1e3 for i in range(len(ev_pairs) - 1) if i % L != L - 1]
                res["append_us_per_layer"] = float(np.median(gaps))
            res["attn_launches_timed"] = len(attn_us)
            res["attn_us_per_layer"] = float(np.mean(attn_us))
            res["attn_us_min"] = float(np.min(attn_us))
            res["attn_us_median"] = float(np.median(attn_us))
            res["features_us"] = float(np.mean([e0.elapsed_time(e1) * 1e3 for e0, e1, _ in stage_ev]))
            res["controller_us"] = float(np.mean([e1.elapsed_time(e2) * 1e3 for _, e1, e2 in stage_ev]))
            res["front_us"] = float(np.mean([e0.elapsed_time(e2) * 1e3 for e0, _, e2 in stage_ev]))
            res["attn_GBps"] = abytes / (res["attn_us_per_layer"] * 1e-6) / 1e9
        return cache, res

    # Releasing device memory (hipFree) makes every bandwidth-bound launch that follows 3-5 % slower until the device has
    # idled for a while (measured: the same cache, the same launches, before and after freeing an unrelated buffer), so
    # nothing is freed before the last timed loop has run: caches that are done with are parked here.  Config 4's five
    # caches take about 150 GB together.
    graveyard = []

    # ---------------- mixed-precision path: the metric ----------------------------------------------
    cache, mixed = run_variant(args.variant, args.steps, args.warmup, not args.no_events)
    # the same step with append fused into the attention launch (one kernel per layer instead of two), continuing on
    # the same cache; its token count stays below max_context because n_steps covers both loops
    fused = None
    if not args.no_fused:
        _, fused = run_variant(args.variant, args.steps, args.warmup, not args.no_events, fused=True, cache=cache)
    # small configs stay resident in the 256 MB Infinity Cache: time the same loop over rotating copies of the cache
    rotating = None
    total_bytes = mixed["attn_bytes_per_layer"] * L
    if total_bytes < 256e6 and not args.no_rotate:
        n_copies = int(min(64, math.ceil(512e6 / total_bytes)))
        copies = [build_cache(args.variant) for _ in range(n_copies - 1)]
        _, rot = run_variant(args.variant, args.steps, args.warmup, not args.no_events, cache=cache, rotate=copies)
        rotating = {"copies": n_copies, "total_MB": n_copies * total_bytes / 1e6, "us_per_step": rot["ms_per_step"] * 1e3,
                    "attn_us_per_layer": rot.get("attn_us_per_layer"),
                    "note": "four-call path, step s on copy s mod copies (at most 64 copies are built)"}
        graveyard.extend(copies)
    graph_res = None
    if not args.no_fused and not args.no_graph:
        _, graph_res = run_variant(args.variant, args.steps, args.warmup, False, fused=True, cache=cache, graph=True)

    # the front end alone, back to back on the launch stream with no event records in between (the in-step figures
    # above carry an event record per bracket and start behind a 100-us attention launch): 100 calls each, the steps'
    # logits in turn
    def front_loop(fn):
        for s_ in range(3):
            fn(s_)
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record()
        for s_ in range(100):
            fn(s_)
        f1.record()
        torch.cuda.synchronize()
        return f0.elapsed_time(f1) * 1e3 / 100

    fcounts = torch.from_numpy(counts_np).to(dev)
    ftotals = torch.tensor([N, Vobs], dtype=torch.int64, device=dev)
    flen = step_len[0]
    front_alone = {
        "fused_us": front_loop(lambda s_: kvq.kvq_features_controller(step_logits[s_ % n_steps], step_ids[s_ % n_steps], fcounts, ftotals,
                                                                     True, sum_p2, flen, Hq, mlp, feats, step_bits.view(-1), fws)),
        "separate_us": front_loop(lambda s_: (kvq.kvq_features(step_logits[s_ % n_steps], step_ids[s_ % n_steps], fcounts, ftotals, True, flen,
                                                              Hq, feats, fws, sum_p2=sum_p2),
                                              kvq.kvq_controller(feats, mlp, step_bits.view(-1)))),
        "note": "kvq_features_controller (two launches) against kvq_features + kvq_controller (four launches), 100 calls back "
                "to back without event records or cache bookkeeping; a call that launches one small kernel costs about 7 us of host time whatever the kernel does"}

    # measured streaming-read rate of a trivial kernel on this device (context for the 8 TB/s nominal peak)
    probe = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    probe.zero_()
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for _ in range(2):
        benchprobe.read(probe, sink)
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    for _ in range(5):
        benchprobe.read(probe, sink)
    p1.record()
    torch.cuda.synchronize()
    stream_gbps = 5 * probe.numel() / (p0.elapsed_time(p1) * 1e-3) / 1e9
    # one plain copy of known size (1 GiB read + 1 GiB written): the reference reading for the hardware byte counters
    half = probe.numel() // 2
    benchprobe.copy(probe[half:], probe[:half])
    torch.cuda.synchronize()
    # what a trivial kernel reaches when it writes a byte for every three it reads (the prefill append's ratio): the
    # last quarter of the buffer is written from the three quarters before it
    quarter = probe.numel() // 4
    for _ in range(2):
        benchprobe.mix3(probe[3 * quarter:], probe[:3 * quarter])
    p0.record()
    for _ in range(5):
        benchprobe.mix3(probe[3 * quarter:], probe[:3 * quarter])
    p1.record()
    torch.cuda.synchronize()
    mix3_gbps = 5 * 4 * quarter / (p0.elapsed_time(p1) * 1e-3) / 1e9
    del probe

    # ---------------- prefill-stage kernels at this config's shape --------------------------------------
    prefill = None
    if not args.no_prefill:
        ctx = min(int(cfg.context), 8192)
        n_rows = B * ctx
        f = torch.from_numpy(wl.bulk_features(cfg, n_rows, chunk=7)).to(dev)
        bb = torch.empty(n_rows, dtype=torch.uint8, device=dev)
        kvq.kvq_controller(f, mlp, bb)                            # warm-up
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(5):
            kvq.kvq_controller(f, mlp, bb)
        c1.record()
        torch.cuda.synchronize()
        ctrl_us = c0.elapsed_time(c1) * 1e3 / 5
        macs = sum(int(w.numel()) for w in mlp.W)
        if cfg.bits_kind == "uniform":
            pb = torch.from_numpy(wl.uniform_bits(cfg, B, ctx)).to(dev)
        elif cfg.bits_kind == "runs":
            pb = torch.from_numpy(np.stack([wl.run_bits(cfg, s_, ctx) for s_ in range(B)])).to(dev)
        else:
            pb = bb.view(B, ctx)
        Tc = min(2048, ctx)
        nch = ctx // Tc
        # a prompt chunk goes through every layer back to back, each layer with K/V of its own: PL layers here, layer 0
        # with the bookkeeping, the others timed as "what every further layer costs" (in steady state a call also
        # carries the write-back of what the call before it left in the caches)
        PL = 5
        pc = kvq.Cache(PL, B, Hq, Hkv, Tc * nch)
        evs = []
        for c in range(nch):
            kv_l = [wl.kv_chunk_fast(cfg, l_ % L, 9000 + c, B, Tc, dev) for l_ in range(PL)]
            bt = pb[:, c * Tc:(c + 1) * Tc].contiguous()
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(PL + 1)]
            marks[0].record()
            for l_ in range(PL):
                kvq.kvq_append(pc, l_, kv_l[l_][0], kv_l[l_][1], bt if l_ == 0 else None, None, B, Tc)
                marks[l_ + 1].record()
            evs.append(marks)
            del kv_l
        torch.cuda.synchronize()
        pflags, _ = pc.status()
        if pflags:
            raise RuntimeError("prefill append raised device flags %d" % pflags)
        cnt = pc.counts()[:B, :4].to(torch.float64).sum(dim=0).tolist()
        app_bytes = sum(n * Hkv * (256 + wl.BYTES_PER_TOKEN_HEAD[w]) for n, w in zip(cnt, (2, 4, 8, 16))) / nch
        us0 = float(np.median([m[0].elapsed_time(m[1]) * 1e3 for m in evs]))
        us1 = float(np.median([m[i].elapsed_time(m[i + 1]) * 1e3 for m in evs for i in range(1, PL)]))
        prefill = {
            "controller": {"rows": n_rows, "us": ctrl_us, "rows_per_s": n_rows / (ctrl_us * 1e-6),
                           "TFLOPs": 2 * macs * n_rows / (ctrl_us * 1e-6) / 1e12, "frac_of_fp32_mfma_peak": 2 * macs * n_rows / (ctrl_us * 1e-6) / 1e12 / 157.3},
            "append": {"tokens_per_seq_per_call": Tc, "bytes_per_call": app_bytes, "us_layer0_with_bookkeeping": us0, "us_other_layers": us1,
                       "GBps_other_layers": app_bytes / (us1 * 1e-6) / 1e9, "frac_of_hbm_peak": app_bytes / (us1 * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                       "frac_of_stream_mix3": app_bytes / (us1 * 1e-6) / 1e9 / mix3_gbps},
            "note": "bulk controller (fp32 MFMA) on batch x context rows in one call; bulk append in 2048-token chunks, five layers "
                    "back to back per chunk with K/V of their own (median over the layers after the first); "
                    "algorithmic bytes = 256 B read + the class's bytes written per (token, kv-head)"}
        # the controller's training step (Sec. 3.8, Algorithm 1) on mini-batches of labelled feature rows
        tr = {}
        hp = kvq.make_train_hparams(1.0, 0.3, 0.7, [0.2, 0.35, 0.6, 1.0], [0.55, 0.8, 0.95, 1.0], lr=1e-3)
        tw = kvq.MlpWeights([w.clone() for w in mlp.W], [b_.clone() for b_ in mlp.b])
        tm = kvq.MlpWeights([torch.zeros_like(w) for w in mlp.W], [torch.zeros_like(b_) for b_ in mlp.b])
        tv = kvq.MlpWeights([torch.zeros_like(w) for w in mlp.W], [torch.zeros_like(b_) for b_ in mlp.b])
        for nb in (256, 4096):
            tws = torch.empty(kvq.kvq_controller_train_workspace(tw, nb), dtype=torch.uint8, device=dev)
            for t_ in range(1, 4):
                kvq.kvq_controller_train_step(f[:nb], bb[:nb], tw, tm, tv, hp, t_, tws)
            t0_, t1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0_.record()
            for t_ in range(4, 24):
                kvq.kvq_controller_train_step(f[:nb], bb[:nb], tw, tm, tv, hp, t_, tws)
            t1_.record()
            torch.cuda.synchronize()
            us_ = t0_.elapsed_time(t1_) * 1e3 / 20
            tr["batch_%d" % nb] = {"us_per_step": us_, "GFLOPs": 6 * macs * nb / (us_ * 1e-6) / 1e9}
        prefill["train_step"] = tr
        graveyard.append(pc)
        del f, bb, pb

    # ---------------- CPU oracle on a bounded sample -------------------------------------------------
    cpu = None
    if not args.no_cpu:
        import oracle
        ns = min(args.cpu_seqs, B) if args.cpu_seqs > 0 else B
        T = int(lens0.max())
        # the oracle runs its own pipeline on the same seeded inputs: controller -> quantize/append -> attention
        exp_bits = []
        for s in range(ns):
            n_s = int(lens0[s])
            if cfg.bits_kind == "controller":
                b_s, _ = oracle.controller(wl.bulk_features(cfg, T, chunk=100 + s), Ws, bs)
            elif cfg.bits_kind == "runs":
                b_s = wl.run_bits(cfg, s, T)
            else:
                b_s = wl.uniform_bits(cfg, B, T)[s]
            exp_bits.append(np.asarray(b_s[:n_s], np.uint8))
        Lmax = max(len(b) for b in exp_bits)
        # layer 0's source K/V of the sample sequences, regenerated from their seeds and copied to the host
        codes = np.zeros((ns, Lmax, Hkv, 2, 128), np.uint8)
        meta = np.zeros((ns, Lmax, Hkv, 2, 2), np.uint16)
        bits_h = np.zeros((ns, Lmax), np.uint8)
        CH = 512
        for ci, t in enumerate(range(0, T, CH)):
            tc = min(CH, T - t)
            K, V = wl.kv_chunk_fast(cfg, 0, ci, B, tc, dev)
            Kh = K[:ns].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            Vh = V[:ns].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            for s in range(ns):
                r = int(min(max(lens0[s] - t, 0), tc))
                if r:
                    c, m = oracle.append(Kh[s, :r], Vh[s, :r], exp_bits[s][t:t + r], parallel=True)
                    codes[s, t:t + r], meta[s, t:t + r], bits_h[s, t:t + r] = c, m, exp_bits[s][t:t + r]
            del K, V
        lens_h = np.array([min(int(lens0[s]), Lmax) for s in range(ns)], np.int32)
        q = step_q[0][0][:ns].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        best, nthr = None, 1
        for _ in range(3):
            c0 = time.perf_counter()
            _, _, _, nthr = oracle.decode_attn_batch(q, bits_h, codes, meta, lens_h, Hq)
            dt = time.perf_counter() - c0
            best = dt if best is None else min(best, dt)
        scale = (float(lens0.sum()) / float(lens_h.sum())) * L
        # the rest of the step, once each: features (explicit attention rows of the final layer: the oracle takes the
        # literal two-pass variance), controller, and the quantize-and-append of one token per sequence and layer
        rng_c = np.random.default_rng(1)
        lg = step_logits[0].cpu().numpy()
        ids_h = step_ids[0].cpu().numpy()
        ld = int(lens_h.max())
        probs = rng_c.random((B, Hq, ld))
        probs /= probs.sum(axis=2, keepdims=True)
        # these three legs are spread over the host cores row by row / sequence by sequence (the oracle's calls release
        # the interpreter lock), like the attention leg
        from concurrent.futures import ThreadPoolExecutor
        nw = max(1, min(nthr, B))
        cuts = np.linspace(0, B, nw + 1).astype(int)
        parts = [(int(a), int(b)) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
        with ThreadPoolExecutor(max_workers=nw) as pool:
            c0 = time.perf_counter()
            f_h = np.concatenate(list(pool.map(
                lambda ab: oracle.features(lg[ab[0]:ab[1]], ids_h[ab[0]:ab[1]], counts_np, N, Vobs, probs[ab[0]:ab[1]],
                                           np.full(ab[1] - ab[0], ld, np.int32)), parts)))
            oracle.counts_update(ids_h, counts_np, N, Vobs)
            t_feat = time.perf_counter() - c0
            c0 = time.perf_counter()
            b_h, _ = oracle.controller(f_h, Ws, bs)
            t_ctrl = time.perf_counter() - c0
            k1 = step_k[0][0][0].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)   # [B,1,Hkv,64]
            v1 = step_k[0][0][1].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            c0 = time.perf_counter()
            list(pool.map(lambda s_: oracle.append(k1[s_], v1[s_], np.asarray(b_h[s_:s_ + 1], np.uint8)), range(B)))
            t_app = (time.perf_counter() - c0) * L
        del probs
        total = best * scale + t_feat + t_ctrl + t_app
        cpu = {"value": total * 1e6, "unit": "us/step", "cores": nthr, "kind": "oracle",
               "sample": "decode attention of %d of %d sequences of ONE layer at full context (min of 3 runs, %.2f s each on %d "
                         "threads), scaled by tokens to the batch and by %d layers = %.2f s; plus, timed once: features of the "
                         "batch %.3f s, controller %.4f s, quantize-and-append of one token per sequence x %d layers %.3f s "
                         "(features and append spread over %d threads by rows / sequences, the controller's %d rows on one)" % (ns, B, best, nthr, L, best * scale, t_feat, t_ctrl, L, t_app, nw, B)}
    tok = mixed["tokens_per_class"]
    tot = sum(tok) or 1.0
    result = {
        "metric": "mixed-precision decode-attn us/step",
        "value": mixed["ms_per_step"] * 1e3,
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": mixed["ms_per_step"],
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u2/u4/u8 codes + f16 scale/min, f16 storage class, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": cfg.name, "variant": args.variant, "config_index": cfg.index, "layers": L, "batch": B, "context": cfg.context,
                   "q_heads": Hq, "kv_heads": Hkv, "head_dim": 64,
                   "mix_2_4_8_16": [round(x / tot, 4) for x in tok],
                   "expected_bits": round(sum(x * w for x, w in zip(tok, (2, 4, 8, 16))) / tot, 3)},
        "stages_us": {"features": mixed.get("features_us"), "controller": mixed.get("controller_us"),
                      "append_per_layer": mixed.get("append_us_per_layer"),
                      "attn_per_layer": mixed.get("attn_us_per_layer"), "attn_per_layer_median": mixed.get("attn_us_median"),
                      "attn_per_layer_min": mixed.get("attn_us_min"), "attn_launches_timed": mixed.get("attn_launches_timed")},
        "stream_read_GBps": stream_gbps,
        "stream_mix3_GBps": mix3_gbps,
        "fused_path": None if fused is None else {
            "us_per_step": fused["ms_per_step"] * 1e3, "launch_us_per_layer": fused.get("attn_us_per_layer"),
            "front_us": fused.get("front_us"),
            "note": "same step through kvq_features_controller (features + controller + count update + bookkeeping, two launches) and "
                    "kvq_append_decode_attn (append + attention, one launch per layer); `value` above is the four-call path"},
        "graph_replay": None if graph_res is None else {
            "us_per_step": graph_res["ms_per_step"] * 1e3,
            "note": "the fused path's step captured once as a HIP graph and replayed (launch overhead off the host)"},
        "front_end_alone": front_alone,
        "rotating_copies": rotating,
        "prefill": prefill,
        "compare": compare,
    }
    # HBM bytes per launch by the hardware counters: taken in rocprofv3 --pmc runs of this command and condensed by
    # benchprobe/pmc_summary.py into profiles/; printed only while the attention kernel's sources are the ones profiled
    traffic, traffic_note = None, None
    tname = "k_decode_split_cfg%d%s_traffic.txt" % (cfg.index, "" if args.variant == "mixed" else "_" + args.variant)
    tpath = os.path.join(ROOT, "profiles", tname)
    if os.path.exists(tpath) and L == cfg.n_layers:
        from benchprobe.pmc_summary import sources_sha256
        kv = dict(line.strip().split("=", 1) for line in open(tpath) if "=" in line and not line.startswith("#"))
        if kv.get("sources_sha256") == sources_sha256():
            traffic = float(kv["traffic_bytes_per_launch"])
        else:
            traffic_note = "profiles/%s was taken from other kernel sources than the ones in this tree" % tname
    if "attn_GBps" in mixed:
        result["roofline"] = {"bound": "hbm", "achieved": mixed["attn_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": mixed["attn_GBps"] / HBM_PEAK_GBPS, "traffic": traffic,
                              "kernel": "k_decode_split", "bytes_per_launch": mixed["attn_bytes_per_layer"],
                              "frac_of_stream_read": mixed["attn_GBps"] / stream_gbps}
        if traffic_note:
            result["roofline"]["traffic_note"] = traffic_note
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


if __name__ == "__main__":
    main()
