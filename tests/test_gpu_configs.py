"""GPU parity on the five benchmark configurations' shapes, driven by the seeded workload generators.

Configs 1-3 run their real batch / context / head shapes (with fewer layers than the full stack, since layers
are shape-identical and independent); configs 4 and 5 run ONE layer at the full shape, in the launch
configuration the benchmark times (library defaults), and are checked on sampled sequences against the oracle
plus properties that hold for every output.  Bit widths fed to kvq_append come from the ORACLE's controller, so
that a controller tie can never leak into the bit-exact cache comparison; the GPU controller is compared
separately under the tie rule.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import ATOL, RTOL, assert_attn_close, dev, to_bits_u16
from paper_2604_04722_amd import binding as kvq
import workloads as wl

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def controller_bits_both(cfg, feats):
    """bits from the oracle (returned) and from the GPU (checked against them under the tie rule)."""
    Ws, bs = wl.calibrated_mlp(cfg) if cfg.bits_kind == "controller" else wl.xavier_mlp(cfg)
    want, logits = oracle.controller(feats, Ws, bs)
    d = dev()
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    got = torch.zeros(feats.shape[0], dtype=torch.uint8, device=d)
    kvq.kvq_controller(torch.from_numpy(feats).to(d), mlp, got)
    got = got.cpu().numpy()
    srt = np.sort(logits, axis=1)
    tie = (srt[:, -1] - srt[:, -2]) <= 1e-5
    assert np.all((got == want) | tie), "controller assignment differs off a tie"
    return want


def prefill(cfg, cache, layer_count, bits, lens, chunk=512, layers=None):
    """Append bits[s, :lens[s]] tokens of every sequence, all layers (or `layers`, which must start with 0: the layer-0
    call does the bookkeeping), from kv_chunk_fast draws."""
    layers = list(range(layer_count)) if layers is None else list(layers)
    assert layers[0] == 0
    B = bits.shape[0]
    d = dev()
    Tmax = int(lens.max())
    for ci, t in enumerate(range(0, Tmax, chunk)):
        tc = min(chunk, Tmax - t)
        rem = np.clip(lens - t, 0, tc)
        for r in sorted(set(rem.tolist())):
            if r == 0:
                continue
            idx = np.where(rem == r)[0]
            ids = torch.from_numpy(idx.astype(np.int32)).to(d)
            bt = torch.from_numpy(np.ascontiguousarray(bits[idx, t:t + r])).to(d)
            for layer in layers:
                K, V = wl.kv_chunk_fast(cfg, layer, ci, B, tc, d)
                if len(idx) == B and r == tc:
                    kvq.kvq_append(cache, layer, K, V, bt if layer == 0 else None, None, B, tc)
                else:
                    kvq.kvq_append(cache, layer, K[idx, :r].contiguous(), V[idx, :r].contiguous(),
                                   bt if layer == 0 else None, ids, len(idx), r)


def oracle_cache_for(cfg, layer, seqs, bits, lens, chunk=512):
    """Canonical arrays of the sampled sequences, quantized by the oracle from host copies of the same draws."""
    B = bits.shape[0]
    d = dev()
    Tmax = int(lens.max())
    Hkv = cfg.n_kv_heads
    codes = {s: np.zeros((int(lens[s]), Hkv, 2, 128), np.uint8) for s in seqs}
    meta = {s: np.zeros((int(lens[s]), Hkv, 2, 2), np.uint16) for s in seqs}
    for ci, t in enumerate(range(0, Tmax, chunk)):
        tc = min(chunk, Tmax - t)
        K, V = wl.kv_chunk_fast(cfg, layer, ci, B, tc, d)
        for s in seqs:
            r = int(min(max(lens[s] - t, 0), tc))
            if r == 0:
                continue
            c, m = oracle.append(to_bits_u16(K[s, :r]), to_bits_u16(V[s, :r]), bits[s, t:t + r], parallel=True)
            codes[s][t:t + r], meta[s][t:t + r] = c, m
        del K, V
    return codes, meta


def check_sampled(cfg, cache, layer, seqs, bits, lens, codes, meta, q):
    B, Hq = bits.shape[0], cfg.n_q_heads
    d = dev()
    out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=d)
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=d)
    p2 = torch.zeros((B, Hq), dtype=torch.float32, device=d)
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=d)
    kvq.kvq_decode_attn(cache, layer, q, None, B, out, ws, lse, p2)      # library-default launch configuration
    torch.cuda.synchronize()
    out_h, lse_h, p2_h = out.cpu().numpy(), lse.cpu().numpy(), p2.cpu().numpy()
    # properties that hold for every output, whatever the size
    assert np.all(np.isfinite(out_h)) and np.all(np.isfinite(lse_h))
    assert np.all(p2_h > 0) and np.all(p2_h <= 1.0 + 1e-5)               # sum p^2 in (0, 1]
    assert np.all(p2_h * lens[:, None] >= 1.0 - 1e-3)                    # >= 1/l by Cauchy-Schwarz
    for s in seqs:
        n = int(lens[s])
        eb, ec, em = cache.export(layer, s, n)
        assert np.array_equal(eb.cpu().numpy(), bits[s, :n])
        assert np.array_equal(em.cpu().numpy().view(np.uint16), meta[s]), "scales / minima differ (seq %d)" % s
        assert np.array_equal(ec.cpu().numpy(), codes[s]), "packed codes differ (seq %d)" % s
        want, want_lse, probs = oracle.decode_attn(to_bits_u16(q[s]), bits[s, :n], codes[s], meta[s], Hq, want_probs=True)
        assert_attn_close(out_h[s], want, "cfg %d seq %d" % (cfg.index, s))
        np.testing.assert_allclose(lse_h[s], want_lse, rtol=1e-4, atol=1e-4)
        np.testing.assert_allclose(p2_h[s], (probs ** 2).sum(axis=1), rtol=2e-3)


def test_config4_full_shape_one_layer_sampled_sequences():
    cfg = wl.CONFIGS[4]
    say("config 4: B=%d ctx=%d %dq/%dkv, one layer, library-default launch" % (cfg.batch, cfg.context, cfg.n_q_heads, cfg.n_kv_heads))
    B, T = cfg.batch, cfg.context
    lens = np.full(B, T, np.int64)
    bits = np.stack([controller_bits_both(cfg, wl.bulk_features(cfg, T, chunk=100 + s)) for s in range(B)])
    mix = np.array([(bits == w).mean() for w in (2, 4, 8, 16)])
    assert np.max(np.abs(mix - np.array(cfg.mix))) < 0.03
    pools = [int(sum(-(-int((bits[s] == w).sum()) // 256) + 1 for s in range(B))) for w in (2, 4, 8, 16)]
    cache = kvq.Cache(1, B, cfg.n_q_heads, cfg.n_kv_heads, T, pool_pages=pools)
    prefill(cfg, cache, 1, bits, lens)
    assert cache.status()[0] == 0
    seqs = [0, 13, 31]
    codes, meta = oracle_cache_for(cfg, 0, seqs, bits, lens)
    q = wl.queries(cfg, 0, 0, B, dev())
    check_sampled(cfg, cache, 0, seqs, bits, lens, codes, meta, q)
    # the same K/V as a static 4-bit cache and as an FP16 cache, same shape, sampled the same way
    cache.destroy()
    for width in (4, 16):
        say("config 4 comparison cache: all %d-bit" % width)
        bw = np.full((B, T), width, np.uint8)
        pools = [0, 0, 0, 0]
        pools[{4: 1, 16: 3}[width]] = B * (T // 256 + 1)
        pools = [p or 1 for p in pools]
        c2 = kvq.Cache(1, B, cfg.n_q_heads, cfg.n_kv_heads, T, pool_pages=pools)
        prefill(cfg, c2, 1, bw, lens)
        assert c2.status()[0] == 0
        codes2, meta2 = oracle_cache_for(cfg, 0, [5], bw, lens)
        check_sampled(cfg, c2, 0, [5], bw, lens, codes2, meta2, q)
        c2.destroy()


def test_config4_prefill_in_the_2048_token_calls_the_benchmark_times():
    cfg = wl.CONFIGS[4]
    say("config 4 prefill leg: B=%d, calls of 2048 tokens per sequence (the block-at-a-time writer at its benchmark shape)" % cfg.batch)
    B, T, CH = cfg.batch, cfg.context, 2048
    lens = np.full(B, T, np.int64)
    bits = np.stack([controller_bits_both(cfg, wl.bulk_features(cfg, T, chunk=100 + s)) for s in range(B)])
    pools = [int(sum(-(-int((bits[s] == w).sum()) // 256) + 1 for s in range(B))) for w in (2, 4, 8, 16)]
    cache = kvq.Cache(1, B, cfg.n_q_heads, cfg.n_kv_heads, T, pool_pages=pools)
    prefill(cfg, cache, 1, bits, lens, chunk=CH)
    assert cache.status()[0] == 0
    seqs = [7, 30]
    codes, meta = oracle_cache_for(cfg, 0, seqs, bits, lens, chunk=CH)
    q = wl.queries(cfg, 0, 0, B, dev())
    check_sampled(cfg, cache, 0, seqs, bits, lens, codes, meta, q)
    # every sequence, cheaply: class counts and the free pages they imply
    counts = cache.counts().cpu().numpy() if hasattr(cache.counts(), "cpu") else np.asarray(cache.counts())
    for s in range(B):
        assert [int(x) for x in counts[s, :4]] == [int((bits[s] == w).sum()) for w in (2, 4, 8, 16)]
    cache.destroy()


def test_config4_last_layer_of_the_full_24_layer_cache():
    """Layer addressing with multi-GB strides: the cache is created with all 24 layers and the pools bench.py gives it,
    layers 0 and 23 are written, and the LAST layer is compared with the oracle (export and attention, one sequence)."""
    cfg = wl.CONFIGS[4]
    B, T, L = cfg.batch, cfg.context, cfg.n_layers
    say("config 4: %d-layer cache (%d sequences x %d tokens), layers 0 and %d written, layer %d checked" % (L, B, T, L - 1, L - 1))
    lens = np.full(B, T, np.int64)
    bits = np.stack([controller_bits_both(cfg, wl.bulk_features(cfg, T, chunk=100 + s)) for s in range(B)])
    pools = [int(sum(-(-int((bits[s] == w).sum() + 64) // 256) + 1 for s in range(B))) for w in (2, 4, 8, 16)]
    cache = kvq.Cache(L, B, cfg.n_q_heads, cfg.n_kv_heads, T + 64, pool_pages=pools)
    prefill(cfg, cache, L, bits, lens, layers=[0, L - 1])
    assert cache.status()[0] == 0
    seqs = [B - 1]
    codes, meta = oracle_cache_for(cfg, L - 1, seqs, bits, lens)
    q = wl.queries(cfg, L - 1, 0, B, dev())
    check_sampled(cfg, cache, L - 1, seqs, bits, lens, codes, meta, q)
    cache.destroy()


@pytest.mark.parametrize("B", [16, 64])
def test_config5_ragged_long_context_run_clustered_widths_one_layer(B):
    """B = 64 is the config's real batch: 4096 waves for 2048 places, two waves per workgroup, longest-first launch
    order (the launch the benchmark times).  B = 16 is the same workload in the four-waves-per-workgroup, single-round
    regime."""
    cfg = wl.CONFIGS[5]
    say("config 5 shape: B=%d of %d, ragged ctx in [%d, %d], runs of equal width, one layer" % (B, cfg.batch, cfg.min_context, cfg.context))
    lens = wl.ragged_lengths(cfg).astype(np.int64)[:B]
    Tmax = int(lens.max())
    bits = np.stack([wl.run_bits(cfg, s, Tmax) for s in range(B)])
    pools = [int(sum(-(-int((bits[s, :lens[s]] == w).sum()) // 256) + 1 for s in range(B))) for w in (2, 4, 8, 16)]
    cache = kvq.Cache(1, B, cfg.n_q_heads, cfg.n_kv_heads, cfg.context, pool_pages=pools)
    prefill(cfg, cache, 1, bits, lens, chunk=1024)
    assert cache.status()[0] == 0
    counts = cache.counts()
    assert np.array_equal(counts[:B, 4].numpy(), lens)
    order = np.argsort(lens)
    seqs = [int(order[0]), int(order[-1])]
    if B == cfg.batch:
        seqs += [int(order[B // 3]), int(order[2 * B // 3])]           # shortest, longest and two in between
        mix = np.array([sum(int((bits[s, :lens[s]] == w).sum()) for s in range(B)) for w in (2, 4, 8, 16)], np.float64)
        assert np.max(np.abs(mix / mix.sum() - np.array(cfg.mix))) < 0.03
    codes, meta = oracle_cache_for(cfg, 0, seqs, bits, lens, chunk=1024)
    q = wl.queries(cfg, 0, 0, B, dev())
    check_sampled(cfg, cache, 0, seqs, bits, lens, codes, meta, q)
    cache.destroy()


def test_config3_shape_decode_steps_with_append_all_sequences_checked():
    cfg = wl.CONFIGS[3]
    L, steps = 2, 3
    say("config 3 shape: B=%d ctx=%d %dq/%dkv student-t channels, %d of %d layers, %d decode steps" %
        (cfg.batch, cfg.context, cfg.n_q_heads, cfg.n_kv_heads, L, cfg.n_layers, steps))
    B, T, Hq, Hkv = cfg.batch, cfg.context - steps, cfg.n_q_heads, cfg.n_kv_heads
    d = dev()
    lens = np.full(B, T, np.int64)
    bits = np.stack([controller_bits_both(cfg, wl.bulk_features(cfg, T, chunk=100 + s)) for s in range(B)])
    mix = np.array([(bits == w).mean() for w in (2, 4, 8, 16)])
    assert np.max(np.abs(mix - np.array(cfg.mix))) < 0.03
    cache = kvq.Cache(L, B, Hq, Hkv, cfg.context)
    prefill(cfg, cache, L, bits, lens)
    seqs = list(range(B))
    oc = [oracle_cache_for(cfg, l, seqs, bits, lens) for l in range(L)]
    all_bits = {s: bits[s].copy() for s in seqs}
    for step in range(steps):
        sb = controller_bits_both(cfg, wl.bulk_features(cfg, B, chunk=900 + step))
        bt = torch.from_numpy(sb.reshape(B, 1)).to(d)
        for l in range(L):
            k1, v1 = wl.kv_chunk_fast(cfg, l, 7000 + step, B, 1, d)
            kvq.kvq_append(cache, l, k1, v1, bt if l == 0 else None, None, B, 1)
            for s in seqs:
                c, m = oracle.append(to_bits_u16(k1[s]), to_bits_u16(v1[s]), sb[s:s + 1])
                oc[l][0][s] = np.concatenate([oc[l][0][s], c])
                oc[l][1][s] = np.concatenate([oc[l][1][s], m])
        for s in seqs:
            all_bits[s] = np.concatenate([all_bits[s], sb[s:s + 1]])
        n = T + step + 1
        bm = np.stack([all_bits[s] for s in seqs])
        for l in range(L):
            q = wl.queries(cfg, l, step, B, d)
            check_sampled(cfg, cache, l, seqs if step == steps - 1 else [0, B - 1], bm, np.full(B, n, np.int64), oc[l][0], oc[l][1], q)
    assert cache.status()[0] == 0
    cache.destroy()


def test_config2_shape_feature_controller_chain_feeds_the_cache():
    cfg = wl.CONFIGS[2]
    L, steps = 3, 4
    say("config 2 shape: B=1 ctx=%d %dq/%dkv, %d of %d layers; features -> controller -> append -> attention x %d steps" %
        (cfg.context, cfg.n_q_heads, cfg.n_kv_heads, L, cfg.n_layers, steps))
    B, T, Hq, Hkv = 1, cfg.context - steps, cfg.n_q_heads, cfg.n_kv_heads
    d = dev()
    Ws, bs = wl.calibrated_mlp(cfg)
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    lens = np.full(B, T, np.int64)
    bits = np.stack([controller_bits_both(cfg, wl.bulk_features(cfg, T, chunk=100))])
    cache = kvq.Cache(L, B, Hq, Hkv, cfg.context)
    prefill(cfg, cache, L, bits, lens)
    oc = [oracle_cache_for(cfg, l, [0], bits, lens) for l in range(L)]
    counts, N, Vobs, probs_tab = wl.zipf_table(cfg)
    counts_d = torch.from_numpy(counts).to(d)
    totals_d = torch.tensor([N, Vobs], dtype=torch.int64, device=d)
    o_counts, o_N, o_V = counts.copy(), N, Vobs
    fws = torch.empty(kvq.kvq_features_workspace(B, wl.VOCAB), dtype=torch.uint8, device=d)
    aws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=d)
    sum_p2 = torch.full((B, Hq), 1.0 / T, dtype=torch.float32, device=d)
    o_probs = np.full((B, Hq, T), 1.0 / T)                  # the oracle's attention row of the previous step
    cur_bits = bits[0].copy()
    n = T
    for step in range(steps):
        logits = wl.logits(cfg, step, B, d)
        ids = wl.zipf_ids(cfg, probs_tab, step, B)
        feats = torch.zeros((B, 4), dtype=torch.float32, device=d)
        alen = torch.tensor([n], dtype=torch.int32, device=d)
        kvq.kvq_features(logits, torch.from_numpy(ids).to(d), counts_d, totals_d, True, alen, Hq, feats, fws, sum_p2=sum_p2)
        want_f = oracle.features(logits.cpu().numpy(), ids, o_counts, o_N, o_V, o_probs, np.array([n], np.int32))
        o_counts, o_N, o_V = oracle.counts_update(ids, o_counts, o_N, o_V)
        got_f = feats.cpu().numpy()
        np.testing.assert_allclose(got_f[:, [0, 1, 3]], want_f[:, [0, 1, 3]], rtol=2e-5, atol=1e-6)
        assert abs(got_f[0, 2] - want_f[0, 2]) <= 2e-3 * abs(want_f[0, 2]) + 2e-6 / n ** 2   # V from sum_p2 (2e-3 rel on sum p^2)
        # the oracle decides on ITS features; the GPU controller is checked on the same (oracle) features
        want_bits, want_logits = oracle.controller(want_f, Ws, bs)
        gb = torch.zeros(B, dtype=torch.uint8, device=d)
        kvq.kvq_controller(torch.from_numpy(want_f).to(d), mlp, gb)
        srt = np.sort(want_logits, axis=1)
        assert np.all((gb.cpu().numpy() == want_bits) | ((srt[:, -1] - srt[:, -2]) <= 1e-5))
        bt = torch.from_numpy(want_bits.reshape(B, 1)).to(d)
        cur_bits = np.concatenate([cur_bits, want_bits])
        n += 1
        for l in range(L):
            k1, v1 = wl.kv_chunk_fast(cfg, l, 8000 + step, B, 1, d)
            kvq.kvq_append(cache, l, k1, v1, bt if l == 0 else None, None, B, 1)
            c, m = oracle.append(to_bits_u16(k1[0]), to_bits_u16(v1[0]), want_bits)
            oc[l][0][0] = np.concatenate([oc[l][0][0], c])
            oc[l][1][0] = np.concatenate([oc[l][1][0], m])
            q = wl.queries(cfg, l, step, B, d)
            out = torch.zeros((B, Hq, 64), dtype=torch.float32, device=d)
            kvq.kvq_decode_attn(cache, l, q, None, B, out, aws, None, sum_p2 if l == L - 1 else None)
            want, _, probs = oracle.decode_attn(to_bits_u16(q[0]), cur_bits, oc[l][0][0], oc[l][1][0], Hq, want_probs=True)
            assert_attn_close(out.cpu().numpy()[0], want, "step %d layer %d" % (step, l))
            if l == L - 1:
                o_probs = probs[None]                        # final-layer attention row feeds the next step's V_t
    assert np.array_equal(counts_d.cpu().numpy(), o_counts)
    assert cache.status()[0] == 0
    cache.destroy()
