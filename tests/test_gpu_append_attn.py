"""GPU parity: kvq_append / kvq_cache_export bit-exact, kvq_decode_attn within tolerance, against the CPU oracle.

Every test prints what it is about to run (flushed) before touching the GPU.
"""
import numpy as np
import pytest
import torch

from helpers import (OracleCache, assert_attn_close, assert_export_equals, dev, tuning, gpu_f16, make_kv, to_bits_u16)
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def build_both(B, T, Hq, Hkv, bits, seed, n_layers=1, max_context=None, chunk=None, kinds=("outlier", "outlier"),
               page_tokens=0, pool_pages=(0, 0, 0, 0)):
    """Appends T tokens per sequence (bits[B,T]) to a fresh GPU cache and to an oracle cache, layer by layer."""
    max_context = max_context or max(T, 1)
    cache = kvq.Cache(n_layers, B, Hq, Hkv, max_context, page_tokens=page_tokens, pool_pages=pool_pages)
    ocs = [OracleCache(B, Hkv) for _ in range(n_layers)]
    chunk = chunk or max(T, 1)
    for t0 in range(0, T, chunk):
        tc = min(chunk, T - t0)
        bt = torch.from_numpy(np.ascontiguousarray(bits[:, t0:t0 + tc])).to(dev())
        for L in range(n_layers):
            K = make_kv((B, tc, Hkv, 64), seed + 1000 * L + t0, outlier=kinds[0] == "outlier")
            V = make_kv((B, tc, Hkv, 64), seed + 1000 * L + t0 + 500, outlier=kinds[1] == "outlier")
            kvq.kvq_append(cache, L, gpu_f16(K), gpu_f16(V), bt if L == 0 else None, None, B, tc)
            for b in range(B):
                ocs[L].append(b, K[b], V[b], bits[b, t0:t0 + tc])
    torch.cuda.synchronize()
    return cache, ocs


def run_attn(cache, layer, q16, B, Hq, want_aux=True):
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
    out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=dev()) if want_aux else None
    p2 = torch.zeros((B, Hq), dtype=torch.float32, device=dev()) if want_aux else None
    kvq.kvq_decode_attn(cache, layer, gpu_f16(q16), None, B, out, ws, lse, p2)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (lse.cpu().numpy() if want_aux else None), (p2.cpu().numpy() if want_aux else None)


@pytest.mark.parametrize("b", [2, 4, 8, 16])
@pytest.mark.parametrize("T", [1, 63, 64, 65, 300])
def test_uniform_width_append_is_bit_exact(b, T):
    say("append uniform b=%d T=%d" % (b, T))
    B, Hq, Hkv = 2, 4, 2
    bits = np.full((B, T), b, np.uint8)
    cache, ocs = build_both(B, T, Hq, Hkv, bits, seed=b * 100 + T)
    for s in range(B):
        assert_export_equals(cache, 0, s, ocs[0])
    assert cache.status()[0] == 0


def test_config1_shape_mixed_append_bit_exact_and_attention_matches():
    say("config 1 shape: ctx 512, 9q/3kv, uniform random widths, one bulk append")
    import workloads as wl
    cfg = wl.CONFIGS[1]
    bits = wl.uniform_bits(cfg, 1, cfg.context)
    cache, ocs = build_both(1, cfg.context, cfg.n_q_heads, cfg.n_kv_heads, bits, seed=11)
    assert_export_equals(cache, 0, 0, ocs[0])
    q = make_kv((1, cfg.n_q_heads, 64), 12, outlier=False)
    for splits in (0, 1, 3):
        with tuning(attn_splits=splits):
            out, lse, p2 = run_attn(cache, 0, q, 1, cfg.n_q_heads)
        want, want_lse, probs = ocs[0].attn(0, q[0], cfg.n_q_heads, want_probs=True)
        assert_attn_close(out[0], want, "splits=%d" % splits)
        np.testing.assert_allclose(lse[0], want_lse, rtol=1e-4, atol=1e-4)
        np.testing.assert_allclose(p2[0], (probs ** 2).sum(axis=1), rtol=2e-3)


def test_token_by_token_decode_appends_match_bulk_and_oracle():
    say("decode-style appends: 140 steps of T=1 on 3 sequences, 2 layers, mixed widths")
    B, T, Hq, Hkv = 3, 140, 6, 2
    bits = np.random.default_rng(5).choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    cache, ocs = build_both(B, T, Hq, Hkv, bits, seed=21, n_layers=2, max_context=256, chunk=1)
    for L in range(2):
        for s in range(B):
            assert_export_equals(cache, L, s, ocs[L])
    q = make_kv((B, Hq, 64), 22, outlier=False)
    for L in range(2):
        out, lse, _ = run_attn(cache, L, q, B, Hq)
        for s in range(B):
            want, want_lse, _ = ocs[L].attn(s, q[s], Hq)
            assert_attn_close(out[s], want, "layer %d seq %d" % (L, s))
            np.testing.assert_allclose(lse[s], want_lse, rtol=1e-4, atol=1e-4)


@pytest.mark.parametrize("T", [1, 2, 3, 64, 65, 255, 256, 257, 511, 513, 1030])
@pytest.mark.parametrize("width", [2, 4, 8, 16, 0])
def test_attention_lengths_around_block_and_page_edges(T, width):
    say("attention T=%d width=%s" % (T, width or "mixed"))
    B, Hq, Hkv = 2, 4, 4
    rng = np.random.default_rng(T * 7 + width)
    bits = np.full((B, T), width, np.uint8) if width else rng.choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    cache, ocs = build_both(B, T, Hq, Hkv, bits, seed=31 + T)
    q = make_kv((B, Hq, 64), 32 + T, outlier=False)
    out, lse, p2 = run_attn(cache, 0, q, B, Hq)
    for s in range(B):
        want, want_lse, probs = ocs[0].attn(s, q[s], Hq, want_probs=True)
        assert_attn_close(out[s], want, "seq %d" % s)
        np.testing.assert_allclose(lse[s], want_lse, rtol=1e-4, atol=1e-4)
        np.testing.assert_allclose(p2[s], (probs ** 2).sum(axis=1), rtol=2e-3)


@pytest.mark.parametrize("Hq,Hkv", [(9, 3), (15, 5), (32, 32), (8, 1)])
@pytest.mark.parametrize("waves", [1, 2, 4, 8])
def test_attention_head_layouts_wave_counts_and_splits(Hq, Hkv, waves):
    say("attention Hq=%d Hkv=%d waves=%d" % (Hq, Hkv, waves))
    B, T = 2, 700
    bits = np.random.default_rng(Hq + waves).choice([2, 4, 8, 16], (B, T), p=[0.5, 0.25, 0.15, 0.1]).astype(np.uint8)
    cache, ocs = build_both(B, T, Hq, Hkv, bits, seed=41)
    q = make_kv((B, Hq, 64), 42, outlier=False)
    for splits in (1, 2, 5):
        with tuning(attn_splits=splits, attn_waves=waves):
            out, _, _ = run_attn(cache, 0, q, B, Hq, want_aux=False)
        for s in range(B):
            want, _, _ = ocs[0].attn(s, q[s], Hq)
            assert_attn_close(out[s], want, "splits %d seq %d" % (splits, s))


def test_ragged_lengths_empty_sequence_and_seq_ids():
    say("ragged batch with an empty sequence and a permuted seq_ids list")
    Hq, Hkv, max_ctx = 6, 3, 512
    lens = [300, 0, 1, 129]
    B = len(lens)
    cache = kvq.Cache(1, B, Hq, Hkv, max_ctx)
    oc = OracleCache(B, Hkv)
    rng = np.random.default_rng(9)
    for s, n in enumerate(lens):
        if n == 0:
            continue
        bits = rng.choice([2, 4, 8, 16], (1, n)).astype(np.uint8)
        K, V = make_kv((1, n, Hkv, 64), 50 + s), make_kv((1, n, Hkv, 64), 60 + s)
        ids = torch.tensor([s], dtype=torch.int32, device=dev())
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), ids, 1, n)
        oc.append(s, K[0], V[0], bits[0])
    torch.cuda.synchronize()
    for s in range(B):
        assert_export_equals(cache, 0, s, oc)
    order = [3, 1, 0, 2]
    q = make_kv((B, Hq, 64), 70, outlier=False)
    ids = torch.tensor(order, dtype=torch.int32, device=dev())
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
    out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
    kvq.kvq_decode_attn(cache, 0, gpu_f16(q), ids, B, out, ws, lse, None)
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for i, s in enumerate(order):
        if lens[s] == 0:
            assert np.all(out[i] == 0) and np.all(np.isneginf(lse[i]))
            continue
        want, want_lse, _ = oc.attn(s, q[i], Hq)
        assert_attn_close(out[i], want, "slot %d seq %d" % (i, s))
        np.testing.assert_allclose(lse[i], want_lse, rtol=1e-4, atol=1e-4)


@pytest.mark.parametrize("mu", [2.0, 5.0, -3.0])
@pytest.mark.parametrize("width", [2, 4, 8, 0])
def test_queries_with_a_nonzero_mean_on_heavy_tailed_keys(mu, width):
    """The kernel reads a code as h = 1 + c/M and subtracts the constant part M * sum(q) afterwards, so its rounding error
    grows with |sum(q)|: queries ~ N(mu, 1) (sum q in the hundreds) on keys with Student-t channel scales, every width
    alone and the mix (width 0), against the same tolerance as everything else."""
    say("attention with q ~ N(%g, 1), width %s" % (mu, width or "mixed"))
    B, T, Hq, Hkv = 2, 900, 6, 2
    rng = np.random.default_rng(int(100 + 10 * mu + width))
    bits = (rng.choice([2, 4, 8, 16], (B, T), p=[0.4, 0.3, 0.2, 0.1]) if width == 0 else np.full((B, T), width)).astype(np.uint8)
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    oc = OracleCache(B, Hkv)
    t3 = np.abs(rng.standard_normal((Hkv, 64)) / np.sqrt((rng.standard_normal((3, Hkv, 64)) ** 2).sum(axis=0) / 3.0)).clip(0.1, 50.0)
    K = (rng.standard_normal((B, T, Hkv, 64)) * t3).astype(np.float16)
    V = (rng.standard_normal((B, T, Hkv, 64)) * t3[::-1]).astype(np.float16)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for b in range(B):
        oc.append(b, K[b], V[b], bits[b])
    q = (rng.standard_normal((B, Hq, 64)) + mu).astype(np.float16)
    for waves, splits in ((0, 0), (2, 1), (4, 3)):
        with tuning(attn_waves=waves, attn_splits=splits):
            out, lse, _ = run_attn(cache, 0, q, B, Hq)
        for b in range(B):
            want, want_lse, _ = oc.attn(b, q[b], Hq)
            assert_attn_close(out[b], want, "mu %g width %d seq %d (waves %d, splits %d)" % (mu, width, b, waves, splits))
            np.testing.assert_allclose(lse[b], want_lse, rtol=1e-4, atol=2e-4)


@pytest.mark.parametrize("B,fused", [(8, False), (16, False), (16, True), (64, False)])
def test_longest_first_launch_order_on_a_ragged_batch(B, fused):
    say("longest-first launch order, ragged batch of %d, fused=%s" % (B, fused))
    Hq, Hkv, max_ctx = 4, 2, 512
    rng = np.random.default_rng(100 + B)
    lens = rng.integers(0, 400, B)
    lens[1] = lens[5] = 77                                       # equal lengths: ranks break the tie by position
    lens[2] = 0
    cache = kvq.Cache(1, B, Hq, Hkv, max_ctx)
    oc = OracleCache(B, Hkv)
    for s_, n in enumerate(lens):
        if n == 0:
            continue
        bits = rng.choice([2, 4, 8, 16], (1, n)).astype(np.uint8)
        K, V = make_kv((1, n, Hkv, 64), 700 + s_), make_kv((1, n, Hkv, 64), 800 + s_)
        ids = torch.tensor([s_], dtype=torch.int32, device=dev())
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), ids, 1, n)
        oc.append(s_, K[0], V[0], bits[0])
    order = rng.permutation(B)
    ids = torch.from_numpy(order.astype(np.int32)).to(dev())
    q = make_kv((B, Hq, 64), 900, outlier=False)
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
    out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
    with tuning(attn_longest_first=1):
        if fused:
            kn, vn = make_kv((B, 1, Hkv, 64), 901), make_kv((B, 1, Hkv, 64), 902)
            nb = rng.choice([2, 4, 8, 16], B).astype(np.uint8)
            kvq.kvq_append_decode_attn(cache, 0, gpu_f16(kn), gpu_f16(vn), torch.from_numpy(nb).to(dev()), gpu_f16(q), ids, B, out, ws, lse, None)
            for i, s_ in enumerate(order):
                oc.append(s_, kn[i], vn[i], nb[i:i + 1])
        else:
            kvq.kvq_decode_attn(cache, 0, gpu_f16(q), ids, B, out, ws, lse, None)
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for i, s_ in enumerate(order):
        if len(oc.bits[s_]) == 0:
            assert np.all(out[i] == 0) and np.all(np.isneginf(lse[i]))
            continue
        want, want_lse, _ = oc.attn(s_, q[i], Hq)
        assert_attn_close(out[i], want, "slot %d seq %d" % (i, s_))
        np.testing.assert_allclose(lse[i], want_lse, rtol=1e-4, atol=1e-4)
    if fused:
        for s_ in range(B):
            assert_export_equals(cache, 0, s_, oc)


@pytest.mark.parametrize("waves", [0, 2, 8])
def test_launch_of_several_rounds_ragged_batch_both_range_rules(waves):
    """More workgroups than the device has places for (40 sequences x 32 query heads): the launch runs in rounds, takes its
    sequences longest first (ranks dealt to the XCDs in alternating direction) and cuts the units by the second set of unit
    costs; with 8 waves per workgroup and these short contexts the classes get whole waves, with 2 one cost range per wave."""
    say("several rounds, ragged batch of 40, %d waves per workgroup" % waves)
    B, Hq, Hkv, max_ctx = 40, 32, 4, 1024
    rng = np.random.default_rng(4200 + waves)
    lens = rng.integers(60, 700, B)
    lens[3] = lens[17] = 333
    cache = kvq.Cache(1, B, Hq, Hkv, max_ctx)
    oc = OracleCache(B, Hkv)
    for s_, n in enumerate(lens):
        bits = rng.choice([2, 4, 8, 16], (1, n), p=[0.7, 0.2, 0.08, 0.02]).astype(np.uint8)
        K, V = make_kv((1, n, Hkv, 64), 1700 + s_), make_kv((1, n, Hkv, 64), 1800 + s_)
        ids = torch.tensor([s_], dtype=torch.int32, device=dev())
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), ids, 1, n)
        oc.append(s_, K[0], V[0], bits[0])
    q = make_kv((B, Hq, 64), 1900, outlier=False)
    with tuning(attn_waves=waves):
        out, lse, _ = run_attn(cache, 0, q, B, Hq)
    for s_ in rng.choice(B, 10, replace=False):
        want, want_lse, _ = oc.attn(int(s_), q[s_], Hq)
        assert_attn_close(out[s_], want, "seq %d (%d tokens)" % (s_, lens[s_]))
        np.testing.assert_allclose(lse[s_], want_lse, rtol=1e-4, atol=1e-4)
    assert np.all(np.isfinite(out))


def test_degenerate_vectors_constant_tiny_huge_and_signed_zero():
    say("degenerate vectors: constant, sub-resolution, +-65504, signed zeros")
    B, T, Hq, Hkv = 1, 8, 2, 2
    K = make_kv((B, T, Hkv, 64), 80, outlier=False)
    V = make_kv((B, T, Hkv, 64), 81, outlier=False)
    K[0, 0] = np.float16(1.5)                                   # constant vector
    V[0, 0] = np.float16(-0.0)                                  # constant zero, negative sign
    K[0, 1] = 0.0
    K[0, 1, :, 3] = np.uint16(1).view(np.float16)               # range of one subnormal step
    K[0, 2, :, ::2] = np.float16(65504.0)
    K[0, 2, :, 1::2] = np.float16(-65504.0)                     # widest possible range
    V[0, 3] = np.abs(V[0, 3])
    V[0, 3, :, 5] = np.float16(-0.0)                            # minimum is a negative zero
    V[0, 3, :, 6] = np.float16(0.0)
    K[0, 4] = (np.random.default_rng(1).standard_normal((Hkv, 64)) * 1e-6).astype(np.float16)   # subnormal range
    for width in (2, 4, 8, 16):
        bits = np.full((B, T), width, np.uint8)
        cache = kvq.Cache(1, B, Hq, Hkv, T)
        oc = OracleCache(B, Hkv)
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
        oc.append(0, K[0], V[0], bits[0])
        assert_export_equals(cache, 0, 0, oc)


def tie_vectors(shape, seed):
    """fp16 vectors whose quotients (x - min) / scale sit on, or within a few ulp of, half-integers: each vector holds its
    minimum 0, a maximum that fixes an exactly representable scale, and otherwise values (k + 1/2) * scale nudged by
    0, +-1 or +-2 fp16 ulps; a second family uses scales that are NOT exact in fp16 (the stored scale is rounded)."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(shape[:-1]))
    out = np.zeros((n, 64), np.float16)
    for v in range(n):
        levels = (3, 15, 255)[v % 3]
        if v % 2 == 0:
            scale = np.float16(2.0 ** rng.integers(-6, 3))                 # exact: quotients are exact half-integers
        else:
            scale = np.float16(rng.uniform(0.01, 1.5))                      # max / levels rounds when stored
        k = rng.integers(0, levels, 64)
        x = ((k + 0.5) * np.float32(scale)).astype(np.float16)
        nudge = rng.integers(-2, 3, 64)
        x = (x.view(np.uint16).astype(np.int32) + nudge).astype(np.uint16).view(np.float16)
        x[0] = 0.0
        x[1] = np.float16(np.float32(scale) * levels)
        out[v] = x[rng.permutation(64)]
    return out.reshape(shape)


@pytest.mark.parametrize("T", [8, 100])          # the wave-per-vector kernel, then the lane-per-token bulk kernel
def test_quotients_on_and_next_to_rounding_ties_are_bit_exact(T):
    say("append with quotients on / next to ties, T=%d" % T)
    B, Hq, Hkv = 2, 4, 4
    K = tie_vectors((B, T, Hkv, 64), 300 + T)
    V = tie_vectors((B, T, Hkv, 64), 400 + T)
    bits = np.tile(np.array([2, 4, 8, 16, 8, 4, 2, 2], np.uint8), (B, (T + 7) // 8))[:, :T].copy()
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    oc = OracleCache(B, Hkv)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for b in range(B):
        oc.append(b, K[b], V[b], bits[b])
        assert_export_equals(cache, 0, b, oc)


def test_bulk_append_degenerate_vectors_and_all_layers_in_one_call():
    say("bulk append (T=70, layer=-1): constant, sub-resolution, +-65504, signed-zero vectors, ragged tile tail")
    B, T, Hq, Hkv, L = 2, 70, 2, 2, 3
    rng = np.random.default_rng(9)
    K = np.stack([make_kv((B, T, Hkv, 64), 500 + l, outlier=l % 2 == 0) for l in range(L)])
    V = np.stack([make_kv((B, T, Hkv, 64), 600 + l, outlier=False) for l in range(L)])
    K[:, 0, 0] = np.float16(1.5)
    V[:, 0, 0] = np.float16(-0.0)
    K[:, 0, 1] = 0.0
    K[:, 0, 1, :, 3] = np.uint16(1).view(np.float16)
    K[:, 1, 2, :, ::2] = np.float16(65504.0)
    K[:, 1, 2, :, 1::2] = np.float16(-65504.0)
    V[:, 1, 3] = np.abs(V[:, 1, 3])
    V[:, 1, 3, :, 5] = np.float16(-0.0)
    V[:, 1, 3, :, 6] = np.float16(0.0)
    K[:, 0, 69] = (rng.standard_normal((L, Hkv, 64)) * 1e-6).astype(np.float16)
    bits = rng.choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    bits[:, :4] = np.array([2, 4, 8, 16], np.uint8)
    cache = kvq.Cache(L, B, Hq, Hkv, T)
    kvq.kvq_append(cache, -1, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for l in range(L):
        oc = OracleCache(B, Hkv)
        for b in range(B):
            oc.append(b, K[l, b], V[l, b], bits[b])
            assert_export_equals(cache, l, b, oc)
    assert cache.status()[0] == 0


@pytest.mark.parametrize("stream_min", [1, 16, 65])
@pytest.mark.parametrize("pattern", ["iid", "runs", "one_class"])
def test_bulk_append_streaming_and_cached_stores_write_the_same_bytes(stream_min, pattern):
    say("bulk append, store kind by run length: stream_min=%d pattern=%s" % (stream_min, pattern))
    B, T, Hq, Hkv = 2, 333, 4, 4
    rng = np.random.default_rng(800 + stream_min)
    if pattern == "iid":
        bits = rng.choice([2, 4, 8, 16], (B, T), p=[0.5, 0.25, 0.15, 0.1]).astype(np.uint8)
    elif pattern == "runs":
        bits = np.repeat(rng.choice([2, 4, 8, 16], (B, T // 20 + 1)), 20, axis=1)[:, :T].astype(np.uint8)
    else:
        bits = np.full((B, T), 8, np.uint8)
    K, V = make_kv((B, T, Hkv, 64), 801), make_kv((B, T, Hkv, 64), 802, outlier=False)
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    oc = OracleCache(B, Hkv)
    with tuning(append_stream_min=stream_min):
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for s in range(B):
        oc.append(s, K[s], V[s], bits[s])
        assert_export_equals(cache, 0, s, oc)
    assert cache.status()[0] == 0


def test_student_t_heavy_tailed_channels_and_long_mixed_context():
    say("heavy-tailed channels, ctx 3000, mix 40/30/20/10, 15q/5kv")
    B, T, Hq, Hkv = 2, 3000, 15, 5
    rng = np.random.default_rng(90)
    mult = np.clip(np.abs(rng.standard_t(3, size=(Hkv, 64))), 0.1, 50)
    K = (rng.standard_normal((B, T, Hkv, 64)) * mult).astype(np.float16)
    V = (rng.standard_normal((B, T, Hkv, 64)) * mult).astype(np.float16)
    bits = rng.choice([2, 4, 8, 16], (B, T), p=[0.4, 0.3, 0.2, 0.1]).astype(np.uint8)
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    oc = OracleCache(B, Hkv)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for s in range(B):
        oc.append(s, K[s], V[s], bits[s])
        assert_export_equals(cache, 0, s, oc)
    q = make_kv((B, Hq, 64), 91, outlier=False)
    out, lse, _ = run_attn(cache, 0, q, B, Hq)
    for s in range(B):
        want, want_lse, _ = oc.attn(s, q[s], Hq)
        assert_attn_close(out[s], want, "seq %d" % s)


def test_peaked_attention_and_large_scores():
    say("peaked attention: one key aligned with q, scores up to ~+-60")
    B, T, Hq, Hkv = 1, 500, 4, 4
    K = make_kv((B, T, Hkv, 64), 100, outlier=False)
    V = make_kv((B, T, Hkv, 64), 101)
    q = make_kv((B, Hq, 64), 102, outlier=False, scale=3.0)
    K[0, 123] = (q[0] * 2.0).astype(np.float16)                 # head h's key 123 is parallel to its query
    bits = np.random.default_rng(103).choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    bits[0, 123] = 16
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    oc = OracleCache(B, Hkv)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    oc.append(0, K[0], V[0], bits[0])
    out, lse, p2 = run_attn(cache, 0, q, B, Hq)
    want, want_lse, probs = oc.attn(0, q[0], Hq, want_probs=True)
    assert probs.max() > 0.99
    assert_attn_close(out[0], want)
    np.testing.assert_allclose(lse[0], want_lse, rtol=1e-4)


def test_sticky_flags_context_full_pool_exhausted_bad_bits_never_fault():
    say("device-side conditions: context full, pool exhausted, invalid width")
    B, Hq, Hkv = 2, 2, 2
    cache = kvq.Cache(1, B, Hq, Hkv, 300, pool_pages=(1, 1, 1, 1))
    K, V = make_kv((B, 256, Hkv, 64), 110), make_kv((B, 256, Hkv, 64), 111)
    bits = np.full((B, 256), 4, np.uint8)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, 256)
    flags, free = cache.status()
    assert flags & kvq.FLAG_POOL_EXHAUSTED and free[1] == 0      # two sequences, one 4-bit page
    cache.reset()
    assert cache.status() == (0, [1, 1, 1, 1])
    bits[:, 0] = 3                                               # not a width
    kvq.kvq_append(cache, 0, gpu_f16(K[:1]), gpu_f16(V[:1]), torch.from_numpy(bits[:1]).to(dev()), None, 1, 256)
    assert cache.status()[0] & kvq.FLAG_BAD_BITS
    counts = cache.counts()
    assert int(counts[0, 3]) == 1 and int(counts[0, 1]) == 255   # the bad token went to the FP16 class
    kvq.kvq_append(cache, 0, gpu_f16(K[:1, :100]), gpu_f16(V[:1, :100]), torch.from_numpy(bits[:1, 1:101].copy()).to(dev()), None, 1, 100)
    assert cache.status()[0] & kvq.FLAG_CONTEXT_FULL             # 256 + 100 > 300: skipped
    assert int(cache.counts()[0, 4]) == 256


def test_free_seqs_returns_pages_and_sequences_can_be_reused():
    say("free_seqs / reuse")
    B, Hq, Hkv, T = 2, 2, 1, 600
    cache = kvq.Cache(1, B, Hq, Hkv, 1024, pool_pages=(4, 4, 4, 4))
    rng = np.random.default_rng(120)
    oc = OracleCache(B, Hkv)
    bits = rng.choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    K, V = make_kv((B, T, Hkv, 64), 121), make_kv((B, T, Hkv, 64), 122)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    free_before = cache.status()[1]
    cache.free_seqs(torch.tensor([0], dtype=torch.int32, device=dev()), 1)
    free_after = cache.status()[1]
    assert all(a >= b for a, b in zip(free_after, free_before)) and sum(free_after) > sum(free_before)
    assert int(cache.counts()[0, 4]) == 0
    K2, V2 = make_kv((1, T, Hkv, 64), 123), make_kv((1, T, Hkv, 64), 124)
    ids = torch.tensor([0], dtype=torch.int32, device=dev())
    kvq.kvq_append(cache, 0, gpu_f16(K2), gpu_f16(V2), torch.from_numpy(bits[1:2].copy()).to(dev()), ids, 1, T)
    oc.append(0, K2[0], V2[0], bits[1])
    oc.append(1, K[1], V[1], bits[1])
    assert_export_equals(cache, 0, 0, oc)
    assert_export_equals(cache, 0, 1, oc)
    assert cache.status()[0] == 0


def test_host_side_argument_checks_change_nothing():
    say("host-side argument validation")
    cache = kvq.Cache(2, 2, 4, 2, 256)
    K = gpu_f16(make_kv((2, 1, 2, 64), 1))
    bits = torch.full((2, 1), 4, dtype=torch.uint8, device=dev())
    with pytest.raises(kvq.KvqError):
        kvq.kvq_append(cache, 2, K, K, bits, None, 2, 1)          # layer out of range
    kvq.kvq_append(cache, 0, K, K, None, None, 2, 1)              # no bits: no bookkeeping, and nothing pending to write
    with pytest.raises(kvq.KvqError):
        kvq.kvq_append(cache, 0, K, K, bits, None, 3, 1)          # more sequences than slots
    with pytest.raises(kvq.KvqError):
        kvq.kvq_append(cache, 0, K, K, bits, None, 2, 257)        # T beyond max_context
    out = torch.zeros((2, 4, 64), dtype=torch.float32, device=dev())
    ws = torch.empty(16, dtype=torch.uint8, device=dev())
    with pytest.raises(kvq.KvqError):
        kvq.kvq_decode_attn(cache, 5, K, None, 2, out, ws)
    with tuning(attn_splits=4):
        with pytest.raises(kvq.KvqError):
            kvq.kvq_decode_attn(cache, 0, K, None, 2, out, ws)    # workspace too small for 4 splits
    with tuning(attn_splits=4):
        with pytest.raises(kvq.KvqError):                         # the fused call checks its workspace before it books the token
            kvq.kvq_append_decode_attn(cache, 0, K, K, bits.view(-1), K, None, 2, out, ws)
    assert int(cache.counts()[:, 4].sum()) == 0 and cache.status()[0] == 0
    with pytest.raises(kvq.KvqError):
        kvq.Cache(1, 1, 3, 2, 256)                                # Hq not a multiple of Hkv
    with pytest.raises(kvq.KvqError):
        kvq.Cache(1, 1, 2, 2, 256, head_dim=128)


def test_running_twice_gives_bitwise_identical_attention():
    say("determinism: two runs, identical bits")
    B, T, Hq, Hkv = 2, 2000, 8, 8
    bits = np.random.default_rng(130).choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    cache, _ = build_both(B, T, Hq, Hkv, bits, seed=131)
    q = make_kv((B, Hq, 64), 132, outlier=False)
    with tuning(attn_splits=3):
        a, _, _ = run_attn(cache, 0, q, B, Hq)
        b, _, _ = run_attn(cache, 0, q, B, Hq)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (9, 3)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 0), (3, 0), (1, 8), (2, 8), (1, 1)])
def test_fused_append_attention_equals_the_oracle_and_the_two_call_path(Hq, Hkv, splits, waves):
    say("fused append+attention Hq=%d Hkv=%d splits=%d waves=%d: decode steps from an empty cache and after a prefill" % (Hq, Hkv, splits, waves))
    B, L, T0, steps = 3, 2, 333, 70
    rng = np.random.default_rng(140 + Hq)
    for prefill_len in (0, T0):
        cache = kvq.Cache(L, B, Hq, Hkv, 512)
        ref = kvq.Cache(L, B, Hq, Hkv, 512)                       # same tokens through kvq_append + kvq_decode_attn
        ocs = [OracleCache(B, Hkv) for _ in range(L)]
        if prefill_len:
            bits = rng.choice([2, 4, 8, 16], (B, prefill_len)).astype(np.uint8)
            bt = torch.from_numpy(bits).to(dev())
            for l in range(L):
                K, V = make_kv((B, prefill_len, Hkv, 64), 150 + l), make_kv((B, prefill_len, Hkv, 64), 160 + l)
                for c in (cache, ref):
                    kvq.kvq_append(c, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, None, B, prefill_len)
                for s in range(B):
                    ocs[l].append(s, K[s], V[s], bits[s])
        ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
        for step in range(steps):
            sb = rng.choice([2, 4, 8, 16], (B, 1)).astype(np.uint8)
            bt = torch.from_numpy(sb).to(dev())
            for l in range(L):
                K, V = make_kv((B, 1, Hkv, 64), 1000 + 10 * step + l), make_kv((B, 1, Hkv, 64), 5000 + 10 * step + l)
                q = make_kv((B, Hq, 64), 9000 + 10 * step + l, outlier=False)
                out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
                lse = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
                p2 = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
                with tuning(attn_splits=splits, attn_waves=waves):
                    kvq.kvq_append_decode_attn(cache, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, gpu_f16(q), None, B,
                                               out, ws, lse, p2)
                for s in range(B):
                    ocs[l].append(s, K[s, 0:1].reshape(1, Hkv, 64), V[s, 0:1].reshape(1, Hkv, 64), sb[s])
                if step % 23 == 0 or step == steps - 1:
                    out2 = torch.zeros_like(out)
                    kvq.kvq_append(ref, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, None, B, 1)
                    with tuning(attn_splits=splits, attn_waves=waves):
                        kvq.kvq_decode_attn(ref, l, gpu_f16(q), None, B, out2, ws)
                    torch.cuda.synchronize()
                    o, o2 = out.cpu().numpy(), out2.cpu().numpy()
                    for s in range(B):
                        want, want_lse, probs = ocs[l].attn(s, q[s], Hq, want_probs=True)
                        assert_attn_close(o[s], want, "fused step %d layer %d seq %d" % (step, l, s))
                        assert_attn_close(o2[s], want, "two-call step %d layer %d seq %d" % (step, l, s))
                        np.testing.assert_allclose(lse.cpu().numpy()[s], want_lse, rtol=1e-4, atol=1e-4)
                        np.testing.assert_allclose(p2.cpu().numpy()[s], (probs ** 2).sum(axis=1), rtol=2e-3)
                else:
                    kvq.kvq_append(ref, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, None, B, 1)
        torch.cuda.synchronize()
        for l in range(L):
            for s in range(B):
                assert_export_equals(cache, l, s, ocs[l])         # what the fused kernel stored is bit-exact
        assert cache.status()[0] == 0


def test_cache_usage_reports_expected_bits_and_bytes_like_the_oracle_accounting():
    say("cache usage: E[b], stored bits per element, payload and page bytes")
    import oracle
    B, Hq, Hkv, L = 3, 6, 3, 2
    lens = [700, 0, 41]
    cache = kvq.Cache(L, B, Hq, Hkv, 1024)
    assert cache.usage()["expected_bits"] == 0.0 and cache.usage()["payload_bytes"] == 0
    rng = np.random.default_rng(61)
    all_bits = []
    for s_, n in enumerate(lens):
        if n == 0:
            continue
        bits = rng.choice([2, 4, 8, 16], (1, n), p=[0.5, 0.25, 0.15, 0.1]).astype(np.uint8)
        all_bits.append(bits[0])
        ids = torch.tensor([s_], dtype=torch.int32, device=dev())
        for l in range(L):
            K, V = make_kv((1, n, Hkv, 64), 50 + s_ + 10 * l), make_kv((1, n, Hkv, 64), 60 + s_ + 10 * l)
            kvq.kvq_append(cache, l, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()) if l == 0 else None, ids, 1, n)
    u = cache.usage()
    cat = np.concatenate(all_bits)
    eb, ef, nb = oracle.accounting(cat, Hkv, L)
    assert u["tokens"] == [int((cat == w).sum()) for w in (2, 4, 8, 16)]
    assert u["expected_bits"] == pytest.approx(eb, rel=1e-14) and u["effective_bits"] == pytest.approx(ef, rel=1e-14)
    assert u["payload_bytes"] == nb
    # pages: one per started 256 slots of a class and sequence; a page holds 256 tokens of every layer and kv-head
    pt = 256
    pages = [sum(-(-int((b == w).sum()) // pt) for b in all_bits) for w in (2, 4, 8, 16)]
    assert u["pages_in_use"] == pages
    assert u["page_bytes_in_use"] == sum(p * pt * per * Hkv * L for p, per in zip(pages, (40, 72, 136, 256)))
    assert u["page_bytes_in_use"] >= u["payload_bytes"]


def test_export_import_roundtrip_restores_a_cache_bit_for_bit():
    say("save / restore: export every (layer, sequence), import into a fresh cache, compare exports and attention")
    B, Hq, Hkv, L = 3, 6, 3, 2
    lens = [333, 0, 70]
    rng = np.random.default_rng(71)
    src = kvq.Cache(L, B, Hq, Hkv, 512)
    ocs = [OracleCache(B, Hkv) for _ in range(L)]
    for s_, n in enumerate(lens):
        if n == 0:
            continue
        bits = rng.choice([2, 4, 8, 16], (1, n)).astype(np.uint8)
        ids = torch.tensor([s_], dtype=torch.int32, device=dev())
        for l in range(L):
            K, V = make_kv((1, n, Hkv, 64), 150 + s_ + 10 * l), make_kv((1, n, Hkv, 64), 160 + s_ + 10 * l)
            kvq.kvq_append(src, l, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()) if l == 0 else None, ids, 1, n)
            ocs[l].append(s_, K[0], V[0], bits[0])
    # restore into another cache, sequences in another order and into other slots (0 -> 2, 2 -> 0)
    dst = kvq.Cache(L, B, Hq, Hkv, 512)
    place = {0: 2, 2: 0}
    for s_ in (2, 0):
        n = lens[s_]
        for l in range(L):
            bits_d, codes_d, meta_d = src.export(l, s_, n)
            kvq.kvq_cache_import(dst, l, place[s_], bits_d if l == 0 else None, codes_d, meta_d, n)
    torch.cuda.synchronize()
    assert dst.status()[0] == 0
    for l in range(L):
        for s_ in (0, 2):
            for x, y in zip(src.export(l, s_, lens[s_]), dst.export(l, place[s_], lens[s_])):
                assert torch.equal(x, y)
            # the restored sequence equals the oracle's canonical arrays, too
            oc = OracleCache(B, Hkv)
            oc.bits[place[s_]], oc.codes[place[s_]], oc.meta[place[s_]] = ocs[l].bits[s_], ocs[l].codes[s_], ocs[l].meta[s_]
            assert_export_equals(dst, l, place[s_], oc)
    # attention on the restored cache: bit for bit the original's
    q = make_kv((B, Hq, 64), 170, outlier=False)
    ws = torch.empty(kvq.kvq_decode_attn_workspace(src, B), dtype=torch.uint8, device=dev())
    for l in range(L):
        o1 = torch.zeros((B, Hq, 64), dtype=torch.float32, device=dev())
        o2 = torch.zeros_like(o1)
        kvq.kvq_decode_attn(src, l, gpu_f16(q), torch.tensor([0, 1, 2], dtype=torch.int32, device=dev()), B, o1, ws)
        kvq.kvq_decode_attn(dst, l, gpu_f16(q), torch.tensor([2, 1, 0], dtype=torch.int32, device=dev()), B, o2, ws)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)
    # a restored sequence keeps growing like any other
    K, V = make_kv((1, 1, Hkv, 64), 180), make_kv((1, 1, Hkv, 64), 181)
    one = torch.tensor([[8]], dtype=torch.uint8, device=dev())
    kvq.kvq_append(dst, 0, gpu_f16(K), gpu_f16(V), one, torch.tensor([2], dtype=torch.int32, device=dev()), 1, 1)
    assert int(dst.counts()[2, 4]) == lens[0] + 1
    with pytest.raises(kvq.KvqError):
        kvq.kvq_cache_import(dst, 0, 1, None, codes_d, meta_d, 5)        # layer 0 needs the widths
    with pytest.raises(kvq.KvqError):
        kvq.kvq_cache_import(dst, 0, 7, bits_d, codes_d, meta_d, 5)      # no such sequence slot
