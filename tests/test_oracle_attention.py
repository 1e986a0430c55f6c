"""Pins for the oracle's decode attention (paper Sec. 3.2: a = Softmax(q K^T / sqrt(d_k)) V over the cache)."""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle


def rand_f16(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


def cache_of(K, V, bits):
    """K, V fp16 [T,Hkv,64] -> canonical arrays via the oracle's append (pinned in test_oracle_fp16_quantizer)."""
    return oracle.append(K.view(np.uint16), V.view(np.uint16), np.asarray(bits, np.uint8))


def plain_attention(q, K, V, Hq):
    """Textbook attention in numpy fp64; K, V [T,Hkv,64] (any float dtype), q [Hq,64]; block-contiguous GQA."""
    T, Hkv, _ = K.shape
    g = Hq // Hkv
    Kx = np.repeat(K.astype(np.float64), g, axis=1)         # [T,Hq,64]: query head h reads kv-head h // g
    Vx = np.repeat(V.astype(np.float64), g, axis=1)
    s = np.einsum("hc,thc->ht", q.astype(np.float64), Kx) / 8.0
    p = scipy.special.softmax(s, axis=1)
    return np.einsum("ht,thc->hc", p, Vx), scipy.special.logsumexp(s, axis=1), p


def dequant_numpy(codes, meta, bits):
    """Independent numpy dequantizer for canonical arrays -> fp64 [T,Hkv,2,64]."""
    T, Hkv = codes.shape[:2]
    out = np.zeros((T, Hkv, 2, 64))
    for t in range(T):
        b = int(bits[t])
        for h in range(Hkv):
            for w in range(2):
                raw = codes[t, h, w]
                if b == 16:
                    out[t, h, w] = raw.view(np.float16).astype(np.float64)
                else:
                    stream = np.unpackbits(raw[: 8 * b], bitorder="little").reshape(64, b)
                    c = (stream * (1 << np.arange(b))).sum(axis=1)
                    sc = float(meta[t, h, w, 0:1].view(np.float16)[0])
                    zp = float(meta[t, h, w, 1:2].view(np.float16)[0])
                    out[t, h, w] = zp + c * sc
    return out


@pytest.mark.parametrize("T,Hq,Hkv", [(1, 4, 4), (7, 9, 3), (130, 15, 5), (257, 8, 8), (33, 6, 1)])
def test_all_fp16_cache_equals_plain_attention_on_the_original_tensors(T, Hq, Hkv):
    K, V, q = rand_f16((T, Hkv, 64), 1), rand_f16((T, Hkv, 64), 2), rand_f16((Hq, 64), 3)
    codes, meta = cache_of(K, V, [16] * T)
    out, lse, probs = oracle.decode_attn(q.view(np.uint16), [16] * T, codes, meta, Hq, want_probs=True)
    want, want_lse, want_p = plain_attention(q, K, V, Hq)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, want_lse, rtol=1e-12)
    np.testing.assert_allclose(probs, want_p, rtol=1e-11, atol=1e-15)


def test_all_fp16_cache_equals_torch_sdpa_fp64():
    T, Hq, Hkv = 96, 9, 3
    K, V, q = rand_f16((T, Hkv, 64), 4), rand_f16((T, Hkv, 64), 5), rand_f16((Hq, 64), 6)
    codes, meta = cache_of(K, V, [16] * T)
    out, _, _ = oracle.decode_attn(q.view(np.uint16), [16] * T, codes, meta, Hq)
    tq = torch.from_numpy(q.astype(np.float64)).reshape(1, Hq, 1, 64)
    tk = torch.from_numpy(K.astype(np.float64)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.from_numpy(V.astype(np.float64)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-12)


def test_mixed_precision_cache_equals_plain_attention_over_independently_dequantized_tensors():
    T, Hq, Hkv = 200, 9, 3
    K, V, q = rand_f16((T, Hkv, 64), 7, 2.0), rand_f16((T, Hkv, 64), 8, 2.0), rand_f16((Hq, 64), 9)
    bits = np.random.default_rng(10).choice([2, 4, 8, 16], T).astype(np.uint8)
    codes, meta = cache_of(K, V, bits)
    deq = dequant_numpy(codes, meta, bits)
    out, lse, probs = oracle.decode_attn(q.view(np.uint16), bits, codes, meta, Hq, want_probs=True)
    want, want_lse, want_p = plain_attention(q, deq[:, :, 0], deq[:, :, 1], Hq)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, want_lse, rtol=1e-12)
    np.testing.assert_allclose(probs.sum(axis=1), 1.0, rtol=1e-13)
    # and quantization actually changed something (the test is not vacuous)
    assert np.max(np.abs(deq[:, :, 0] - K.astype(np.float64))) > 1e-2


@pytest.mark.parametrize("b", [2, 4, 8, 16])
def test_single_token_context_returns_its_dequantized_value(b):
    K, V, q = rand_f16((1, 2, 64), 11), rand_f16((1, 2, 64), 12), rand_f16((4, 64), 13)
    codes, meta = cache_of(K, V, [b])
    out, lse, _ = oracle.decode_attn(q.view(np.uint16), [b], codes, meta, 4)
    deq = dequant_numpy(codes, meta, [b])
    for h in range(4):
        assert np.array_equal(out[h], deq[0, h // 2, 1])
        assert lse[h] == pytest.approx(float(q[h].astype(np.float64) @ deq[0, h // 2, 0]) / 8.0, rel=1e-13)


def test_equal_keys_give_the_mean_of_the_values():
    T = 37
    k0 = rand_f16((1, 1, 64), 14)
    K = np.repeat(k0, T, axis=0)
    V, q = rand_f16((T, 1, 64), 15), rand_f16((2, 64), 16)
    codes, meta = cache_of(K, V, [16] * T)
    out, _, probs = oracle.decode_attn(q.view(np.uint16), [16] * T, codes, meta, 2, want_probs=True)
    np.testing.assert_allclose(probs, 1.0 / T, rtol=1e-13)
    np.testing.assert_allclose(out, np.broadcast_to(V.astype(np.float64).mean(axis=0), (2, 64)), rtol=1e-12, atol=1e-14)


def test_one_dominant_key_selects_its_value():
    T, j = 50, 31
    q = np.zeros((1, 64), np.float16)
    q[0, 0] = 8.0
    K = rand_f16((T, 1, 64), 17, 0.1)
    K[:, 0, 0] = 0.0
    K[j, 0, 0] = 60.0                                   # score 60 vs 0 for the rest
    V = rand_f16((T, 1, 64), 18)
    codes, meta = cache_of(K, V, [16] * T)
    out, _, _ = oracle.decode_attn(q.view(np.uint16), [16] * T, codes, meta, 1)
    np.testing.assert_allclose(out[0], V[j, 0].astype(np.float64), atol=1e-20 + 50 * math.exp(-60) * 5)


def test_permuting_cached_tokens_leaves_the_output_unchanged():
    T, Hq, Hkv = 64, 4, 2
    K, V, q = rand_f16((T, Hkv, 64), 19), rand_f16((T, Hkv, 64), 20), rand_f16((Hq, 64), 21)
    bits = np.random.default_rng(22).choice([2, 4, 8, 16], T).astype(np.uint8)
    codes, meta = cache_of(K, V, bits)
    perm = np.random.default_rng(23).permutation(T)
    a, la, _ = oracle.decode_attn(q.view(np.uint16), bits, codes, meta, Hq)
    b, lb, _ = oracle.decode_attn(q.view(np.uint16), bits[perm], codes[perm], meta[perm], Hq)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(la, lb, rtol=1e-13)


@pytest.mark.parametrize("T", [1, 2, 3, 4])
def test_tiny_contexts_by_brute_force_scalar_arithmetic(T):
    Hq = Hkv = 1
    K, V, q = rand_f16((T, 1, 64), 24 + T), rand_f16((T, 1, 64), 34 + T), rand_f16((1, 64), 44)
    codes, meta = cache_of(K, V, [16] * T)
    out, lse, _ = oracle.decode_attn(q.view(np.uint16), [16] * T, codes, meta, Hq)
    s = [sum(float(q[0, c]) * float(K[j, 0, c]) for c in range(64)) / math.sqrt(64) for j in range(T)]
    e = [math.exp(x) for x in s]
    Z = sum(e)
    for c in range(64):
        want = sum(e[j] / Z * float(V[j, 0, c]) for j in range(T))
        assert out[0, c] == pytest.approx(want, rel=1e-12, abs=1e-14)
    assert lse[0] == pytest.approx(math.log(Z), rel=1e-12)


def test_grouped_query_heads_share_their_kv_head_block_contiguously():
    T, Hq, Hkv = 20, 6, 2
    K, V = rand_f16((T, Hkv, 64), 50), rand_f16((T, Hkv, 64), 51)
    q1 = rand_f16((1, 64), 52)
    q = np.repeat(q1, Hq, axis=0)                      # identical queries: outputs differ only through the kv-head
    codes, meta = cache_of(K, V, [8] * T)
    out, _, _ = oracle.decode_attn(q.view(np.uint16), [8] * T, codes, meta, Hq)
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[1], out[2])       # heads 0..2 -> kv-head 0
    assert np.array_equal(out[3], out[4]) and np.array_equal(out[4], out[5])       # heads 3..5 -> kv-head 1
    assert np.max(np.abs(out[0] - out[3])) > 1e-3


def test_batch_wrapper_equals_per_sequence_calls_and_reports_sum_of_squared_probabilities():
    B, L, Hq, Hkv = 3, 90, 6, 2
    lens = np.array([90, 1, 47], np.int32)
    rng = np.random.default_rng(60)
    q = rand_f16((B, Hq, 64), 61)
    bits = rng.choice([2, 4, 8, 16], (B, L)).astype(np.uint8)
    codes = np.zeros((B, L, Hkv, 2, 128), np.uint8)
    meta = np.zeros((B, L, Hkv, 2, 2), np.uint16)
    for b in range(B):
        K, V = rand_f16((L, Hkv, 64), 70 + b), rand_f16((L, Hkv, 64), 80 + b)
        codes[b], meta[b] = cache_of(K, V, bits[b])
    out, lse, p2, nthr = oracle.decode_attn_batch(q.view(np.uint16), bits, codes, meta, lens, Hq)
    assert nthr >= 1
    for b in range(B):
        n = lens[b]
        o1, l1, p = oracle.decode_attn(q[b].view(np.uint16), bits[b, :n], codes[b, :n], meta[b, :n], Hq, want_probs=True)
        np.testing.assert_allclose(out[b], o1, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lse[b], l1, rtol=1e-13)
        np.testing.assert_allclose(p2[b], (p ** 2).sum(axis=1), rtol=1e-12)
