"""Pins of the oracle's static per-channel key quantizer (a variant Q_b; the paper leaves Q_b open in Sec. 3.7) and of
attention over such a cache.  Nothing compares the oracle with itself: closed forms, a separately written vectorised
numpy quantizer, hand cases, and plain fp64 attention on explicitly dequantized keys."""
import numpy as np
import pytest

import oracle

H16 = lambda a: np.asarray(a, np.float16).view(np.uint16)


def unpack_codes(codes_bytes, bits):
    stream = np.unpackbits(codes_bytes[: 64 * bits // 8], bitorder="little")
    w = (1 << np.arange(bits)).astype(np.int64)
    return (stream.reshape(64, bits) * w).sum(axis=1)


def numpy_kch(x16, bits, mn16, rg16):
    levels = np.float32(2 ** bits - 1)
    step = (rg16.astype(np.float32) / levels).astype(np.float16).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = (x16.astype(np.float32) - mn16.astype(np.float32)) / step
    code = np.where(step == 0, 0, np.clip(np.rint(t), 0, levels)).astype(np.int64)
    return code, mn16.astype(np.float64) + code * step.astype(np.float64)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_grid_points_come_back_exactly_and_out_of_range_values_clamp(bits):
    levels = 2 ** bits - 1
    rng = np.random.default_rng(bits)
    mn = (rng.integers(-8, 8, 64) * 0.5).astype(np.float16)
    step = np.float16(2.0) ** rng.integers(-3, 2, 64)                 # exact powers of two
    rg = (step.astype(np.float32) * levels).astype(np.float16)        # exactly representable: levels < 2048
    k = rng.integers(0, levels + 1, 64)
    x = (mn.astype(np.float32) + k * step.astype(np.float32)).astype(np.float16)
    codes = oracle.kch_quantize_vec(H16(x), bits, H16(mn), H16(rg))
    assert np.array_equal(unpack_codes(codes, bits), k)
    assert np.array_equal(oracle.kch_dequantize_vec(codes, bits, H16(mn), H16(rg)), x.astype(np.float64))
    # below the minimum -> code 0, above the top -> code levels
    lo = (mn.astype(np.float32) - 3.0).astype(np.float16)
    hi = (mn.astype(np.float32) + rg.astype(np.float32) + 5.0).astype(np.float16)
    assert not unpack_codes(oracle.kch_quantize_vec(H16(lo), bits, H16(mn), H16(rg)), bits).any()
    assert np.all(unpack_codes(oracle.kch_quantize_vec(H16(hi), bits, H16(mn), H16(rg)), bits) == levels)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_equals_a_vectorised_numpy_quantizer_and_errs_by_at_most_half_a_step_inside_the_range(bits):
    rng = np.random.default_rng(10 + bits)
    sig = np.abs(rng.standard_normal(64)) + 0.2
    sig[[3, 40]] *= 10
    mn = (-3.0 * sig).astype(np.float16)
    rg = (6.0 * sig).astype(np.float16)
    rg[7] = 0.0                                                        # a dead channel: step 0, code 0, k^ = min
    for _ in range(50):
        x = (rng.standard_normal(64) * sig).astype(np.float16)
        codes = oracle.kch_quantize_vec(H16(x), bits, H16(mn), H16(rg))
        want_code, want_deq = numpy_kch(x, bits, mn, rg)
        assert np.array_equal(unpack_codes(codes, bits), want_code)
        deq = oracle.kch_dequantize_vec(codes, bits, H16(mn), H16(rg))
        np.testing.assert_allclose(deq, want_deq, rtol=0, atol=0)
        step = (rg.astype(np.float32) / np.float32(2 ** bits - 1)).astype(np.float16).astype(np.float64)
        inside = (x.astype(np.float64) >= mn.astype(np.float64)) & (x.astype(np.float64) <= mn.astype(np.float64) + step * (2 ** bits - 1))
        assert np.all(np.abs(deq - x.astype(np.float64))[inside] <= 0.5 * step[inside] * (1 + 1e-6) + 1e-12)
        assert deq[7] == float(mn[7])


def test_sixteen_bit_tokens_and_values_are_untouched_by_the_variant():
    rng = np.random.default_rng(3)
    K = rng.standard_normal((5, 2, 64)).astype(np.float16)
    V = rng.standard_normal((5, 2, 64)).astype(np.float16)
    bits = np.array([16, 2, 16, 8, 4], np.uint8)
    mn = np.full((2, 64), -4.0, np.float16)
    rg = np.full((2, 64), 8.0, np.float16)
    codes, meta = oracle.append_kch(K.view(np.uint16), V.view(np.uint16), bits, H16(mn), H16(rg))
    c0, m0 = oracle.append(K.view(np.uint16), V.view(np.uint16), bits)
    assert np.array_equal(codes[:, :, 1], c0[:, :, 1]) and np.array_equal(meta[:, :, 1], m0[:, :, 1])     # V identical
    assert np.array_equal(codes[[0, 2], :, 0], c0[[0, 2], :, 0])                                            # FP16 K identical
    assert not meta[:, :, 0].any()                                                                          # no per-token K meta
    with pytest.raises(ValueError):
        oracle.append_kch(K.view(np.uint16), V.view(np.uint16), np.array([2, 3, 4, 8, 16], np.uint8), H16(mn), H16(rg))


def test_attention_equals_plain_fp64_attention_on_the_dequantized_keys_and_values():
    rng = np.random.default_rng(4)
    T, Hq, Hkv = 90, 6, 2
    K = (rng.standard_normal((T, Hkv, 64)) * 1.5).astype(np.float16)
    V = rng.standard_normal((T, Hkv, 64)).astype(np.float16)
    q = rng.standard_normal((Hq, 64)).astype(np.float16)
    bits = rng.choice([2, 4, 8, 16], T).astype(np.uint8)
    mn = np.full((Hkv, 64), -5.0, np.float16)
    rg = np.full((Hkv, 64), 10.0, np.float16)
    codes, meta = oracle.append_kch(K.view(np.uint16), V.view(np.uint16), bits, H16(mn), H16(rg))
    out, lse = oracle.decode_attn_kch(q.view(np.uint16), bits, codes, meta, H16(mn), H16(rg), Hq)
    Kh = np.stack([[oracle.kch_dequantize_vec(codes[t, h, 0], int(bits[t]), H16(mn[h]), H16(rg[h])) for h in range(Hkv)] for t in range(T)])
    Vh = np.stack([[oracle.dequantize_vec(codes[t, h, 1], int(meta[t, h, 1, 0]), int(meta[t, h, 1, 1]), int(bits[t])) for h in range(Hkv)] for t in range(T)])
    for h in range(Hq):
        kvh = h // (Hq // Hkv)
        s = Kh[:, kvh] @ q[h].astype(np.float64) / 8.0
        p = np.exp(s - s.max())
        p /= p.sum()
        np.testing.assert_allclose(out[h], p @ Vh[:, kvh], rtol=1e-12, atol=1e-14)
        assert lse[h] == pytest.approx(s.max() + np.log(np.exp(s - s.max()).sum()), rel=1e-13)
    # all tokens at 16 bits: the variant changes nothing at all
    b16 = np.full(T, 16, np.uint8)
    c1, m1 = oracle.append_kch(K.view(np.uint16), V.view(np.uint16), b16, H16(mn), H16(rg))
    o1, l1 = oracle.decode_attn_kch(q.view(np.uint16), b16, c1, m1, H16(mn), H16(rg), Hq)
    o2, l2, _ = oracle.decode_attn(q.view(np.uint16), b16, c1, m1, Hq)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
