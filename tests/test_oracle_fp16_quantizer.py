"""Pins for the oracle's fp16 helpers and its quantizer Q_b (paper Sec. 3.7).

Nothing here compares the oracle with itself: every expected value is a closed form, a numpy
library conversion, a hand-derived case, or an independently written vectorised quantizer.
"""
import numpy as np
import pytest

import oracle


# --------------------------------------------------------------------------------------------
# binary16 <-> binary32
# --------------------------------------------------------------------------------------------

def test_f16_to_f32_all_65536_patterns_match_numpy():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.f16_to_f32_array(h)
    want = h.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_roundtrips_every_half():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = h.view(np.float16).astype(np.float32)
    ok = ~np.isnan(f)
    back = oracle.f32_to_f16_array(f)
    assert np.array_equal(back[ok], h[ok])


def test_f32_to_f16_matches_numpy_rne_on_random_ties_subnormals_overflow():
    rng = np.random.default_rng(7)
    parts = [
        rng.standard_normal(400_000).astype(np.float32) * 3.0,
        (rng.standard_normal(200_000) * 1e-6).astype(np.float32),          # fp16 subnormal range
        (rng.standard_normal(200_000) * 3e4).astype(np.float32),           # near overflow
        rng.integers(0, 2**32, 400_000, dtype=np.uint64).astype(np.uint32).view(np.float32),  # any bit pattern
    ]
    # exact ties: midpoints between consecutive halves (all finite positive halves and their negatives)
    h = np.arange(0, 0x7bff, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)       # exact in fp32 (12 significant bits)
    parts += [mid, -mid, np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e30, -65520.0, 0.0, -0.0], np.float32)]
    f = np.concatenate(parts)
    f = f[~np.isnan(f)]
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    got = oracle.f32_to_f16_array(f)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------------------------------
# helpers that are NOT the oracle
# --------------------------------------------------------------------------------------------

def unpack_codes(codes_bytes: np.ndarray, bits: int) -> np.ndarray:
    """Element i sits at bits [i*b, i*b+b) of the little-endian byte stream."""
    stream = np.unpackbits(codes_bytes[: 64 * bits // 8], bitorder="little")
    w = (1 << np.arange(bits)).astype(np.int64)
    return (stream.reshape(64, bits) * w).sum(axis=1)


def static_quantizer_numpy(x16: np.ndarray, bits: int):
    """A separately written, vectorised static b-bit min/max quantizer over the last axis (binary32 steps)."""
    levels = np.float32(2 ** bits - 1)
    x = x16.astype(np.float32)
    mn = x.min(axis=-1, keepdims=True)
    mx = x.max(axis=-1, keepdims=True)
    mn = np.where(mn == 0, np.float32(0.0), mn)                       # canonical +0
    scale_h = ((mx - mn) / levels).astype(np.float16)
    s = scale_h.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = (x - mn) / s
    code = np.clip(np.rint(t), 0, levels)
    code = np.where(s == 0, 0, code).astype(np.int64)
    return code, scale_h.view(np.uint16)[..., 0], mn.astype(np.float16).view(np.uint16)[..., 0]


def gen_vectors(kind: str, n: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    if kind == "normal":
        x = rng.standard_normal((n, 64))
    elif kind == "outlier":
        x = rng.standard_normal((n, 64))
        x[:, [3, 17, 40, 63]] *= 10.0
    elif kind == "student":
        x = rng.standard_normal((n, 64)) * np.clip(np.abs(rng.standard_t(3, size=(1, 64))), 0.1, 50)
    elif kind == "tiny":
        x = rng.standard_normal((n, 64)) * 1e-6
    elif kind == "huge":
        x = rng.uniform(-65504, 65504, size=(n, 64))
    else:
        raise ValueError(kind)
    return x.astype(np.float16)


# --------------------------------------------------------------------------------------------
# quantizer pins
# --------------------------------------------------------------------------------------------

@pytest.mark.parametrize("bits,grid_step", [(2, 1.0), (4, 1.0), (8, 1.0 / 16)])
def test_grid_lossless_inputs_give_exact_scale_codes_and_roundtrip(bits, grid_step):
    levels = 2 ** bits - 1
    rng = np.random.default_rng(bits)
    idx = rng.integers(0, levels + 1, 64)
    idx[5] = 0
    idx[9] = levels
    x = (idx * grid_step).astype(np.float16)
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), bits)
    assert np.float16(grid_step).view(np.uint16) == s
    assert z == 0
    assert np.array_equal(unpack_codes(codes, bits), idx)
    assert np.array_equal(oracle.dequantize_vec(codes, s, z, bits), x.astype(np.float64))


def test_hand_worked_two_bit_vector():
    # x = -1 + 0.5*k for k cycling 0,1,2,3: min -1, max 0.5, scale 0.5, codes k; four codes per byte: 0b11100100
    k = np.arange(64) % 4
    x = (-1.0 + 0.5 * k).astype(np.float16)
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 2)
    assert s == 0x3800 and z == 0xBC00                      # 0.5 and -1.0 in binary16
    assert np.all(codes[:16] == 0xE4) and np.all(codes[16:] == 0)


def test_hand_worked_four_and_eight_bit_packing_order():
    x = np.zeros(64, np.float16)
    x[0], x[1], x[2], x[63] = 15.0, 1.0, 2.0, 3.0           # scale 1 at 4 bits
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 4)
    assert (s, z) == (0x3C00, 0)
    assert codes[0] == 0x1F and codes[1] == 0x02 and codes[31] == 0x30 and np.all(codes[32:] == 0)
    x[0] = 255.0                                            # scale 1 at 8 bits
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 8)
    assert (s, z) == (0x3C00, 0)
    assert list(codes[:3]) == [255, 1, 2] and codes[63] == 3 and np.all(codes[64:] == 0)


def test_sixteen_bit_class_stores_the_fp16_patterns():
    x = gen_vectors("outlier", 1, 3)[0]
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 16)
    assert (s, z) == (0, 0)
    assert np.array_equal(codes.view(np.uint16), x.view(np.uint16))
    assert np.array_equal(oracle.dequantize_vec(codes, 0, 0, 16), x.astype(np.float64))


def test_rint_is_half_to_even():
    # min 0, max 3 -> scale 1 at 2 bits; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    x = np.zeros(64, np.float16)
    x[1], x[2], x[3], x[4] = 3.0, 0.5, 1.5, 2.5
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 2)
    c = unpack_codes(codes, 2)
    assert list(c[:5]) == [0, 3, 0, 2, 2]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_constant_vector_has_zero_scale_zero_codes_and_exact_dequant(bits):
    x = np.full(64, -2.71875, np.float16)
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), bits)
    assert s == 0 and z == x.view(np.uint16)[0] and not codes.any()
    assert np.array_equal(oracle.dequantize_vec(codes, s, z, bits), x.astype(np.float64))


def test_zero_minimum_of_either_sign_is_stored_as_plus_zero():
    x = np.abs(gen_vectors("normal", 1, 11)[0])
    x[7] = np.float16(-0.0)
    x[8] = np.float16(0.0)
    for order in (x, x[::-1].copy()):
        _, _, z = oracle.quantize_vec(order.view(np.uint16), 4)
        assert z == 0


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_vectors_of_zeros_of_any_sign_are_constant_vectors_with_scale_plus_zero(bits):
    # the constant-vector case: scale 0 (bit pattern +0), codes 0, zero-point +0, whatever the signs and their order
    pz, nz = np.float16(0.0), np.float16(-0.0)
    for x in (np.full(64, nz), np.full(64, pz), np.where(np.arange(64) % 2 == 0, nz, pz), np.where(np.arange(64) % 2 == 0, pz, nz)):
        x = x.astype(np.float16)
        codes, s, z = oracle.quantize_vec(x.view(np.uint16), bits)
        assert s == 0 and z == 0 and not codes.any()
    # a negative minimum with a zero maximum of either sign: same scale and codes for both signs
    a = -np.abs(gen_vectors("normal", 1, 12)[0])
    a[5] = pz
    b = a.copy()
    b[5] = nz
    ca, sa, za = oracle.quantize_vec(a.view(np.uint16), bits)
    cb, sb, zb = oracle.quantize_vec(b.view(np.uint16), bits)
    assert sa == sb and za == zb and np.array_equal(ca, cb)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("kind", ["normal", "outlier", "student", "huge"])
def test_min_gets_code_zero_max_gets_top_code_and_error_is_at_most_half_a_step(bits, kind):
    levels = 2 ** bits - 1
    X = gen_vectors(kind, 300, 100 + bits)
    for x in X:
        codes, s, z = oracle.quantize_vec(x.view(np.uint16), bits)
        c = unpack_codes(codes, bits)
        xf = x.astype(np.float64)
        assert c[np.argmin(xf)] == 0 and c[np.argmax(xf)] == levels
        assert np.uint16(z).view(np.float16) == x.min()
        step = float(np.uint16(s).view(np.float16))
        deq = oracle.dequantize_vec(codes, s, z, bits)
        # |x - x^| <= step/2, up to the binary32 rounding of (x-min)/step, wherever no clamping happened;
        # the scale is rounded to fp16, so the top of the range may clamp: there the error is at most
        # levels * |scale32 - scale_h| <= levels * 2^-11 * step on top of the half step.
        bound = step * (0.5 + levels * 2.0 ** -11) * (1 + 2.0 ** -20)
        assert np.max(np.abs(deq - xf)) <= bound


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_dequantize_is_zero_plus_code_times_scale(bits):
    rng = np.random.default_rng(bits)
    x = gen_vectors("outlier", 1, 5)[0]
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), bits)
    c = unpack_codes(codes, bits)
    want = float(np.uint16(z).view(np.float16)) + c.astype(np.float64) * float(np.uint16(s).view(np.float16))
    assert np.array_equal(oracle.dequantize_vec(codes, s, z, bits), want)
    # and for arbitrary codes / meta, not only ones a quantizer would produce
    raw = rng.integers(0, 256, 128, dtype=np.uint8)
    raw[64 * bits // 8:] = 0
    want = -3.5 + unpack_codes(raw, bits).astype(np.float64) * 0.0625
    assert np.array_equal(oracle.dequantize_vec(raw, 0x2C00, 0xC300, bits), want)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_every_byte_value_unpacks_and_repacks(bits):
    per = 8 // bits
    for byte in range(256):
        raw = np.zeros(128, np.uint8)
        raw[3] = byte
        want = [(byte >> (bits * i)) & (2 ** bits - 1) for i in range(per)]
        deq = oracle.dequantize_vec(raw, 0x3C00, 0, bits)          # scale 1, zero 0: dequant == code
        assert list(deq[3 * per: 4 * per].astype(int)) == want
        assert deq.sum() == sum(want)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("kind", ["normal", "outlier", "student", "tiny", "huge"])
def test_uniform_b_bit_adaptive_path_equals_a_static_b_bit_quantizer(bits, kind):
    T, Hkv = 40, 3
    K = gen_vectors(kind, T * Hkv, 1000 + bits).reshape(T, Hkv, 64)
    V = gen_vectors(kind, T * Hkv, 2000 + bits).reshape(T, Hkv, 64)
    codes, meta = oracle.append(K.view(np.uint16), V.view(np.uint16), np.full(T, bits, np.uint8))
    for which, X in ((0, K), (1, V)):
        c_want, s_want, z_want = static_quantizer_numpy(X, bits)
        assert np.array_equal(meta[:, :, which, 0], s_want)
        assert np.array_equal(meta[:, :, which, 1], z_want)
        for t in range(T):
            for h in range(Hkv):
                assert np.array_equal(unpack_codes(codes[t, h, which], bits), c_want[t, h])


def test_subnormal_range_and_sub_resolution_vectors():
    # range of two fp16 subnormal steps: at 2 bits the scale 2/3 step rounds to one step and the top element gets
    # code 2; at 4 and 8 bits (and at 2 bits for a range of one step) the scale underflows to zero: every code is 0
    x = np.zeros(64, np.float16)
    x[10] = np.uint16(2).view(np.float16)
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 2)
    assert s == 1 and unpack_codes(codes, 2)[10] == 2 and unpack_codes(codes, 2).sum() == 2
    for bits in (4, 8):
        codes, s, z = oracle.quantize_vec(x.view(np.uint16), bits)
        assert s == 0 and not codes.any()
    x[10] = np.uint16(1).view(np.float16)
    codes, s, z = oracle.quantize_vec(x.view(np.uint16), 2)
    assert s == 0 and not codes.any()


def test_append_rejects_unknown_bit_width_and_mixes_widths_per_token():
    K = gen_vectors("normal", 8, 1).reshape(4, 2, 64)
    V = gen_vectors("normal", 8, 2).reshape(4, 2, 64)
    with pytest.raises(ValueError):
        oracle.append(K.view(np.uint16), V.view(np.uint16), np.array([2, 3, 4, 8], np.uint8))
    bits = np.array([2, 16, 8, 4], np.uint8)
    codes, meta = oracle.append(K.view(np.uint16), V.view(np.uint16), bits)
    for t, b in enumerate(bits):
        for h in range(2):
            for which, X in ((0, K), (1, V)):
                c1, s1, z1 = oracle.quantize_vec(X[t, h].view(np.uint16), int(b))
                if b == 16:
                    assert np.array_equal(codes[t, h, which].view(np.uint16), X[t, h].view(np.uint16))
                else:
                    cw, sw, zw = static_quantizer_numpy(X[t, h][None], int(b))
                    assert np.array_equal(unpack_codes(codes[t, h, which], int(b)), cw[0])
                    assert meta[t, h, which, 0] == sw[0] and meta[t, h, which, 1] == zw[0]


def test_threaded_append_wrapper_equals_the_plain_loop():
    K = gen_vectors("outlier", 300 * 3, 77).reshape(300, 3, 64)
    V = gen_vectors("student", 300 * 3, 78).reshape(300, 3, 64)
    bits = np.random.default_rng(79).choice([2, 4, 8, 16], 300).astype(np.uint8)
    a = oracle.append(K.view(np.uint16), V.view(np.uint16), bits)
    b = oracle.append(K.view(np.uint16), V.view(np.uint16), bits, parallel=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_accounting_closed_forms_and_the_bytes_the_canonical_arrays_really_hold():
    # uniform widths: E[b] = b; stored bits per element = b + 32/64 for b < 16 (an fp16 scale and minimum per 64 codes)
    for b, eff, per in ((2, 2.5, 40), (4, 4.5, 72), (8, 8.5, 136), (16, 16.0, 256)):
        eb, ef, nb = oracle.accounting(np.full(1000, b, np.uint8), Hkv=3, layers=5)
        assert eb == b and ef == eff and nb == 1000 * per * 3 * 5
    # the 50/25/15/10 mix of the 1.7B-shaped workload: E[b] = 0.5*2 + 0.25*4 + 0.15*8 + 0.1*16 = 4.8
    bits = np.repeat(np.array([2, 4, 8, 16], np.uint8), [500, 250, 150, 100])
    eb, ef, nb = oracle.accounting(bits, Hkv=32, layers=24)
    assert eb == pytest.approx(4.8, rel=1e-15)
    assert nb == (500 * 40 + 250 * 72 + 150 * 136 + 100 * 256) * 32 * 24
    assert ef == pytest.approx(nb * 8 / (1000 * 32 * 24 * 128), rel=1e-15)
    # brute force against what the quantizer writes: count the bytes a canonical record actually uses
    rng = np.random.default_rng(8)
    bits = rng.choice([2, 4, 8, 16], 40).astype(np.uint8)
    K = gen_vectors("normal", 40 * 2, 31).reshape(40, 2, 64)
    V = gen_vectors("outlier", 40 * 2, 32).reshape(40, 2, 64)
    codes, meta = oracle.append(K.view(np.uint16), V.view(np.uint16), bits)
    used = 0
    for t in range(40):
        used += 2 * 2 * (64 * int(bits[t]) // 8) + (0 if bits[t] == 16 else 2 * 2 * 4)
        assert not codes[t, :, :, 64 * int(bits[t]) // 8:].any()            # nothing beyond the code bytes
    assert oracle.accounting(bits, Hkv=2, layers=1)[2] == used
    with pytest.raises(ValueError):
        oracle.accounting(np.array([2, 3], np.uint8), 1, 1)
