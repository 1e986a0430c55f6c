"""ctypes front end of the CPU oracle (``kvq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  The product package never imports this module, and this module never
imports the product package.  All arithmetic lives in the C file; this file only marshals numpy
arrays, so that the C source stays the single thing a reader has to check against the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvq_oracle.c")
_LIB = os.path.join(_HERE, "libkvq_oracle.so")

D = 64          # head dimension
REC = 128       # bytes per packed-vector record in the canonical arrays
INDEX_TO_BIT = (2, 4, 8, 16)

# -O2 without any value-changing flag: the quantizer's binary32 steps must stay IEEE-exact.
GCC_FLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a few hundred ms).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *GCC_FLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.kvq_oracle_f16_to_f32.restype = ctypes.c_float
        _lib.kvq_oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.kvq_oracle_f32_to_f16.restype = ctypes.c_uint16
        _lib.kvq_oracle_f32_to_f16.argtypes = [ctypes.c_float]
        _lib.kvq_oracle_append.restype = ctypes.c_int
        _lib.kvq_oracle_append_parallel.restype = ctypes.c_int
        _lib.kvq_oracle_decode_attn_batch.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def f16_to_f32(h: int) -> float:
    return float(lib().kvq_oracle_f16_to_f32(int(h)))


def f32_to_f16(f: float) -> int:
    return int(lib().kvq_oracle_f32_to_f16(ctypes.c_float(f)))


def f32_to_f16_array(f) -> np.ndarray:
    a = _c(f, np.float32).ravel()
    out = np.zeros(a.shape[0], np.uint16)
    lib().kvq_oracle_f32_to_f16_array(_p(a), ctypes.c_int64(a.shape[0]), _p(out))
    return out


def f16_to_f32_array(h) -> np.ndarray:
    a = _c(h, np.uint16).ravel()
    out = np.zeros(a.shape[0], np.float32)
    lib().kvq_oracle_f16_to_f32_array(_p(a), ctypes.c_int64(a.shape[0]), _p(out))
    return out


def as_f16_bits(x) -> np.ndarray:
    """View an fp16 array (numpy float16, or anything convertible) as its uint16 bit patterns."""
    a = np.ascontiguousarray(x)
    if a.dtype != np.float16:
        a = a.astype(np.float16)
    return a.view(np.uint16)


def quantize_vec(x_bits, bits: int):
    """Q_b of one 64-vector.  x_bits: uint16[64].  Returns (codes uint8[128], scale_bits, zero_bits)."""
    x = _c(x_bits, np.uint16)
    assert x.shape == (D,)
    codes = np.zeros(REC, np.uint8)
    s = ctypes.c_uint16(0)
    z = ctypes.c_uint16(0)
    lib().kvq_oracle_quantize_vec(_p(x), ctypes.c_int(bits), _p(codes), ctypes.byref(s), ctypes.byref(z))
    return codes, int(s.value), int(z.value)


def dequantize_vec(codes, scale_bits: int, zero_bits: int, bits: int) -> np.ndarray:
    c = _c(codes, np.uint8)
    assert c.shape == (REC,)
    out = np.zeros(D, np.float64)
    lib().kvq_oracle_dequantize_vec(_p(c), ctypes.c_uint16(scale_bits), ctypes.c_uint16(zero_bits),
                                    ctypes.c_int(bits), _p(out))
    return out


def append(k_bits, v_bits, bits, parallel: bool = False):
    """Quantize T tokens of one sequence/layer.  k_bits, v_bits: uint16[T,Hkv,64]; bits: uint8[T].

    Returns (codes uint8[T,Hkv,2,128], meta uint16[T,Hkv,2,2]).
    """
    k = _c(k_bits, np.uint16)
    v = _c(v_bits, np.uint16)
    b = _c(bits, np.uint8)
    T, Hkv, d = k.shape
    assert d == D and v.shape == k.shape and b.shape == (T,)
    codes = np.zeros((T, Hkv, 2, REC), np.uint8)
    meta = np.zeros((T, Hkv, 2, 2), np.uint16)
    fn = lib().kvq_oracle_append_parallel if parallel else lib().kvq_oracle_append
    rc = fn(_p(k), _p(v), _p(b), ctypes.c_int64(T), ctypes.c_int(Hkv), _p(codes), _p(meta))
    if rc != 0:
        raise ValueError("bit width must be one of 2, 4, 8, 16")
    return codes, meta


def decode_attn(q_bits, bits, codes, meta, Hq: int, want_probs: bool = False):
    """Exact-softmax attention of one sequence over its canonical cache arrays.

    q_bits uint16[Hq,64]; bits uint8[len]; codes uint8[len,Hkv,2,128]; meta uint16[len,Hkv,2,2].
    Returns (out f64[Hq,64], lse f64[Hq], probs f64[Hq,len] or None).
    """
    q = _c(q_bits, np.uint16)
    b = _c(bits, np.uint8)
    c = _c(codes, np.uint8)
    m = _c(meta, np.uint16)
    ln = b.shape[0]
    Hkv = c.shape[1] if ln > 0 else (m.shape[1] if m.ndim == 4 else 1)
    assert q.shape == (Hq, D) and Hq % Hkv == 0
    out = np.zeros((Hq, D), np.float64)
    lse = np.zeros(Hq, np.float64)
    probs = np.zeros((Hq, max(ln, 1)), np.float64) if want_probs else None
    lib().kvq_oracle_decode_attn(_p(q), _p(b), _p(c), _p(m), ctypes.c_int64(ln), ctypes.c_int(Hq),
                                 ctypes.c_int(Hkv), _p(out), _p(lse), _p(probs), ctypes.c_int64(max(ln, 1)))
    if want_probs:
        probs = probs[:, :ln]
    return out, lse, probs


def decode_attn_batch(q_bits, bits, codes, meta, lens, Hq: int):
    """Batch form over fixed-stride arrays; OpenMP over (sequence, kv-head).

    q_bits uint16[B,Hq,64]; bits uint8[B,L]; codes uint8[B,L,Hkv,2,128]; meta uint16[B,L,Hkv,2,2]; lens int32[B].
    Returns (out f64[B,Hq,64], lse f64[B,Hq], sum_p2 f64[B,Hq], threads_used).
    """
    q = _c(q_bits, np.uint16)
    b = _c(bits, np.uint8)
    c = _c(codes, np.uint8)
    m = _c(meta, np.uint16)
    ln = _c(lens, np.int32)
    B, L = b.shape
    Hkv = c.shape[2]
    assert q.shape == (B, Hq, D) and c.shape == (B, L, Hkv, 2, REC) and m.shape == (B, L, Hkv, 2, 2)
    assert Hq % Hkv == 0 and ln.shape == (B,) and int(ln.max(initial=0)) <= L
    out = np.zeros((B, Hq, D), np.float64)
    lse = np.zeros((B, Hq), np.float64)
    p2 = np.zeros((B, Hq), np.float64)
    nthr = lib().kvq_oracle_decode_attn_batch(_p(q), _p(b), _p(c), _p(m), _p(ln), ctypes.c_int(B),
                                              ctypes.c_int64(L), ctypes.c_int(Hq), ctypes.c_int(Hkv),
                                              _p(out), _p(lse), _p(p2))
    return out, lse, p2, int(nthr)


def features(logits, ids, counts, N: int, Vobs: int, attn_probs, attn_len) -> np.ndarray:
    """s_t = [H, R, V, C] for n tokens.

    logits f32[n,vocab]; ids int32[n]; counts int64[vocab]; attn_probs f64[n,Hq,ld]; attn_len int32[n].
    Returns f32[n,4].
    """
    z = _c(logits, np.float32)
    i = _c(ids, np.int32)
    c = _c(counts, np.int64)
    a = _c(attn_probs, np.float64)
    ln = _c(attn_len, np.int32)
    n, vocab = z.shape
    _, Hq, ld = a.shape
    assert a.shape[0] == n and i.shape == (n,) and ln.shape == (n,) and c.shape == (vocab,)
    assert int(ln.max(initial=0)) <= ld and int(ln.min(initial=1)) >= 1
    out = np.zeros((n, 4), np.float32)
    lib().kvq_oracle_features(_p(z), ctypes.c_int64(n), ctypes.c_int64(vocab), _p(i), _p(c),
                              ctypes.c_int64(N), ctypes.c_int64(Vobs), _p(a), _p(ln), ctypes.c_int(Hq),
                              ctypes.c_int64(ld), _p(out))
    return out


def counts_update(ids, counts, N: int, Vobs: int):
    """Count the n tokens after they were scored.  Returns (counts', N', Vobs'); inputs are not modified."""
    i = _c(ids, np.int32)
    c = np.array(counts, dtype=np.int64, copy=True)
    tot = np.array([N, Vobs], np.int64)
    lib().kvq_oracle_counts_update(_p(i), ctypes.c_int64(i.shape[0]), _p(c), _p(tot))
    return c, int(tot[0]), int(tot[1])


def controller(feats, weights: Sequence[np.ndarray], biases: Sequence[np.ndarray]):
    """MLP forward + argmax + IndexToBit.  weights[l] f32[out_l,in_l] row-major; biases[l] f32[out_l].

    Returns (bits uint8[n], logits f64[n,n_out]).
    """
    f = _c(feats, np.float32)
    n = f.shape[0]
    Ws = [_c(w, np.float32) for w in weights]
    bs = [_c(b, np.float32) for b in biases]
    nl = len(Ws)
    dims = [Ws[0].shape[1]] + [w.shape[0] for w in Ws]
    assert f.shape == (n, dims[0]) and all(Ws[l].shape == (dims[l + 1], dims[l]) for l in range(nl))
    assert all(bs[l].shape == (dims[l + 1],) for l in range(nl)) and dims[-1] <= 4
    dims_a = np.asarray(dims, np.int32)
    Wp = (ctypes.c_void_p * nl)(*[w.ctypes.data for w in Ws])
    bp = (ctypes.c_void_p * nl)(*[b.ctypes.data for b in bs])
    bits = np.zeros(n, np.uint8)
    logits = np.zeros((n, dims[-1]), np.float64)
    lib().kvq_oracle_controller(_p(f), ctypes.c_int64(n), ctypes.c_int(nl), _p(dims_a), Wp, bp, _p(bits), _p(logits))
    return bits, logits


def accounting(bits, Hkv: int, layers: int):
    """(E[b], stored bits per element, payload bytes) of a cache whose tokens have the given widths."""
    b = _c(bits, np.uint8).ravel()
    eb, ef, nb = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_int64(0)
    rc = lib().kvq_oracle_accounting(_p(b), ctypes.c_int64(b.shape[0]), ctypes.c_int(Hkv), ctypes.c_int(layers),
                                     ctypes.byref(eb), ctypes.byref(ef), ctypes.byref(nb))
    if rc != 0:
        raise ValueError("illegal bit width")
    return eb.value, ef.value, nb.value


def rule_policy(feats, w, bias: float, thr):
    """(bits, score) of the stand-in rule-based policy: score = bias + w . s, class = number of thresholds exceeded."""
    f = _c(feats, np.float32)
    wv, tv = _c(w, np.float32), _c(thr, np.float32)
    assert f.ndim == 2 and f.shape[1] == 4 and wv.shape == (4,) and tv.shape == (3,) and np.all(np.diff(tv) >= 0)
    n = f.shape[0]
    bits = np.zeros(n, np.uint8)
    score = np.zeros(n, np.float64)
    lib().kvq_oracle_rule_policy(_p(f), ctypes.c_int64(n), _p(wv), ctypes.c_float(bias), _p(tv), _p(bits), _p(score))
    return bits, score


def kch_quantize_vec(x_bits, bits: int, kmin_bits, krange_bits) -> np.ndarray:
    """Static per-channel variant for one K vector: codes uint8[128] (canonical packing)."""
    x, mn, rg = _c(x_bits, np.uint16), _c(kmin_bits, np.uint16), _c(krange_bits, np.uint16)
    assert x.shape == (D,) and mn.shape == (D,) and rg.shape == (D,)
    codes = np.zeros(REC, np.uint8)
    lib().kvq_oracle_kch_quantize_vec(_p(x), ctypes.c_int(bits), _p(mn), _p(rg), _p(codes))
    return codes


def kch_dequantize_vec(codes, bits: int, kmin_bits, krange_bits) -> np.ndarray:
    c, mn, rg = _c(codes, np.uint8), _c(kmin_bits, np.uint16), _c(krange_bits, np.uint16)
    out = np.zeros(D, np.float64)
    lib().kvq_oracle_kch_dequantize_vec(_p(c), ctypes.c_int(bits), _p(mn), _p(rg), _p(out))
    return out


def append_kch(k_bits, v_bits, bits, kmin_bits, krange_bits):
    """append() with the per-channel variant for K; kmin / krange are uint16 [Hkv, 64]."""
    k, v, b = _c(k_bits, np.uint16), _c(v_bits, np.uint16), _c(bits, np.uint8)
    mn, rg = _c(kmin_bits, np.uint16), _c(krange_bits, np.uint16)
    T, Hkv, d = k.shape
    assert d == D and v.shape == k.shape and b.shape == (T,) and mn.shape == (Hkv, D) and rg.shape == (Hkv, D)
    codes = np.zeros((T, Hkv, 2, REC), np.uint8)
    meta = np.zeros((T, Hkv, 2, 2), np.uint16)
    lib().kvq_oracle_append_kch.restype = ctypes.c_int
    rc = lib().kvq_oracle_append_kch(_p(k), _p(v), _p(b), ctypes.c_int64(T), ctypes.c_int(Hkv), _p(mn), _p(rg), _p(codes), _p(meta))
    if rc != 0:
        raise ValueError("illegal bit width")
    return codes, meta


def decode_attn_kch(q_bits, bits, codes, meta, kmin_bits, krange_bits, Hq: int):
    """decode_attn() over a cache whose keys use the per-channel variant.  Returns (out [Hq,64], lse [Hq])."""
    q, b, c, m = _c(q_bits, np.uint16), _c(bits, np.uint8), _c(codes, np.uint8), _c(meta, np.uint16)
    mn, rg = _c(kmin_bits, np.uint16), _c(krange_bits, np.uint16)
    n = b.shape[0]
    Hkv = c.shape[1] if n else mn.shape[0]
    out = np.zeros((Hq, D), np.float64)
    lse = np.zeros(Hq, np.float64)
    lib().kvq_oracle_decode_attn_kch(_p(q), _p(b), _p(c), _p(m), _p(mn), _p(rg), ctypes.c_int64(n), ctypes.c_int(Hq),
                                     ctypes.c_int(Hkv), _p(out), _p(lse))
    return out, lse
