"""Shared plumbing of the GPU parity tests: moves seeded inputs to both sides and compares results.

No arithmetic of the method lives here.  The oracle is called with host copies of exactly the tensors the
HIP path received; no expected value ever comes from the HIP path.
"""
from __future__ import annotations

import os

import numpy as np
import torch

import oracle
from paper_2604_04722_amd import binding as kvq

ATOL, RTOL = 2e-3, 1e-3        # attention tolerance: |gpu - oracle| <= ATOL + RTOL*|oracle|


def dev():
    return torch.device("cuda")


def to_bits_u16(t: torch.Tensor) -> np.ndarray:
    """fp16 torch tensor -> uint16 numpy bit patterns (host)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def make_kv(shape, seed, outlier=True, scale=1.0):
    """fp16 tensor ~ N(0,1)*scale with four x10 channels (host numpy, float16)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape) * scale
    if outlier:
        ch = rng.permutation(64)[:4]
        x[..., ch] *= 10.0
    return x.astype(np.float16)


def gpu_f16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16)).view(torch.float16).to(dev())


class OracleCache:
    """Canonical arrays of one layer for B sequences, grown by oracle.append."""

    def __init__(self, B, Hkv):
        self.B, self.Hkv = B, Hkv
        self.bits = [np.zeros(0, np.uint8) for _ in range(B)]
        self.codes = [np.zeros((0, Hkv, 2, 128), np.uint8) for _ in range(B)]
        self.meta = [np.zeros((0, Hkv, 2, 2), np.uint16) for _ in range(B)]

    def append(self, seq, k16, v16, bits):
        c, m = oracle.append(k16.view(np.uint16), v16.view(np.uint16), bits)
        self.bits[seq] = np.concatenate([self.bits[seq], np.asarray(bits, np.uint8)])
        self.codes[seq] = np.concatenate([self.codes[seq], c])
        self.meta[seq] = np.concatenate([self.meta[seq], m])

    def attn(self, seq, q16, Hq, want_probs=False):
        return oracle.decode_attn(q16.view(np.uint16), self.bits[seq], self.codes[seq], self.meta[seq], Hq, want_probs)


def assert_export_equals(cache: kvq.Cache, layer: int, seq: int, oc: OracleCache):
    n = len(oc.bits[seq])
    bits, codes, meta = cache.export(layer, seq, max(n, 1))
    torch.cuda.synchronize()
    counts = cache.counts()
    assert int(counts[seq, 4]) == n, "length mismatch: gpu %d oracle %d" % (int(counts[seq, 4]), n)
    for c, w in enumerate((2, 4, 8, 16)):
        assert int(counts[seq, c]) == int((oc.bits[seq] == w).sum())
    if n == 0:
        return
    gb = bits.cpu().numpy()[:n]
    gc = codes.cpu().numpy()[:n]
    gm = meta.cpu().numpy().view(np.uint16)[:n]
    assert np.array_equal(gb, oc.bits[seq]), "bit widths differ"
    if not np.array_equal(gm, oc.meta[seq]):
        bad = np.argwhere(gm != oc.meta[seq])[0]
        raise AssertionError("scale/min differ first at (token, head, K|V, field) = %s: gpu %04x oracle %04x"
                             % (bad, gm[tuple(bad)], oc.meta[seq][tuple(bad)]))
    if not np.array_equal(gc, oc.codes[seq]):
        bad = np.argwhere(gc != oc.codes[seq])[0]
        raise AssertionError("packed codes differ first at (token, head, K|V, byte) = %s (b=%d)" % (bad, gb[bad[0]]))


def assert_attn_close(got: np.ndarray, want: np.ndarray, what=""):
    err = np.abs(got.astype(np.float64) - want)
    tol = ATOL + RTOL * np.abs(want)
    if not np.all(err <= tol):
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError("%s attention differs at %s: gpu %.6g oracle %.6g (|err| %.3g > tol %.3g); max abs err %.3g"
                             % (what, i, got[i], want[i], err[i], tol[i], err.max()))
    assert np.all(np.isfinite(got))


tuning = kvq.tuning            # context manager over the library's launch-shape table (forces a code path for one test)
