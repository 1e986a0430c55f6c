"""GPU parity on seeded random shapes: batch, head layout, ragged lengths, width mixes (also single-class and
run-clustered), chunked appends, permuted sequence lists, forced wave counts / splits / launch order, both attention entry
points.  Every case is compared with the oracle: export bit for bit, attention within tolerance."""
import numpy as np
import pytest
import torch

from helpers import OracleCache, assert_attn_close, assert_export_equals, dev, tuning, gpu_f16, make_kv
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu


def random_bits(rng, n):
    kind = rng.integers(0, 4)
    if kind == 0:                                              # one class only
        return np.full(n, rng.choice([2, 4, 8, 16]), np.uint8)
    if kind == 1:                                              # runs
        out = np.empty(0, np.uint8)
        while len(out) < n:
            out = np.concatenate([out, np.full(rng.integers(1, 65), rng.choice([2, 4, 8, 16], p=[0.7, 0.2, 0.08, 0.02]), np.uint8)])
        return out[:n]
    p = rng.dirichlet(np.ones(4) * (0.3 if kind == 2 else 3.0))
    return rng.choice([2, 4, 8, 16], n, p=p).astype(np.uint8)


@pytest.mark.parametrize("case", list(range(24)) + [100, 101, 102, 103, 104, 105])
def test_random_case(case):
    rng = np.random.default_rng(9000 + case)
    long_ctx = case >= 100                                      # a few cases with thousands of tokens: many pages and units
    B = int(rng.choice([1, 2, 3, 8])) if long_ctx else int(rng.choice([1, 2, 3, 5, 8, 16]))
    Hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 1, 2, 3, 4, 8]))
    Hq = Hkv * G
    lens = rng.integers(0, 6001 if long_ctx else 701, B)
    if case % 5 == 0:
        lens[rng.integers(0, B)] = 0
    waves = int(rng.choice([0, 0, 1, 2, 3, 4, 8]))
    splits = int(rng.choice([0, 0, 1, 2, 5]))
    lf = int(rng.integers(0, 2))
    fused = bool(rng.integers(0, 2))
    block_min_T = (32, 512, 1 << 30)[case % 3]                 # which prefill writer takes the chunks of 32 tokens and more
    print("case %d: B=%d Hq=%d Hkv=%d lens=%s waves=%d splits=%d longest_first=%d fused=%s block writer from T=%d" %
          (case, B, Hq, Hkv, lens.tolist(), waves, splits, lf, fused, block_min_T), flush=True)
    max_ctx = 8192 if long_ctx else 1024
    cache = kvq.Cache(1, B, Hq, Hkv, max_ctx)
    oc = OracleCache(B, Hkv)
    for s in range(B):
        n, t0 = int(lens[s]), 0
        bits = random_bits(rng, n)
        while t0 < n:                                          # appended in random chunks: all three append kernels take part
            tc = int(min(n - t0, rng.choice([1, 7, 31, 32, 64, 100, 300] + ([1500, 2500] if long_ctx else []))))
            K = make_kv((1, tc, Hkv, 64), 10000 * case + 100 * s + t0, outlier=bool(rng.integers(0, 2)))
            V = make_kv((1, tc, Hkv, 64), 10000 * case + 100 * s + t0 + 50, outlier=False)
            ids = torch.tensor([s], dtype=torch.int32, device=dev())
            with tuning(append_block_min_T=block_min_T):
                kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits[None, t0:t0 + tc].copy()).to(dev()), ids, 1, tc)
            oc.append(s, K[0], V[0], bits[t0:t0 + tc])
            t0 += tc
    torch.cuda.synchronize()
    assert cache.status()[0] == 0
    for s in range(B):
        assert_export_equals(cache, 0, s, oc)
    order = rng.permutation(B)
    ids = torch.from_numpy(order.astype(np.int32)).to(dev())
    q = make_kv((B, Hq, 64), 777 + case, outlier=False, scale=float(rng.choice([0.3, 1.0, 3.0])))
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
    out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
    p2 = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
    with tuning(attn_waves=waves, attn_splits=splits, attn_longest_first=lf):
        if fused:
            kn, vn = make_kv((B, 1, Hkv, 64), 888 + case), make_kv((B, 1, Hkv, 64), 999 + case)
            nb = rng.choice([2, 4, 8, 16], B).astype(np.uint8)
            kvq.kvq_append_decode_attn(cache, 0, gpu_f16(kn), gpu_f16(vn), torch.from_numpy(nb).to(dev()), gpu_f16(q), ids, B,
                                       out, ws, lse, p2)
            for i, s in enumerate(order):
                oc.append(s, kn[i], vn[i], nb[i:i + 1])
        else:
            kvq.kvq_decode_attn(cache, 0, gpu_f16(q), ids, B, out, ws, lse, p2)
    torch.cuda.synchronize()
    out, lse, p2 = out.cpu().numpy(), lse.cpu().numpy(), p2.cpu().numpy()
    for i, s in enumerate(order):
        if len(oc.bits[s]) == 0:
            assert np.all(out[i] == 0) and np.all(np.isneginf(lse[i]))
            continue
        want, want_lse, probs = oc.attn(s, q[i], Hq, want_probs=True)
        assert_attn_close(out[i], want, "case %d slot %d seq %d" % (case, i, s))
        np.testing.assert_allclose(lse[i], want_lse, rtol=1e-4, atol=1e-4)
        np.testing.assert_allclose(p2[i], (probs ** 2).sum(axis=1), rtol=2e-3, atol=1e-9)
    if fused:
        for s in range(B):
            assert_export_equals(cache, 0, s, oc)
    assert cache.status()[0] == 0
