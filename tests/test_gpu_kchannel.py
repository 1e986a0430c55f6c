"""GPU parity for the static per-channel key quantizer (a variant Q_b): export bit for bit, attention within the
tolerance, against the oracle's per-channel routines; decode steps through both attention entry points; the default
per-token mode after switching back."""
import numpy as np
import pytest
import torch

import oracle
from helpers import assert_attn_close, dev, tuning, gpu_f16, make_kv
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu


def calib(L, Hkv, seed, dead_channel=True):
    """per-channel minimum / range of N(0, sigma_c) keys with four x10 channels: +-3.5 sigma"""
    rng = np.random.default_rng(seed)
    sig = np.abs(rng.standard_normal((L, Hkv, 64))) * 0.5 + 0.5
    sig[..., [5, 21, 40, 63]] *= 10.0
    mn = (-3.5 * sig).astype(np.float16)
    rg = (7.0 * sig).astype(np.float16)
    if dead_channel:
        rg[..., 9] = 0.0                                          # step 0: code 0, k^ = min
    return sig, mn, rg


def keys(shape_T, sig_l, seed):
    rng = np.random.default_rng(seed)
    B, T, Hkv = shape_T
    return (rng.standard_normal((B, T, Hkv, 64)) * sig_l[None, None]).astype(np.float16)     # some values fall outside and clamp


class OracleKch:
    def __init__(self, B, Hkv, mn, rg):
        self.mn, self.rg = mn.view(np.uint16), rg.view(np.uint16)
        self.bits = [np.zeros(0, np.uint8) for _ in range(B)]
        self.codes = [np.zeros((0, Hkv, 2, 128), np.uint8) for _ in range(B)]
        self.meta = [np.zeros((0, Hkv, 2, 2), np.uint16) for _ in range(B)]

    def append(self, s, k16, v16, bits):
        c, m = oracle.append_kch(k16.view(np.uint16), v16.view(np.uint16), bits, self.mn, self.rg)
        self.bits[s] = np.concatenate([self.bits[s], np.asarray(bits, np.uint8)])
        self.codes[s] = np.concatenate([self.codes[s], c])
        self.meta[s] = np.concatenate([self.meta[s], m])

    def attn(self, s, q16, Hq):
        return oracle.decode_attn_kch(q16.view(np.uint16), self.bits[s], self.codes[s], self.meta[s], self.mn, self.rg, Hq)


def check_export(cache, layer, s, oc):
    n = len(oc.bits[s])
    b, c, m = cache.export(layer, s, max(n, 1))
    torch.cuda.synchronize()
    assert int(cache.counts()[s, 4]) == n
    if n == 0:
        return
    assert np.array_equal(b.cpu().numpy()[:n], oc.bits[s])
    assert np.array_equal(m.cpu().numpy().view(np.uint16)[:n], oc.meta[s]), "scale / minimum entries differ"
    got = c.cpu().numpy()[:n]
    if not np.array_equal(got, oc.codes[s]):
        bad = np.argwhere(got != oc.codes[s])[0]
        raise AssertionError("codes differ first at (token, head, K|V, byte) = %s" % bad)


@pytest.mark.parametrize("Hq,Hkv,waves,splits", [(8, 8, 0, 0), (9, 3, 0, 0), (4, 2, 8, 1), (6, 2, 1, 3), (4, 4, 3, 2)])
def test_per_channel_keys_prefill_then_decode_steps(Hq, Hkv, waves, splits):
    print("per-channel keys Hq=%d Hkv=%d waves=%d splits=%d" % (Hq, Hkv, waves, splits), flush=True)
    B, L, T0, steps = 3, 2, 400, 40
    sig, mn, rg = calib(L, Hkv, 50 + Hq)
    cache = kvq.Cache(L, B, Hq, Hkv, 512)
    cache.set_k_channel_quant(torch.from_numpy(mn.view(np.int16)).view(torch.float16).to(dev()),
                              torch.from_numpy(rg.view(np.int16)).view(torch.float16).to(dev()))
    ocs = [OracleKch(B, Hkv, mn[l], rg[l]) for l in range(L)]
    rng = np.random.default_rng(60 + Hq)
    lens = [T0, 0, 137]
    for s, n in enumerate(lens):
        if n == 0:
            continue
        bits = rng.choice([2, 4, 8, 16], (1, n), p=[0.4, 0.3, 0.2, 0.1]).astype(np.uint8)
        ids = torch.tensor([s], dtype=torch.int32, device=dev())
        for l in range(L):
            K = keys((1, n, Hkv), sig[l], 100 * s + l)
            V = make_kv((1, n, Hkv, 64), 200 * s + l)
            kvq.kvq_append(cache, l, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()) if l == 0 else None, ids, 1, n)
            ocs[l].append(s, K[0], V[0], bits[0])
    for l in range(L):
        for s in range(B):
            check_export(cache, l, s, ocs[l])
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
    for step in range(steps):
        sb = rng.choice([2, 4, 8, 16], (B, 1)).astype(np.uint8)
        bt = torch.from_numpy(sb).to(dev())
        fused = step % 2 == 0
        for l in range(L):
            K = keys((B, 1, Hkv), sig[l], 5000 + 10 * step + l)
            V = make_kv((B, 1, Hkv, 64), 7000 + 10 * step + l)
            q = make_kv((B, Hq, 64), 9000 + 10 * step + l, outlier=False)
            out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
            lse = torch.zeros((B, Hq), dtype=torch.float32, device=dev())
            with tuning(attn_waves=waves, attn_splits=splits):
                if fused:
                    kvq.kvq_append_decode_attn(cache, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, gpu_f16(q), None, B, out, ws, lse)
                else:
                    kvq.kvq_append(cache, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, None, B, 1)
                    kvq.kvq_decode_attn(cache, l, gpu_f16(q), None, B, out, ws, lse)
            for s in range(B):
                ocs[l].append(s, K[s], V[s], sb[s])
            if step % 13 == 0 or step == steps - 1:
                torch.cuda.synchronize()
                o, ls = out.cpu().numpy(), lse.cpu().numpy()
                for s in range(B):
                    want, want_lse = ocs[l].attn(s, q[s], Hq)
                    assert_attn_close(o[s], want, "step %d layer %d seq %d" % (step, l, s))
                    # the kernel folds each channel's step into the query and rounds the product to fp16 (half an ulp,
                    # 2^-12 relative, per term): with terms up to ~70 on the x10 channels and the 1/8 scale that is a few
                    # 1e-3 on a score, hence on the log-sum-exp; the output keeps the tolerance of the default path
                    np.testing.assert_allclose(ls[s], want_lse, rtol=0, atol=6e-3)
    for l in range(L):
        for s in range(B):
            check_export(cache, l, s, ocs[l])
    assert cache.status()[0] == 0


def test_switching_the_key_quantizer_needs_an_empty_cache_and_can_be_undone():
    print("per-channel keys: mode switch rules", flush=True)
    B, Hq, Hkv = 1, 2, 2
    sig, mn, rg = calib(1, Hkv, 7)
    tmn = torch.from_numpy(mn.view(np.int16)).view(torch.float16).to(dev())
    trg = torch.from_numpy(rg.view(np.int16)).view(torch.float16).to(dev())
    cache = kvq.Cache(1, B, Hq, Hkv, 256)
    K, V = make_kv((B, 5, Hkv, 64), 1), make_kv((B, 5, Hkv, 64), 2)
    bits = np.array([[2, 4, 8, 16, 2]], np.uint8)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, 5)
    with pytest.raises(kvq.KvqError):
        cache.set_k_channel_quant(tmn, trg)                       # not empty
    cache.reset()
    cache.set_k_channel_quant(tmn, trg)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, 5)
    oc = OracleKch(B, Hkv, mn[0], rg[0])
    oc.append(0, K[0], V[0], bits[0])
    check_export(cache, 0, 0, oc)
    cache.reset()
    cache.set_k_channel_quant(None, None)                         # back to the per-token quantizer
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, 5)
    codes, meta = oracle.append(K[0].view(np.uint16), V[0].view(np.uint16), bits[0])
    b, c, m = cache.export(0, 0, 5)
    assert np.array_equal(c.cpu().numpy(), codes) and np.array_equal(m.cpu().numpy().view(np.uint16), meta)


# the wave-per-vector kernel (T = 8), then both prefill writers (64 input tokens, or 64 slots of a class, per wavefront)
@pytest.mark.parametrize("T,block_min_T", [(8, 512), (100, 1 << 30), (333, 1 << 30), (100, 32), (333, 32)])
def test_per_channel_quotients_on_ties_out_of_range_values_and_all_layers_at_once(T, block_min_T):
    print("per-channel keys: ties, saturation, layer = -1, T=%d, block writer from T=%d" % (T, block_min_T), flush=True)
    B, L, Hq, Hkv = 2, 3, 4, 4
    rng = np.random.default_rng(900 + T)
    # ranges whose steps are exact in fp16 for every width: range = 255 * 15 * 2^-e  (divisible by 3, 15 and 255)
    e = rng.integers(4, 9, (L, Hkv, 64))
    rg = (3825.0 * 2.0 ** (-e.astype(np.float64))).astype(np.float16)
    rg[..., 11] = 0.0
    mn = (-rg.astype(np.float64) / 2).astype(np.float16)
    bits = rng.choice([2, 4, 8, 16], (B, T)).astype(np.uint8)
    K = np.zeros((L, B, T, Hkv, 64), np.float16)
    for l in range(L):
        for b in range(B):
            for t in range(T):
                w = int(bits[b, t])
                levels = (1 << w) - 1 if w < 16 else 255
                step = rg[l].astype(np.float64) / levels
                j = rng.integers(-2, levels + 3, (Hkv, 64))                       # some codes fall outside 0..levels
                frac = rng.choice([0.0, 0.5, 0.5 - 2.0 ** -9, 0.5 + 2.0 ** -9, 0.25], (Hkv, 64))
                K[l, b, t] = (mn[l].astype(np.float64) + step * (j + frac)).astype(np.float16)
    V = np.stack([make_kv((B, T, Hkv, 64), 910 + l, outlier=False) for l in range(L)])
    cache = kvq.Cache(L, B, Hq, Hkv, T)
    cache.set_k_channel_quant(torch.from_numpy(mn.view(np.int16)).view(torch.float16).to(dev()),
                              torch.from_numpy(rg.view(np.int16)).view(torch.float16).to(dev()))
    with tuning(append_block_min_T=block_min_T):
        kvq.kvq_append(cache, -1, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for l in range(L):
        oc = OracleKch(B, Hkv, mn[l], rg[l])
        for b in range(B):
            oc.append(b, K[l, b], V[l, b], bits[b])
            check_export(cache, l, b, oc)
    assert cache.status()[0] == 0
