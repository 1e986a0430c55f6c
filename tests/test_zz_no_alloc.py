"""The allocation-free attention entry point against the workspace-taking one it is a variant of.

kvq_decode_attn_static keeps the split launch's partial results in a fixed array inside the library's device image.
Two calls in a row share that array, the second on a smaller input: nothing of the first call may leak into it.
"""
import numpy as np
import pytest
import torch

from helpers import ATOL, RTOL, OracleCache, assert_attn_close, dev, gpu_f16, make_kv, tuning
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def _build(B, T, Hq, Hkv, seed):
    rng = np.random.default_rng(seed)
    bits = rng.choice([2, 4, 8, 16], (B, T), p=[0.4, 0.3, 0.2, 0.1]).astype(np.uint8)
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    oc = OracleCache(B, Hkv)
    K, V = make_kv((B, T, Hkv, 64), seed + 1), make_kv((B, T, Hkv, 64), seed + 2)
    kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    for b in range(B):
        oc.append(b, K[b], V[b], bits[b])
    return cache, oc


def _both(cache, q16, B, Hq):
    d = dev()
    outs = []
    for static in (False, True):
        out = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=d)
        lse = torch.zeros((B, Hq), dtype=torch.float32, device=d)
        p2 = torch.zeros((B, Hq), dtype=torch.float32, device=d)
        if static:
            kvq.kvq_decode_attn_static(cache, 0, gpu_f16(q16), None, B, out, lse, p2)
        else:
            ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=d)
            kvq.kvq_decode_attn(cache, 0, gpu_f16(q16), None, B, out, ws, lse, p2)
        torch.cuda.synchronize()
        outs.append((out.cpu().numpy(), lse.cpu().numpy(), p2.cpu().numpy()))
    return outs


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    say("kvq_decode_attn_static: 6 sequences x 1500 tokens split 5 ways, then 2 sequences x 300 tokens split 3 ways")
    assert kvq.kvq_decode_attn_static_capacity() == 8 << 20
    for (B, T, Hq, Hkv, splits, seed) in ((6, 1500, 8, 2, 5, 31), (2, 300, 8, 2, 3, 37)):
        cache, oc = _build(B, T, Hq, Hkv, seed)
        q = make_kv((B, Hq, 64), seed + 3, outlier=False)
        with tuning(attn_splits=splits):                    # the split launch is the one that uses the scratch array
            (o_ws, l_ws, p_ws), (o_st, l_st, p_st) = _both(cache, q, B, Hq)
        assert np.all(np.isfinite(o_st))
        assert np.all(np.abs(o_st.astype(np.float64) - o_ws) <= ATOL + RTOL * np.abs(o_ws))
        np.testing.assert_allclose(l_st, l_ws, rtol=1e-4, atol=1e-4)
        np.testing.assert_allclose(p_st, p_ws, rtol=2e-3)
        assert np.array_equal(o_st, o_ws)                    # same kernels, same order of operations
        for b in range(B):                                    # and both against the oracle
            want, _, _ = oc.attn(b, q[b], Hq)
            assert_attn_close(o_st[b], want, "static scratch, seq %d" % b)
        cache.destroy()


def test_static_scratch_entry_point_rejects_launches_beyond_its_array():
    say("kvq_decode_attn_static: 64 sequences x 32 heads x 16 splits x 272 B > 8 MiB is refused before any launch")
    B, Hq, Hkv, T = 64, 32, 32, 64
    cache = kvq.Cache(1, B, Hq, Hkv, T)
    q = torch.zeros((B, Hq, 64), dtype=torch.float16, device=dev())
    out = torch.full((B, Hq, 64), 7.0, dtype=torch.float32, device=dev())
    with tuning(attn_splits=16):
        with pytest.raises(kvq.KvqError) as e:
            kvq.kvq_decode_attn_static(cache, 0, q, None, B, out)
    assert e.value.code == kvq.KVQ_ERR_CAPACITY and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                           # nothing was launched
    with tuning(attn_splits=15):                              # 64 x 32 x 15 x 272 B fits
        kvq.kvq_decode_attn_static(cache, 0, q, None, B, out)
    torch.cuda.synchronize()
    assert bool((out == 0.0).all())                           # empty sequences give zeros
    cache.destroy()


def test_static_scratch_entry_point_under_graph_capture_replays_like_the_eager_call():
    """What the entry point is for: a split launch (two kernels, the partial results in the library's own array) captured
    into a HIP graph and replayed several times, with eager work and synchronizations in between, every replay compared
    with the eager result on the inputs of that moment."""
    say("kvq_decode_attn_static captured in a graph: 3 sequences x 900 tokens, 4 splits, 4 replays on changing queries")
    B, T, Hq, Hkv = 3, 900, 8, 2
    cache, oc = _build(B, T, Hq, Hkv, 53)
    d = dev()
    q_dev = torch.zeros((B, Hq, 64), dtype=torch.float16, device=d)
    out_g = torch.zeros((B, Hq, 64), dtype=torch.float32, device=d)
    lse_g = torch.zeros((B, Hq), dtype=torch.float32, device=d)
    with tuning(attn_splits=4):
        kvq.kvq_decode_attn_static(cache, 0, q_dev, None, B, out_g, lse_g)       # warm-up outside the capture (first-use set-up)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            kvq.kvq_decode_attn_static(cache, 0, q_dev, None, B, out_g, lse_g)
        for rep in range(4):
            q = make_kv((B, Hq, 64), 600 + rep, outlier=False)
            q_dev.copy_(gpu_f16(q))
            g.replay()
            torch.cuda.synchronize()
            got, got_lse = out_g.cpu().numpy().copy(), lse_g.cpu().numpy().copy()
            out_e = torch.full((B, Hq, 64), float("nan"), dtype=torch.float32, device=d)
            lse_e = torch.zeros((B, Hq), dtype=torch.float32, device=d)
            kvq.kvq_decode_attn_static(cache, 0, q_dev, None, B, out_e, lse_e)   # eager work between the replays
            torch.cuda.synchronize()
            assert np.array_equal(got, out_e.cpu().numpy()) and np.array_equal(got_lse, lse_e.cpu().numpy()), "replay %d differs from the eager call" % rep
            for b in range(B):
                want, _, _ = oc.attn(b, q[b], Hq)
                assert_attn_close(got[b], want, "graph replay %d, seq %d" % (rep, b))
    cache.destroy()

