"""GPU parity of the two prefill writers behind kvq_append (many tokens per sequence): the kernel that takes 64 input
tokens per wavefront and the one that takes a block of 64 cache slots of one class.  Which one runs is a matter of
prompt length; here both are forced over the same cases, and every stored byte must equal the oracle's.

Every test prints what it is about to run (flushed) before touching the GPU.
"""
import numpy as np
import pytest
import torch

from helpers import OracleCache, assert_attn_close, assert_export_equals, dev, tuning, gpu_f16, make_kv
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu

KERNELS = {"tiles": 1 << 30, "blocks": 32}         # KVQ_APPEND_BLOCK_MIN_T: the block kernel from this T on


def say(*a):
    print(*a, flush=True)


def mix(rng, shape, p=(0.5, 0.25, 0.15, 0.1)):
    return rng.choice([2, 4, 8, 16], shape, p=p).astype(np.uint8)


@pytest.mark.parametrize("kernel", sorted(KERNELS))
@pytest.mark.parametrize("chunks", [(200, 37, 64, 399), (32, 33, 63, 65, 128), (1000,), (64, 1, 64, 5, 300)])
def test_chunked_prompts_start_every_class_at_any_slot(kernel, chunks):
    say("prefill writer %s: chunks %s, two layers" % (kernel, chunks))
    B, Hq, Hkv, n_layers = 3, 6, 3, 2
    total = sum(chunks)
    rng = np.random.default_rng(sum(chunks) + len(chunks))
    cache = kvq.Cache(n_layers, B, Hq, Hkv, total)
    ocs = [OracleCache(B, Hkv) for _ in range(n_layers)]
    with tuning(append_block_min_T=KERNELS[kernel]):
        for ci, T in enumerate(chunks):
            bits = mix(rng, (B, T))
            K = make_kv((n_layers, B, T, Hkv, 64), 900 + ci)
            V = make_kv((n_layers, B, T, Hkv, 64), 950 + ci, outlier=False)
            bt = torch.from_numpy(bits).to(dev())
            if ci % 2 == 0:                                     # all layers in one call, or layer by layer
                kvq.kvq_append(cache, -1, gpu_f16(K), gpu_f16(V), bt, None, B, T)
            else:
                for L in range(n_layers):
                    kvq.kvq_append(cache, L, gpu_f16(K[L]), gpu_f16(V[L]), bt if L == 0 else None, None, B, T)
            for L in range(n_layers):
                for s in range(B):
                    ocs[L].append(s, K[L, s], V[L, s], bits[s])
    torch.cuda.synchronize()
    for L in range(n_layers):
        for s in range(B):
            assert_export_equals(cache, L, s, ocs[L])
    assert cache.status()[0] == 0


@pytest.mark.parametrize("kernel", sorted(KERNELS))
@pytest.mark.parametrize("p", [(1, 0, 0, 0), (0, 0, 0, 1), (0, 0.5, 0, 0.5), (0.02, 0.02, 0.02, 0.94), (0.9, 0.1, 0, 0)])
def test_absent_and_rare_classes(kernel, p):
    say("prefill writer %s: class probabilities %s" % (kernel, p))
    B, T, Hq, Hkv = 2, 450, 2, 2
    rng = np.random.default_rng(int(1000 * p[0]) + 7)
    cache = kvq.Cache(1, B, Hq, Hkv, 2 * T)
    oc = OracleCache(B, Hkv)
    with tuning(append_block_min_T=KERNELS[kernel]):
        for ci in range(2):
            bits = mix(rng, (B, T), p)
            K, V = make_kv((B, T, Hkv, 64), 1000 + ci), make_kv((B, T, Hkv, 64), 1010 + ci)
            kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
            for s in range(B):
                oc.append(s, K[s], V[s], bits[s])
    for s in range(B):
        assert_export_equals(cache, 0, s, oc)
    assert cache.status()[0] == 0


@pytest.mark.parametrize("kernel", sorted(KERNELS))
def test_listed_sequences_a_skipped_one_and_attention_afterwards(kernel):
    say("prefill writer %s: seq_ids subset, one sequence without room (skipped, flagged), then attention" % kernel)
    Hq, Hkv, max_ctx, T = 4, 2, 400, 150
    cache = kvq.Cache(1, 4, Hq, Hkv, max_ctx)
    oc = OracleCache(4, Hkv)
    rng = np.random.default_rng(77)
    with tuning(append_block_min_T=KERNELS[kernel]):
        # sequence 1 is filled to 300 first: a further 150 do not fit
        bits = mix(rng, (1, 300))
        K, V = make_kv((1, 300, Hkv, 64), 1100), make_kv((1, 300, Hkv, 64), 1101)
        ids = torch.tensor([1], dtype=torch.int32, device=dev())
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), ids, 1, 300)
        oc.append(1, K[0], V[0], bits[0])
        order = [3, 1, 0]                                       # sequence 2 is not listed at all
        bits = mix(rng, (3, T))
        K, V = make_kv((3, T, Hkv, 64), 1102), make_kv((3, T, Hkv, 64), 1103)
        ids = torch.tensor(order, dtype=torch.int32, device=dev())
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), ids, 3, T)
    for i, s in enumerate(order):
        if s != 1:
            oc.append(s, K[i], V[i], bits[i])
    flags, _ = cache.status()
    assert flags == kvq.FLAG_CONTEXT_FULL
    assert [int(x) for x in cache.counts()[:, 4]] == [T, 300, 0, T]
    for s in range(4):
        assert_export_equals(cache, 0, s, oc)
    q = make_kv((4, Hq, 64), 1104, outlier=False)
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, 4), dtype=torch.uint8, device=dev())
    out = torch.full((4, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
    kvq.kvq_decode_attn(cache, 0, gpu_f16(q), None, 4, out, ws, None, None)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    for s in (0, 1, 3):
        assert_attn_close(out[s], oc.attn(s, q[s], Hq)[0], "seq %d" % s)
    assert np.all(out[2] == 0)


@pytest.mark.parametrize("kernel", sorted(KERNELS))
def test_an_empty_pool_sends_blocks_to_the_sink_page_without_a_fault(kernel):
    say("prefill writer %s: pools of one page, 700 tokens per sequence" % kernel)
    B, T, Hq, Hkv = 2, 700, 2, 2
    cache = kvq.Cache(1, B, Hq, Hkv, T, pool_pages=(1, 1, 1, 1))
    rng = np.random.default_rng(5)
    bits = mix(rng, (B, T), (0.25, 0.25, 0.25, 0.25))
    K, V = make_kv((B, T, Hkv, 64), 1200), make_kv((B, T, Hkv, 64), 1201)
    with tuning(append_block_min_T=KERNELS[kernel]):
        kvq.kvq_append(cache, 0, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()), None, B, T)
    flags, free = cache.status()
    assert flags == kvq.FLAG_POOL_EXHAUSTED and free == [0, 0, 0, 0]
    assert [int(x) for x in cache.counts()[:, 4]] == [T, T]
