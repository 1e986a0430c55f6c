"""A serving-style run: sequences come and go in a fixed set of slots over a tight page pool, every step appends one
token to each running sequence through one of the two attention entry points, and the oracle mirrors every slot."""
import numpy as np
import pytest
import torch

import oracle
from helpers import OracleCache, assert_attn_close, assert_export_equals, dev, gpu_f16, make_kv
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu


def test_sequences_come_and_go_in_a_tight_pool():
    print("continuous batching: 6 slots, 2 layers, 160 steps, page pool sized for the peak only", flush=True)
    B, L, Hq, Hkv, MAXC = 6, 2, 4, 2, 700
    rng = np.random.default_rng(2024)
    # a sequence holds at most MAXC tokens, i.e. at most 3 pages of 256 per class; the pool has 9 pages per class for
    # six slots (18 would be the worst case), so pages must come back when sequences end
    cache = kvq.Cache(L, B, Hq, Hkv, MAXC, pool_pages=(9, 9, 9, 9))
    ocs = [OracleCache(B, Hkv) for _ in range(L)]
    ws = torch.empty(kvq.kvq_decode_attn_workspace(cache, B), dtype=torch.uint8, device=dev())
    running = {}                                                   # slot -> tokens so far
    budget = {}                                                    # slot -> tokens at which the sequence ends
    mix = [0.45, 0.25, 0.2, 0.1]

    def start(slot, step):
        n = int(rng.choice([1, 5, 31, 32, 64, 100, 257]))         # both append kernels, block and page edges
        bits = rng.choice([2, 4, 8, 16], (1, n), p=mix).astype(np.uint8)
        ids = torch.tensor([slot], dtype=torch.int32, device=dev())
        for l in range(L):
            K, V = make_kv((1, n, Hkv, 64), 10_000 + 97 * step + 7 * slot + l), make_kv((1, n, Hkv, 64), 20_000 + 97 * step + 7 * slot + l)
            kvq.kvq_append(cache, l, gpu_f16(K), gpu_f16(V), torch.from_numpy(bits).to(dev()) if l == 0 else None, ids, 1, n)
            ocs[l].append(slot, K[0], V[0], bits[0])
        running[slot] = n
        budget[slot] = n + int(rng.integers(1, 120))

    def finish(slot):
        cache.free_seqs(torch.tensor([slot], dtype=torch.int32, device=dev()), 1)
        for l in range(L):
            ocs[l].bits[slot] = np.zeros(0, np.uint8)
            ocs[l].codes[slot] = np.zeros((0, Hkv, 2, 128), np.uint8)
            ocs[l].meta[slot] = np.zeros((0, Hkv, 2, 2), np.uint16)
        del running[slot], budget[slot]

    checked = 0
    for step in range(160):
        for slot in range(B):
            if slot not in running and rng.random() < 0.35:
                start(slot, step)
        for slot in [s for s in running if running[s] >= budget[s]]:
            finish(slot)
        act = sorted(running)
        if not act:
            continue
        # the launch-shape hint: the longest live sequence (on every other step a deliberately wrong value: results
        # must not depend on it)
        cache.set_length_hint(max(running.values()) + 1 if step % 2 else int(rng.integers(0, 3 * MAXC)))
        n = len(act)
        ids = torch.tensor(act, dtype=torch.int32, device=dev())
        sb = rng.choice([2, 4, 8, 16], (n, 1), p=mix).astype(np.uint8)
        bt = torch.from_numpy(sb).to(dev())
        fused = step % 3 != 0
        check = step % 8 == 0 or step >= 156
        for l in range(L):
            K, V = make_kv((n, 1, Hkv, 64), 30_000 + 3 * step + l), make_kv((n, 1, Hkv, 64), 40_000 + 3 * step + l)
            q = make_kv((n, Hq, 64), 50_000 + 3 * step + l, outlier=False)
            out = torch.full((n, Hq, 64), float("nan"), dtype=torch.float32, device=dev())
            if fused:
                kvq.kvq_append_decode_attn(cache, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, gpu_f16(q), ids, n, out, ws)
            else:
                kvq.kvq_append(cache, l, gpu_f16(K), gpu_f16(V), bt if l == 0 else None, ids, n, 1)
                kvq.kvq_decode_attn(cache, l, gpu_f16(q), ids, n, out, ws)
            for i, slot in enumerate(act):
                ocs[l].append(slot, K[i], V[i], sb[i])
            if check:
                torch.cuda.synchronize()
                o = out.cpu().numpy()
                for i, slot in enumerate(act):
                    want, _, _ = ocs[l].attn(slot, q[i], Hq)
                    assert_attn_close(o[i], want, "step %d layer %d slot %d (length %d)" % (step, l, slot, len(ocs[l].bits[slot])))
                    checked += 1
        for slot in act:
            running[slot] += 1
    flags, free = cache.status()
    assert flags == 0, "device flags %d raised (free pages %s)" % (flags, free)
    for l in range(L):
        for slot in range(B):
            assert_export_equals(cache, l, slot, ocs[l])
    # every page is either free or held by a running sequence
    for c, w in enumerate((2, 4, 8, 16)):
        held = sum(-(-int((ocs[0].bits[s] == w).sum()) // 256) for s in range(B))
        assert free[c] == 9 - held
    assert checked > 100
