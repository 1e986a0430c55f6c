"""GPU: one decode step (front end + fused append/attention per layer) captured as a HIP graph replays to the same
cache state and outputs as the eager calls.  The library's hot-path entry points only launch kernels, so a caller may
capture them; the replays here are separated by eager work and synchronizations."""
import numpy as np
import pytest
import torch

from helpers import dev
from paper_2604_04722_amd import binding as kvq
import benchprobe
import workloads as wl

pytestmark = pytest.mark.gpu


def test_graph_replay_of_a_decode_step_equals_the_eager_step():
    print("graph replay of a decode step", flush=True)
    d = dev()
    B, Hq, Hkv, L, vocab = 4, 6, 2, 3, 4096
    Ws, bs = wl.calibrated_mlp(wl.CONFIGS[4])
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    g = torch.Generator(device="cpu").manual_seed(5)
    # prefill both caches with the same 300 tokens
    T0 = 300
    K0 = torch.randn((L, B, T0, Hkv, 64), generator=g).to(torch.float16).to(d)
    V0 = torch.randn((L, B, T0, Hkv, 64), generator=g).to(torch.float16).to(d)
    bits0 = torch.from_numpy(np.random.default_rng(6).choice([2, 4, 8, 16], (B, T0)).astype(np.uint8)).to(d)
    caches = [kvq.Cache(L, B, Hq, Hkv, 512) for _ in range(2)]
    for c in caches:
        for l in range(L):
            kvq.kvq_append(c, l, K0[l], V0[l], bits0 if l == 0 else None, None, B, T0)
    # static per-step inputs (a graph replays fixed addresses; the caller refreshes their contents between replays)
    logits = torch.empty((B, vocab), dtype=torch.float32, device=d)
    ids = torch.empty(B, dtype=torch.int32, device=d)
    lens = torch.empty(B, dtype=torch.int32, device=d)
    k = torch.empty((L, B, 1, Hkv, 64), dtype=torch.float16, device=d)
    v = torch.empty_like(k)
    q = torch.empty((L, B, Hq, 64), dtype=torch.float16, device=d)
    state = []
    for c in caches:
        counts = torch.zeros(vocab, dtype=torch.int64, device=d)
        state.append(dict(cache=c, counts=counts, totals=torch.zeros(2, dtype=torch.int64, device=d),
                          feats=torch.zeros((B, 4), dtype=torch.float32, device=d), bits=torch.zeros(B, dtype=torch.uint8, device=d),
                          out=torch.zeros((L, B, Hq, 64), dtype=torch.float32, device=d),
                          p2=torch.full((B, Hq), 0.01, dtype=torch.float32, device=d),
                          ws=torch.empty(kvq.kvq_decode_attn_workspace(c, B), dtype=torch.uint8, device=d),
                          fws=torch.empty(kvq.kvq_features_workspace(B, wl.VOCAB), dtype=torch.uint8, device=d)))

    def step(st):
        kvq.kvq_features_controller(logits, ids, st["counts"], st["totals"], True, st["p2"], lens, Hq, mlp, st["feats"], st["bits"],
                                    st["fws"], cache=st["cache"])
        for l in range(L):
            kvq.kvq_append_decode_attn(st["cache"], l, k[l], v[l], None, q[l], None, B, st["out"][l], st["ws"], None,
                                       st["p2"] if l == L - 1 else None)

    def refresh(i):
        gg = torch.Generator(device="cpu").manual_seed(100 + i)
        logits.copy_(torch.randn((B, vocab), generator=gg) * 3.0)
        ids.copy_(torch.randint(0, vocab, (B,), generator=gg, dtype=torch.int32))
        lens.fill_(T0 + i)
        k.copy_(torch.randn(k.shape, generator=gg).to(torch.float16))
        v.copy_(torch.randn(v.shape, generator=gg).to(torch.float16))
        q.copy_(torch.randn(q.shape, generator=gg).to(torch.float16))

    eager, graphed = state
    refresh(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(graphed)                       # capture only records; the first replay below is step 0 of this cache
    for i in range(6):
        refresh(i)
        step(eager)
        graph.replay()
        torch.cuda.synchronize()
        # eager work and a synchronization between the replays
        assert float((eager["out"] - graphed["out"]).abs().sum()) == 0.0
        assert torch.equal(eager["bits"], graphed["bits"]) and torch.equal(eager["feats"], graphed["feats"])
        assert torch.equal(eager["p2"], graphed["p2"])
        assert torch.equal(eager["cache"].counts(), graphed["cache"].counts())
    assert torch.equal(eager["counts"], graphed["counts"]) and torch.equal(eager["totals"], graphed["totals"])
    assert eager["cache"].status()[0] == 0 and graphed["cache"].status()[0] == 0
    for l in range(L):
        for s in range(B):
            for x, y in zip(eager["cache"].export(l, s, T0 + 6), graphed["cache"].export(l, s, T0 + 6)):
                assert torch.equal(x, y)
    assert eager["cache"].counts()[:, 4].tolist() == [T0 + 6] * B


@pytest.mark.parametrize("n16", [1, 255, 256, 257, 2048 * 8 + 3, 1000003])
def test_measurement_probes_copy_every_byte_and_read_in_bounds(n16):
    """The bandwidth probes behind bench.py's stream ceilings: the copy must reproduce its source at any size (whole
    and ragged regions per workgroup), and neither kernel may touch anything past the end (guard words stay intact)."""
    print("probe kernels, %d 16-byte words" % n16, flush=True)
    g = torch.Generator(device="cpu").manual_seed(n16)
    src = torch.randint(0, 2 ** 31 - 1, (n16 * 4 + 8,), dtype=torch.int32, generator=g).to(dev())
    dst = torch.full((n16 * 4 + 8,), -7, dtype=torch.int32, device=dev())
    benchprobe.copy(dst[:n16 * 4], src[:n16 * 4])
    sink = torch.zeros(1, dtype=torch.int32, device=dev())
    benchprobe.read(src[:n16 * 4], sink)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n16 * 4], src[:n16 * 4])
    assert bool((dst[n16 * 4:] == -7).all())
    # three reads per write: dst = a ^ b ^ c, the sources back to back
    src3 = torch.randint(0, 2 ** 31 - 1, (3 * n16 * 4,), dtype=torch.int32, generator=g).to(dev())
    dst3 = torch.full((n16 * 4 + 8,), -7, dtype=torch.int32, device=dev())
    benchprobe.mix3(dst3[:n16 * 4], src3)
    torch.cuda.synchronize()
    a, b, c = src3[:n16 * 4], src3[n16 * 4:2 * n16 * 4], src3[2 * n16 * 4:]
    assert torch.equal(dst3[:n16 * 4], a ^ b ^ c)
    assert bool((dst3[n16 * 4:] == -7).all())
