"""GPU parity: kvq_features and kvq_controller against the CPU oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from helpers import dev
from paper_2604_04722_amd import binding as kvq
import workloads as wl

pytestmark = pytest.mark.gpu

# Feature tolerances (fp32 kernels vs an fp64 oracle): H, R, C are sums of ~5e4 fp32 terms of one sign, so a
# relative 2e-5 (plus 1e-6 absolute) leaves two orders of margin; V is a difference of order 1/l^2 taken from
# numbers of order 1/l, so its absolute floor scales with 1/l^2.
F_RTOL, F_ATOL = 2e-5, 1e-6


def say(*a):
    print(*a, flush=True)


def front_ws(n, vocab):
    """workspace of the fused front end (slice results and table entries between its two launches)"""
    return torch.empty(kvq.kvq_features_workspace(n, vocab), dtype=torch.uint8, device=dev())


def run_features(logits, ids, counts, N, Vobs, lens, Hq, probs=None, sum_p2=None, update=False):
    n, vocab = logits.shape
    d = dev()
    t_logits = torch.from_numpy(logits).to(d)
    t_ids = torch.from_numpy(ids.astype(np.int32)).to(d)
    t_counts = torch.from_numpy(counts.astype(np.int64)).to(d)
    t_tot = torch.tensor([N, Vobs], dtype=torch.int64, device=d)
    t_len = torch.from_numpy(np.asarray(lens, np.int32)).to(d)
    feats = torch.full((n, 4), float("nan"), dtype=torch.float32, device=d)
    ws = torch.empty(kvq.kvq_features_workspace(n, vocab), dtype=torch.uint8, device=d)
    kvq.kvq_features(t_logits, t_ids, t_counts, t_tot, update, t_len, Hq, feats, ws,
                     attn_probs=None if probs is None else torch.from_numpy(probs.astype(np.float32)).to(d),
                     sum_p2=None if sum_p2 is None else torch.from_numpy(sum_p2.astype(np.float32)).to(d))
    torch.cuda.synchronize()
    return feats.cpu().numpy(), t_counts.cpu().numpy(), t_tot.cpu().numpy()


def check_feats(got, want, lens):
    for col in (0, 1, 3):
        np.testing.assert_allclose(got[:, col], want[:, col], rtol=F_RTOL, atol=F_ATOL)
    l = np.asarray(lens, np.float64)
    assert np.all(np.abs(got[:, 2] - want[:, 2]) <= 1e-4 * np.abs(want[:, 2]) + 2e-6 / l ** 2 + 1e-12)


@pytest.mark.parametrize("n,vocab,sigma", [(1, 49152, 1.0), (16, 49152, 2.0), (64, 49152, 2.0), (5, 1000, 3.0), (3, 4099, 0.5), (2, 7, 1.0)])
def test_features_match_the_oracle(n, vocab, sigma):
    say("features n=%d vocab=%d sigma=%g" % (n, vocab, sigma))
    rng = np.random.default_rng(n * 31 + vocab)
    logits = (rng.standard_normal((n, vocab)) * sigma).astype(np.float32)
    ids = rng.integers(0, vocab, n).astype(np.int32)
    counts = rng.integers(0, 50, vocab).astype(np.int64) * (rng.random(vocab) < 0.6)
    N, Vobs = int(counts.sum()), int((counts > 0).sum())
    Hq, ld = 9, 700
    lens = rng.integers(1, ld + 1, n).astype(np.int32)
    raw = rng.standard_normal((n, Hq, ld)) * 2
    probs = np.zeros((n, Hq, ld), np.float32)
    for t in range(n):
        e = np.exp(raw[t, :, :lens[t]])
        probs[t, :, :lens[t]] = (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
        probs[t, :, lens[t]:] = 9.0                               # must be ignored
    want = oracle.features(logits, ids, counts, N, Vobs, probs.astype(np.float64), lens)
    got, c2, tot2 = run_features(logits, ids, counts, N, Vobs, lens, Hq, probs=probs)
    check_feats(got, want, lens)
    assert np.array_equal(c2, counts) and list(tot2) == [N, Vobs]   # update_counts = 0 leaves the tables alone


def test_features_closed_forms_uniform_and_peaked_rows():
    say("features closed forms")
    vocab = 49152
    logits = np.zeros((3, vocab), np.float32)
    logits[0] = 3.25                                              # uniform: H = ln V, C = 1/V
    logits[1, 77] = 100.0                                         # peaked: H = 0, C = 1
    logits[2, :7] = 5.5
    ids = np.array([0, 1, 2], np.int32)
    counts = np.zeros(vocab, np.int64)
    lens = np.array([64, 64, 64], np.int32)
    probs = np.full((3, 2, 64), 1 / 64, np.float32)
    got, _, _ = run_features(logits, ids, counts, 0, 0, lens, 2, probs=probs)
    assert got[0, 0] == pytest.approx(math.log(vocab), rel=2e-6) and got[0, 3] == pytest.approx(1 / vocab, rel=2e-6)
    assert abs(got[1, 0]) < 1e-6 and got[1, 3] == pytest.approx(1.0, rel=1e-6)
    Z = 7 * math.exp(5.5) + vocab - 7
    assert got[2, 0] == pytest.approx(math.log(Z) - 5.5 * 7 * math.exp(5.5) / Z, rel=5e-6)
    assert np.all(got[:, 1] == 0.0) and np.all(np.abs(got[:, 2]) < 1e-12)


def test_features_from_sum_p2_and_count_updates_with_duplicates():
    say("features: fused sum_p2 input, running counts with duplicate ids in one batch")
    n, vocab, Hq = 8, 2048, 6
    rng = np.random.default_rng(3)
    logits = rng.standard_normal((n, vocab)).astype(np.float32)
    ids = np.array([5, 5, 9, 1000, 5, 9, 3, 2047], np.int32)
    counts = np.zeros(vocab, np.int64)
    counts[9] = 4
    counts[3] = 1
    N, Vobs = 5, 2
    lens = rng.integers(2, 400, n).astype(np.int32)
    probs = np.zeros((n, Hq, 400))
    for t in range(n):
        e = np.exp(rng.standard_normal((Hq, lens[t])) * 3)
        probs[t, :, :lens[t]] = e / e.sum(axis=1, keepdims=True)
    p2 = (probs ** 2).sum(axis=2)
    want = oracle.features(logits, ids, counts, N, Vobs, probs, lens)
    got, c2, tot2 = run_features(logits, ids, counts, N, Vobs, lens, Hq, sum_p2=p2, update=True)
    check_feats(got, want, lens)
    wc, wN, wV = oracle.counts_update(ids, counts, N, Vobs)
    assert np.array_equal(c2, wc) and list(tot2) == [wN, wV]
    # a second call sees the updated table
    want2 = oracle.features(logits, ids, wc, wN, wV, probs, lens)
    got2, _, _ = run_features(logits, ids, c2, int(tot2[0]), int(tot2[1]), lens, Hq, sum_p2=p2)
    check_feats(got2, want2, lens)
    assert np.all(got2[:, 1] != got[:, 1])


def gpu_controller(feats, Ws, bs):
    d = dev()
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    n = feats.shape[0]
    bits = torch.zeros(n, dtype=torch.uint8, device=d)
    logits = torch.zeros((n, 4), dtype=torch.float32, device=d)
    kvq.kvq_controller(torch.from_numpy(feats).to(d), mlp, bits, logits)
    torch.cuda.synchronize()
    return bits.cpu().numpy(), logits.cpu().numpy()


def check_controller(feats, Ws, bs):
    want_bits, want_logits = oracle.controller(feats, Ws, bs)
    got_bits, got_logits = gpu_controller(feats, Ws, bs)
    scale = np.abs(want_logits).max() + 1.0
    np.testing.assert_allclose(got_logits, want_logits, rtol=0, atol=2e-6 * scale * 8)
    # precision assignments: identical, except where the oracle's two best logits are within 1e-5
    srt = np.sort(want_logits, axis=1)
    gap = srt[:, -1] - srt[:, -2]
    differ = got_bits != want_bits
    assert not np.any(differ & (gap > 1e-5)), "assignment differs off a tie at rows %s" % np.where(differ & (gap > 1e-5))[0][:5]
    top2 = np.argsort(want_logits, axis=1)[:, -2:]
    for r in np.where(differ)[0]:
        assert int(np.log2(got_bits[r])) - 1 in top2[r]
    return got_bits, want_bits


@pytest.mark.parametrize("cfg_index", [1, 2, 3, 4])
@pytest.mark.parametrize("n", [1, 64, 3000, 70000])
def test_controller_assignments_match_the_oracle(cfg_index, n):
    say("controller cfg %d n=%d" % (cfg_index, n))
    cfg = wl.CONFIGS[cfg_index]
    Ws, bs = wl.calibrated_mlp(cfg) if cfg_index >= 2 else wl.xavier_mlp(cfg)
    feats = wl.bulk_features(cfg, n, chunk=7)
    got, want = check_controller(feats, Ws, bs)
    if n >= 3000 and cfg_index >= 2:
        mix = np.array([(want == w).mean() for w in (2, 4, 8, 16)])
        assert np.max(np.abs(mix - np.array(cfg.mix))) < 0.03       # the calibrated mix holds on a fresh draw


def test_controller_bulk_call_at_the_benchmark_size():
    say("controller cfg 4, 262 144 rows (batch x context: the prefill call that bench.py times)")
    cfg = wl.CONFIGS[4]
    Ws, bs = wl.calibrated_mlp(cfg)
    got, want = check_controller(wl.bulk_features(cfg, cfg.batch * cfg.context, chunk=7), Ws, bs)
    mix = np.array([(want == w).mean() for w in (2, 4, 8, 16)])
    assert np.max(np.abs(mix - np.array(cfg.mix))) < 0.03


def test_controller_ties_zero_weights_and_two_layer_network():
    say("controller ties / hand-built weights")
    feats = np.random.default_rng(4).standard_normal((10, 4)).astype(np.float32)
    Ws = [np.zeros((8, 4), np.float32), np.zeros((4, 8), np.float32)]
    for b3, expect in (([0.5, 0.5, 0.5, 0.5], 2), ([0.1, 0.7, 0.3, 0.2], 4), ([0.1, 0.2, 0.9, 0.9], 8), ([0, 0, 0, 1e-3], 16)):
        bits, _ = gpu_controller(feats, Ws, [np.zeros(8, np.float32), np.array(b3, np.float32)])
        assert list(bits) == [expect] * 10
    W1 = np.zeros((2, 4), np.float32)
    W1[0, 1], W1[1, 1] = 1.0, -1.0
    W3 = np.array([[0, 0], [1, -1], [2, -2], [3, -3]], np.float32)
    b3 = np.array([0, -0.5, -2.0, -4.5], np.float32)
    f = np.zeros((8, 4), np.float32)
    f[:, 1] = [-5.0, 0.2, 0.7, 1.4, 1.6, 2.4, 2.6, 9.0]
    bits, _ = gpu_controller(f, [W1, np.eye(2, dtype=np.float32), W3], [np.zeros(2, np.float32)] * 2 + [b3])
    assert list(bits) == [2, 2, 4, 4, 8, 8, 16, 16]


def test_controller_row_and_bulk_launch_shapes_agree():
    say("controller: per-step, vector-ALU bulk and matrix-core bulk launch shapes")
    cfg = wl.CONFIGS[4]
    Ws, bs = wl.calibrated_mlp(cfg)
    feats = wl.bulk_features(cfg, 5000, chunk=3)
    # widths 128/128 take the matrix-core shape in bulk: same fp32 products, another summation order
    b_bulk, l_bulk = gpu_controller(feats, Ws, bs)
    b_row, l_row = gpu_controller(feats[:2048], Ws, bs)
    scale = np.abs(l_row).max() + 1.0
    np.testing.assert_allclose(l_bulk[:2048], l_row, rtol=0, atol=2e-6 * scale * 8)
    srt = np.sort(l_row, axis=1)
    assert not np.any((b_bulk[:2048] != b_row) & (srt[:, -1] - srt[:, -2] > 1e-5))
    # widths that are no multiple of 32 take the vector-ALU bulk shape (also widths above 128, here 200 and 256)
    rng = np.random.default_rng(12)
    for widths in ((48, 40), (200, 256)):
        shapes = ((widths[0], 4), (widths[1], widths[0]), (4, widths[1]))
        Wo = [rng.uniform(-0.5, 0.5, s).astype(np.float32) * np.float32(np.sqrt(4.0 / s[1])) for s in shapes]
        bo = [rng.uniform(-0.1, 0.1, s[0]).astype(np.float32) for s in shapes]
        b_bulk, l_bulk = gpu_controller(feats, Wo, bo)
        b_row, l_row = gpu_controller(feats[:2048], Wo, bo)
        scale = np.abs(l_row).max() + 1.0
        np.testing.assert_allclose(l_bulk[:2048], l_row, rtol=0, atol=2e-6 * scale * 8)
        srt = np.sort(l_row, axis=1)
        assert not np.any((b_bulk[:2048] != b_row) & (srt[:, -1] - srt[:, -2] > 1e-5))
        check_controller(feats, Wo, bo)
        check_controller(feats[:100], Wo, bo)


@pytest.mark.parametrize("widths", [(50, 33), (7,), (256, 200), (129, 3)])
def test_per_step_controller_widths_off_the_vector_path_and_the_fused_call_above_256_rows(widths):
    say("per-step controller, hidden widths %s: no multiple of 4 (scalar weight loads), several passes over the work items" % (widths,))
    d = dev()
    rng = np.random.default_rng(900 + sum(widths))
    dims = (4,) + tuple(widths) + (4,)
    Ws = [rng.uniform(-1, 1, (dims[i + 1], dims[i])).astype(np.float32) * np.float32(np.sqrt(3.0 / dims[i])) for i in range(len(dims) - 1)]
    bs = [rng.uniform(-0.3, 0.3, dims[i + 1]).astype(np.float32) for i in range(len(dims) - 1)]
    feats = rng.standard_normal((2048, 4)).astype(np.float32) * np.array([3.0, 4.0, 1e-3, 0.5], np.float32)
    for n in (1, 7, 256, 257, 2048):                              # 1024 threads a row up to 256 rows, 256 threads beyond
        check_controller(feats[:n], Ws, bs)
    # the fused call takes the same two workgroup sizes; its decision equals the separate calls' bit for bit
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    Hq, vocab = 6, 3001
    for n in (9, 300):
        logits, ids, counts, N, Vobs, lens, p2 = _front_inputs(n, vocab, Hq, 77 + n)
        t = lambda a: torch.from_numpy(a).to(d)
        t_logits, t_ids, t_len, t_p2 = t(logits), t(ids), t(lens), t(p2)
        c_a, tot_a = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
        f_a = torch.zeros((n, 4), dtype=torch.float32, device=d)
        b_a = torch.zeros(n, dtype=torch.uint8, device=d)
        l_a = torch.zeros((n, 4), dtype=torch.float32, device=d)
        kvq.kvq_features(t_logits, t_ids, c_a, tot_a, True, t_len, Hq, f_a, front_ws(n, vocab), sum_p2=t_p2)
        kvq.kvq_controller(f_a, mlp, b_a, l_a)
        c_b, tot_b = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
        f_b = torch.full((n, 4), float("nan"), dtype=torch.float32, device=d)
        b_b = torch.zeros(n, dtype=torch.uint8, device=d)
        l_b = torch.zeros((n, 4), dtype=torch.float32, device=d)
        kvq.kvq_features_controller(t_logits, t_ids, c_b, tot_b, True, t_p2, t_len, Hq, mlp, f_b, b_b, front_ws(n, vocab), logits_out=l_b)
        torch.cuda.synchronize()
        assert np.array_equal(f_b.cpu().numpy().view(np.uint32), f_a.cpu().numpy().view(np.uint32))
        assert np.array_equal(l_b.cpu().numpy().view(np.uint32), l_a.cpu().numpy().view(np.uint32))
        assert np.array_equal(b_b.cpu().numpy(), b_a.cpu().numpy())
        assert np.array_equal(c_b.cpu().numpy(), c_a.cpu().numpy()) and np.array_equal(tot_b.cpu().numpy(), tot_a.cpu().numpy())
        want_bits, want_logits = oracle.controller(f_a.cpu().numpy(), Ws, bs)
        srt = np.sort(want_logits, axis=1)
        assert not np.any((b_b.cpu().numpy() != want_bits) & (srt[:, -1] - srt[:, -2] > 1e-5))


@pytest.mark.parametrize("dims", [(4, 32, 4), (4, 64, 4), (4, 128, 4), (4, 32, 32, 4), (4, 64, 128, 4), (4, 128, 32, 4), (4, 128, 64, 4)])
@pytest.mark.parametrize("n", [2049, 4097, 33333])
def test_controller_matrix_core_shape_all_width_combinations(dims, n):
    say("controller matrix-core shape dims %s n=%d" % (dims, n))
    rng = np.random.default_rng(sum(dims) + n)
    Ws = [rng.uniform(-1, 1, (dims[i + 1], dims[i])).astype(np.float32) * np.float32(np.sqrt(3.0 / dims[i])) for i in range(len(dims) - 1)]
    bs = [rng.uniform(-0.3, 0.3, dims[i + 1]).astype(np.float32) for i in range(len(dims) - 1)]
    feats = rng.standard_normal((n, 4)).astype(np.float32) * np.array([3.0, 4.0, 1e-3, 0.5], np.float32)
    check_controller(feats, Ws, bs)


def test_end_to_end_step_features_controller_append_attention():
    say("one decode step end to end: features -> controller -> append -> attention (sum_p2 feeds the next step)")
    cfg = wl.CONFIGS[1]
    d = dev()
    B, Hq, Hkv, vocab = 4, cfg.n_q_heads, cfg.n_kv_heads, wl.VOCAB
    Ws, bs = wl.xavier_mlp(cfg)
    counts, N, Vobs, probs_tab = wl.zipf_table(cfg)
    ids = wl.zipf_ids(cfg, probs_tab, 0, B)
    logits = wl.logits(cfg, 0, B, "cpu").numpy()
    lens = np.array([7, 7, 7, 7], np.int32)
    sum_p2 = np.random.default_rng(8).uniform(1 / 7, 1.0, (B, Hq)).astype(np.float32)
    feats, _, _ = run_features(logits, ids, counts, N, Vobs, lens, Hq, sum_p2=sum_p2)
    # oracle side: the same sum_p2 corresponds to no explicit row, so compare H, R, C and the closed form of V
    probs = np.zeros((B, Hq, 7))
    probs[:, :, 0] = 1.0
    want = oracle.features(logits, ids, counts, N, Vobs, probs, lens)
    np.testing.assert_allclose(feats[:, [0, 1, 3]], want[:, [0, 1, 3]], rtol=F_RTOL, atol=F_ATOL)
    np.testing.assert_allclose(feats[:, 2], (sum_p2.astype(np.float64) / 7 - 1 / 49).mean(axis=1), rtol=1e-4)
    got_bits, want_bits = check_controller(feats, Ws, bs)
    assert set(got_bits.tolist()) <= {2, 4, 8, 16}


@pytest.mark.parametrize("cfg_index", [1, 2, 4])
def test_assignment_chain_gpu_features_into_gpu_controller_against_the_oracle_chain(cfg_index):
    """Precision assignments end to end (Sec. 3.5 features -> Sec. 3.6 controller): GPU features fed to the GPU controller
    against oracle features fed to the oracle controller, on 10 240 rows of logits over the 49152-token vocabulary.  A row
    may disagree only inside the widened tie gap 1e-5 + |W3||W2||W1| * |s_gpu - s_oracle| (spectral norms: the most the
    feature error can move a logit difference, up to the factor 2 of a difference of two logits)."""
    cfg = wl.CONFIGS[cfg_index]
    say("assignment chain, controller %s, 10240 rows" % (cfg.mlp_dims,))
    Ws, bs = wl.calibrated_mlp(cfg) if cfg_index >= 2 else wl.xavier_mlp(cfg)
    lip = float(np.prod([np.linalg.norm(w.astype(np.float64), 2) for w in Ws]))
    d = dev()
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    counts, N, Vobs, probs_tab = wl.zipf_table(wl.CONFIGS[4])
    Hq, CH, n_total = 8, 1024, 10240
    rng = np.random.default_rng(4722 + cfg_index)
    differ = inside = 0
    worst_df = 0.0
    for c0 in range(0, n_total, CH):
        # config-4-style rows (sigma 2) in the first half; the second half with a temperature of its own per row, so
        # that the entropy and confidence features (and with them the decisions) spread over their range
        g = torch.Generator(device="cpu").manual_seed(int(rng.integers(1 << 40)))
        z = torch.randn((CH, wl.VOCAB), generator=g, dtype=torch.float32)
        sig = np.full(CH, 2.0) if c0 < n_total // 2 else rng.uniform(0.3, 7.0, CH)
        z *= torch.from_numpy(sig.astype(np.float32))[:, None]
        logits = z.numpy()
        ids = wl.zipf_ids(wl.CONFIGS[4], probs_tab, 50 + c0 // CH, CH)
        lens = rng.integers(16, 1025, CH).astype(np.int32)
        p2 = (np.exp(rng.normal(0.0, 1.0, (CH, Hq))) / lens[:, None]).clip(max=1.0)       # sum p^2 in [1/l, 1]
        p2 = np.maximum(p2, 1.0 / lens[:, None])
        got_f, _, _ = run_features(logits, ids, counts, N, Vobs, lens, Hq, sum_p2=p2)
        # the oracle takes explicit attention rows; rows with the same sum of squares: one entry a, the rest equal
        want_f = oracle.features(logits, ids, counts, N, Vobs, _rows_with_sum_p2(p2, lens), lens)
        got_b = torch.zeros(CH, dtype=torch.uint8, device=d)
        kvq.kvq_controller(torch.from_numpy(got_f).to(d), mlp, got_b)
        got_b = got_b.cpu().numpy()
        want_b, want_logits = oracle.controller(want_f, Ws, bs)
        srt = np.sort(want_logits, axis=1)
        gap = srt[:, -1] - srt[:, -2]
        df = np.linalg.norm(got_f.astype(np.float64) - want_f.astype(np.float64), axis=1)
        worst_df = max(worst_df, float(df.max()))
        allowed = 1e-5 + 2.0 * lip * df
        bad = got_b != want_b
        assert not np.any(bad & (gap > allowed)), "assignment differs outside the widened gap at rows %s" % (c0 + np.where(bad & (gap > allowed))[0][:5])
        differ += int(bad.sum())
        inside += int((gap <= allowed).sum())
    say("assignment chain cfg %d: %d of %d rows differ (%.4f %%); %d rows lie inside their widened gap; largest |ds| %.3g; |W3||W2||W1| = %.3g"
        % (cfg_index, differ, n_total, 100.0 * differ / n_total, inside, worst_df, lip))


def _rows_with_sum_p2(p2, lens):
    """Attention rows [n, Hq, max l] (fp64) whose squares sum to p2: one entry a, the other l-1 entries (1-a)/(l-1), with
    a the larger root of a^2 + (1-a)^2/(l-1) = p2."""
    n, Hq = p2.shape
    ld = int(lens.max())
    rows = np.zeros((n, Hq, ld))
    for t in range(n):
        l = int(lens[t])
        if l == 1:
            rows[t, :, 0] = 1.0
            continue
        k = l - 1.0
        # a^2 (1 + 1/k) - 2a/k + 1/k - p2 = 0
        A, Bq, C = 1.0 + 1.0 / k, -2.0 / k, 1.0 / k - p2[t]
        disc = np.maximum(Bq * Bq - 4.0 * A * C, 0.0)
        a = (-Bq + np.sqrt(disc)) / (2.0 * A)
        rows[t, :, :l] = ((1.0 - a) / k)[:, None]
        rows[t, :, 0] = a
    return rows


def _front_inputs(n, vocab, Hq, seed, dup=True):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((n, vocab)) * 2.0).astype(np.float32)
    ids = rng.integers(0, vocab, n).astype(np.int32)
    if dup and n >= 4:
        ids[1] = ids[0]
        ids[3] = ids[0]
    counts = rng.integers(0, 50, vocab).astype(np.int64)
    counts[ids[0]] = 0                                           # a first sighting, three times in one batch
    N, Vobs = int(counts.sum()), int((counts > 0).sum())
    lens = rng.integers(5, 900, n).astype(np.int32)
    p2 = rng.uniform(1.0 / lens[:, None], 1.0, (n, Hq)).astype(np.float32)
    return logits, ids, counts, N, Vobs, lens, p2


@pytest.mark.parametrize("n,vocab", [(1, 49152), (5, 5003), (32, 49152), (70, 8192)])
@pytest.mark.parametrize("cfg_index", [2, 4])
def test_fused_features_controller_is_bit_identical_to_the_separate_calls(n, vocab, cfg_index):
    say("fused front end n=%d vocab=%d cfg %d" % (n, vocab, cfg_index))
    d = dev()
    Hq = 6
    Ws, bs = wl.calibrated_mlp(wl.CONFIGS[cfg_index])
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    logits, ids, counts, N, Vobs, lens, p2 = _front_inputs(n, vocab, Hq, 1000 + n + cfg_index)
    t = lambda a, dt=None: torch.from_numpy(a if dt is None else a.astype(dt)).to(d)
    t_logits, t_ids, t_len, t_p2 = t(logits), t(ids), t(lens), t(p2)

    # separate calls, twice in a row (the second sees the updated table)
    c_a, tot_a = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
    ws_a = torch.empty(kvq.kvq_features_workspace(n, vocab), dtype=torch.uint8, device=d)
    sep = []
    for _ in range(2):
        feats = torch.zeros((n, 4), dtype=torch.float32, device=d)
        bits = torch.zeros(n, dtype=torch.uint8, device=d)
        lg = torch.zeros((n, 4), dtype=torch.float32, device=d)
        kvq.kvq_features(t_logits, t_ids, c_a, tot_a, True, t_len, Hq, feats, ws_a, sum_p2=t_p2)
        kvq.kvq_controller(feats, mlp, bits, lg)
        torch.cuda.synchronize()
        sep.append((feats.cpu().numpy(), bits.cpu().numpy(), lg.cpu().numpy(), c_a.cpu().numpy(), tot_a.cpu().numpy()))

    # the fused call, twice
    c_b, tot_b = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
    for it in range(2):
        feats = torch.full((n, 4), float("nan"), dtype=torch.float32, device=d)
        bits = torch.zeros(n, dtype=torch.uint8, device=d)
        lg = torch.zeros((n, 4), dtype=torch.float32, device=d)
        kvq.kvq_features_controller(t_logits, t_ids, c_b, tot_b, True, t_p2, t_len, Hq, mlp, feats, bits, front_ws(n, vocab), logits_out=lg)
        torch.cuda.synchronize()
        f0, b0, l0, c0, t0 = sep[it]
        assert np.array_equal(feats.cpu().numpy().view(np.uint32), f0.view(np.uint32))
        assert np.array_equal(bits.cpu().numpy(), b0)
        assert np.array_equal(lg.cpu().numpy().view(np.uint32), l0.view(np.uint32))
        assert np.array_equal(c_b.cpu().numpy(), c0) and np.array_equal(tot_b.cpu().numpy(), t0)
    # and the oracle agrees with the first call
    wc, wN, wV = oracle.counts_update(ids, counts, N, Vobs)
    assert np.array_equal(sep[0][3], wc) and list(sep[0][4]) == [wN, wV]


def test_fused_front_end_advances_the_cache_like_a_layer0_append():
    say("fused front end + cache bookkeeping over 1100 decode steps (some class crosses a page boundary)")
    d = dev()
    B, Hq, Hkv, L, vocab = 3, 4, 2, 2, 4096
    Ws, bs = wl.calibrated_mlp(wl.CONFIGS[4])
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    cache_a = kvq.Cache(L, B, Hq, Hkv, 2048)
    cache_b = kvq.Cache(L, B, Hq, Hkv, 2048)
    rng = np.random.default_rng(77)
    counts0 = rng.integers(0, 5, vocab).astype(np.int64)
    c_a = torch.from_numpy(counts0).to(d)
    c_b = c_a.clone()
    tot_a = torch.tensor([int(counts0.sum()), int((counts0 > 0).sum())], dtype=torch.int64, device=d)
    tot_b = tot_a.clone()
    ws_a = torch.empty(kvq.kvq_features_workspace(B, vocab), dtype=torch.uint8, device=d)
    aws = torch.empty(kvq.kvq_decode_attn_workspace(cache_a, B), dtype=torch.uint8, device=d)
    seq_ids = torch.tensor([2, 0, 1], dtype=torch.int32, device=d)
    feats_a = torch.zeros((B, 4), dtype=torch.float32, device=d)
    feats_b = torch.zeros((B, 4), dtype=torch.float32, device=d)
    bits_a = torch.zeros((B, 1), dtype=torch.uint8, device=d)
    bits_b = torch.zeros((B, 1), dtype=torch.uint8, device=d)
    out_a = torch.zeros((B, Hq, 64), dtype=torch.float32, device=d)
    out_b = torch.zeros((B, Hq, 64), dtype=torch.float32, device=d)
    p2_a = torch.full((B, Hq), 0.5, dtype=torch.float32, device=d)
    p2_b = p2_a.clone()
    n_steps = 1100
    for step in range(n_steps):
        g = torch.Generator(device="cpu").manual_seed(step)
        logits = (torch.randn((B, vocab), generator=g) * 3.0).to(d)
        ids = torch.randint(0, vocab, (B,), generator=g, dtype=torch.int32).to(d)
        lens = torch.full((B,), step + 1, dtype=torch.int32, device=d)
        K = (torch.randn((L, B, 1, Hkv, 64), generator=g)).to(torch.float16).to(d)
        V = (torch.randn((L, B, 1, Hkv, 64), generator=g)).to(torch.float16).to(d)
        q = (torch.randn((L, B, Hq, 64), generator=g)).to(torch.float16).to(d)
        # path a: five calls per step and layer
        p2_prev = p2_a.clone()
        kvq.kvq_features(logits, ids, c_a, tot_a, True, lens, Hq, feats_a, ws_a, sum_p2=p2_a)
        kvq.kvq_controller(feats_a, mlp, bits_a.view(-1))
        for l in range(L):
            kvq.kvq_append(cache_a, l, K[l], V[l], bits_a if l == 0 else None, seq_ids, B, 1)
            kvq.kvq_decode_attn(cache_a, l, q[l], seq_ids, B, out_a, aws, None, p2_a if l == L - 1 else None)
        # path b: the fused front end (two launches), then one launch per layer
        # (the variance feature of both paths comes from path a's attention: the two attention entry points agree
        # within the attention tolerance, not bit for bit, and this test compares bookkeeping exactly)
        kvq.kvq_features_controller(logits, ids, c_b, tot_b, True, p2_prev, lens, Hq, mlp, feats_b, bits_b.view(-1),
                                    front_ws(logits.shape[0], logits.shape[1]), cache=cache_b, seq_ids=seq_ids)
        for l in range(L):
            kvq.kvq_append_decode_attn(cache_b, l, K[l], V[l], None, q[l], seq_ids, B, out_b, aws, None, p2_b if l == L - 1 else None)
        if step % 100 == 99:
            torch.cuda.synchronize()
            assert torch.equal(bits_a, bits_b) and torch.equal(feats_a, feats_b)
            assert torch.all((out_a - out_b).abs() <= 2e-3 + 1e-3 * out_a.abs())
            assert torch.allclose(p2_a, p2_b, rtol=1e-3, atol=1e-7)
            assert torch.equal(cache_a.counts(), cache_b.counts())
    assert cache_a.status()[0] == 0 and cache_b.status()[0] == 0
    assert torch.equal(c_a, c_b) and torch.equal(tot_a, tot_b)
    for l in range(L):
        for s in range(B):
            ea, eb = cache_a.export(l, s, n_steps), cache_b.export(l, s, n_steps)
            for x, y in zip(ea, eb):
                assert torch.equal(x, y)
    cnt = cache_a.counts().numpy()
    assert cnt[:, 4].tolist() == [n_steps] * 3 and cnt[:, :4].max() > 256


def test_a_sequence_without_an_attention_row_yet_has_zero_variance_feature():
    say("features with attn_len == 0 on some rows (first token of a sequence)")
    d = dev()
    n, vocab, Hq = 6, 4096, 5
    logits, ids, counts, N, Vobs, lens, p2 = _front_inputs(n, vocab, Hq, 77)
    lens = lens.copy()
    lens[[1, 4]] = 0
    Ws, bs = wl.calibrated_mlp(wl.CONFIGS[4])
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    got, _, _ = run_features(logits, ids, counts, N, Vobs, lens, Hq, sum_p2=p2)
    feats = torch.zeros((n, 4), dtype=torch.float32, device=d)
    bits = torch.zeros(n, dtype=torch.uint8, device=d)
    kvq.kvq_features_controller(torch.from_numpy(logits).to(d), torch.from_numpy(ids).to(d), torch.from_numpy(counts).to(d),
                                torch.tensor([N, Vobs], dtype=torch.int64, device=d), False, torch.from_numpy(p2).to(d),
                                torch.from_numpy(lens).to(d), Hq, mlp, feats, bits, front_ws(n, logits.shape[1]))
    torch.cuda.synchronize()
    fused = feats.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), fused.view(np.uint32))
    assert np.all(got[[1, 4], 2] == 0.0) and np.all(np.isfinite(got))
    live = [0, 2, 3, 5]
    want_v = (p2[live].astype(np.float64) / lens[live, None] - 1.0 / lens[live, None].astype(np.float64) ** 2).mean(axis=1)
    np.testing.assert_allclose(got[live, 2], want_v, rtol=2e-3, atol=1e-9)
    # with explicit rows: a zero-length row gives V = 0 too
    probs = np.random.default_rng(3).random((n, Hq, 16))
    probs /= probs.sum(axis=2, keepdims=True)
    l2 = np.array([16, 0, 16, 16, 0, 16], np.int32)
    got2, _, _ = run_features(logits, ids, counts, N, Vobs, l2, Hq, probs=probs)
    assert np.all(got2[[1, 4], 2] == 0.0) and np.all(np.isfinite(got2))
    np.testing.assert_allclose(got2[live, 2], probs[live].var(axis=2).mean(axis=1), rtol=1e-4)


@pytest.mark.parametrize("n", [1, 257, 100000])
def test_rule_policy_matches_the_oracle(n):
    say("rule-based stand-in policy n=%d" % n)
    d = dev()
    feats = wl.bulk_features(wl.CONFIGS[4], n, chunk=11)
    w = np.array([1.0 / math.log(wl.VOCAB), 1.0 / 14.0, 50.0, -1.0], np.float32)
    thr = np.array([0.1, 0.45, 0.8], np.float32)
    want_bits, want_score = oracle.rule_policy(feats, w, 0.05, thr)
    bits = torch.zeros(n, dtype=torch.uint8, device=d)
    score = torch.zeros(n, dtype=torch.float32, device=d)
    kvq.kvq_rule_policy(torch.from_numpy(feats).to(d), kvq.make_rule(w, 0.05, thr), bits, score)
    torch.cuda.synchronize()
    got_bits, got_score = bits.cpu().numpy(), score.cpu().numpy()
    np.testing.assert_allclose(got_score, want_score, rtol=0, atol=4e-7 * (1.0 + np.abs(want_score).max()))
    # identical widths except where the oracle's score lies within 1e-5 of a threshold
    near = np.min(np.abs(want_score[:, None] - thr[None, :].astype(np.float64)), axis=1) <= 1e-5
    assert np.array_equal(got_bits[~near], want_bits[~near])
    assert np.all(np.abs(np.log2(got_bits[near].astype(float)) - np.log2(want_bits[near].astype(float))) <= 1)
    if n >= 1000:
        assert len(set(got_bits.tolist())) == 4
    with pytest.raises(kvq.KvqError):
        kvq.kvq_rule_policy(torch.from_numpy(feats).to(d), kvq.make_rule(w, 0.0, [0.5, 0.4, 0.9]), bits)


# ---- 16-bit logits: the features are those of the exactly widened row --------------------------------------

@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32])
@pytest.mark.parametrize("n,vocab", [(1, 49152), (32, 49152), (5, 5003), (3, 4099), (2, 7), (70, 8192)])
def test_narrow_logits_give_the_features_of_the_widened_row(dtype, n, vocab):
    say("typed features %s n=%d vocab=%d" % (dtype, n, vocab))
    d = dev()
    Hq = 6
    cfg = wl.CONFIGS[4]
    Ws, bs = wl.calibrated_mlp(cfg)
    mlp = kvq.MlpWeights([torch.from_numpy(w).to(d) for w in Ws], [torch.from_numpy(b).to(d) for b in bs])
    logits, ids, counts, N, Vobs, lens, p2 = _front_inputs(n, vocab, Hq, 4000 + n + vocab)
    # an odd vocabulary makes rows of a 16-bit type start at 2-byte (not 16-byte) boundaries: the peel is exercised
    t_narrow = torch.from_numpy(logits).to(dtype).to(d)
    widened = t_narrow.to(torch.float32).cpu().numpy()              # exact: what the kernel is asked to score
    t = lambda a: torch.from_numpy(a).to(d)
    t_ids, t_len, t_p2 = t(ids), t(lens), t(p2)
    var = (p2.astype(np.float64) / lens[:, None] - 1.0 / lens[:, None].astype(np.float64) ** 2).mean(axis=1)
    # the oracle's attention-variance input is a probability row; here the kernels take sum_p2, so the oracle scores
    # H, R, C and the variance column is checked against the closed form
    want = oracle.features(widened, ids, counts, N, Vobs, np.full((n, Hq, 1), 1.0), np.ones(n, np.int32))

    c_a, tot_a = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
    ws = torch.empty(kvq.kvq_features_workspace(n, vocab), dtype=torch.uint8, device=d)
    feats = torch.full((n, 4), float("nan"), dtype=torch.float32, device=d)
    kvq.kvq_features_typed(t_narrow, t_ids, c_a, tot_a, True, t_len, Hq, feats, ws, sum_p2=t_p2)
    bits = torch.zeros(n, dtype=torch.uint8, device=d)
    lg = torch.zeros((n, 4), dtype=torch.float32, device=d)
    kvq.kvq_controller(feats, mlp, bits, lg)
    torch.cuda.synchronize()
    got = feats.cpu().numpy()
    for col in (0, 1, 3):
        np.testing.assert_allclose(got[:, col], want[:, col], rtol=F_RTOL, atol=F_ATOL)
    np.testing.assert_allclose(got[:, 2], var, rtol=2e-3, atol=1e-9)
    wc, wN, wV = oracle.counts_update(ids, counts, N, Vobs)
    assert np.array_equal(c_a.cpu().numpy(), wc) and list(tot_a.cpu().numpy()) == [wN, wV]

    # the fused call on the same narrow logits: bit-identical features, logits and decisions
    c_b, tot_b = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
    feats2 = torch.full((n, 4), float("nan"), dtype=torch.float32, device=d)
    bits2 = torch.zeros(n, dtype=torch.uint8, device=d)
    lg2 = torch.zeros((n, 4), dtype=torch.float32, device=d)
    kvq.kvq_features_controller_typed(t_narrow, t_ids, c_b, tot_b, True, t_p2, t_len, Hq, mlp, feats2, bits2, front_ws(n, vocab), logits_out=lg2)
    torch.cuda.synchronize()
    assert np.array_equal(feats2.cpu().numpy().view(np.uint32), got.view(np.uint32))
    assert np.array_equal(bits2.cpu().numpy(), bits.cpu().numpy())
    assert np.array_equal(lg2.cpu().numpy().view(np.uint32), lg.cpu().numpy().view(np.uint32))
    assert np.array_equal(c_b.cpu().numpy(), wc)

    if dtype == torch.float32:
        # type code F32 is the untyped call
        c_c, tot_c = t(counts), torch.tensor([N, Vobs], dtype=torch.int64, device=d)
        feats3 = torch.full((n, 4), float("nan"), dtype=torch.float32, device=d)
        kvq.kvq_features(t_narrow, t_ids, c_c, tot_c, True, t_len, Hq, feats3, ws, sum_p2=t_p2)
        torch.cuda.synchronize()
        assert np.array_equal(feats3.cpu().numpy().view(np.uint32), got.view(np.uint32))


def test_typed_logits_reject_unknown_type_codes_and_misaligned_rows():
    say("typed features: error paths")
    d = dev()
    n, vocab, Hq = 2, 64, 2
    lib = kvq.load_library()
    z = torch.zeros((n, vocab + 1), dtype=torch.float16, device=d)
    ids = torch.zeros(n, dtype=torch.int32, device=d)
    counts = torch.zeros(vocab, dtype=torch.int64, device=d)
    tot = torch.zeros(2, dtype=torch.int64, device=d)
    lens = torch.ones(n, dtype=torch.int32, device=d)
    p2 = torch.ones((n, Hq), dtype=torch.float32, device=d)
    feats = torch.zeros((n, 4), dtype=torch.float32, device=d)
    ws = torch.empty(kvq.kvq_features_workspace(n, vocab), dtype=torch.uint8, device=d)

    def call(ptr, code):
        return lib.kvq_features_typed(ptr, code, n, vocab, ids.data_ptr(), counts.data_ptr(), tot.data_ptr(), 0, None, p2.data_ptr(),
                                      lens.data_ptr(), Hq, 0, feats.data_ptr(), ws.data_ptr(), ws.numel(), None)
    assert call(z.data_ptr(), 7) == kvq.KVQ_ERR_INVALID_ARG
    assert call(z.data_ptr() + 1, kvq.DTYPE_F16) == kvq.KVQ_ERR_INVALID_ARG          # odd address for a 2-byte type
    assert call(z.data_ptr() + 2, kvq.DTYPE_F32) == kvq.KVQ_ERR_INVALID_ARG          # 2 mod 4 for a 4-byte type
    assert call(z.data_ptr() + 2, kvq.DTYPE_F16) == kvq.KVQ_OK                       # 2-byte aligned rows are fine
    torch.cuda.synchronize()
    with pytest.raises(ValueError):
        kvq.kvq_features_typed(z.to(torch.float64)[:, :vocab].contiguous(), ids, counts, tot, False, lens, Hq, feats, ws, sum_p2=p2)
