"""Pins for the oracle's saliency features (paper Sec. 3.5) and controller forward (paper Sec. 3.6)."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import oracle

VOCAB = 49152


def feats_of(logits, ids=None, counts=None, N=0, Vobs=0, probs=None, lens=None):
    logits = np.asarray(logits, np.float32)
    n, vocab = logits.shape
    ids = np.zeros(n, np.int32) if ids is None else np.asarray(ids, np.int32)
    counts = np.zeros(vocab, np.int64) if counts is None else np.asarray(counts, np.int64)
    if probs is None:
        probs = np.full((n, 1, 4), 0.25)
        lens = np.full(n, 4, np.int32)
    return oracle.features(logits, ids, counts, N, Vobs, probs, lens)


# ---------------------------------------------------------------- entropy H_t and confidence C_t

def test_uniform_logits_give_log_vocab_and_one_over_vocab():
    f = feats_of(np.full((1, VOCAB), 3.25))
    assert f[0, 0] == np.float32(math.log(VOCAB))          # 10.802673...
    assert f[0, 3] == np.float32(1.0 / VOCAB)


def test_one_overwhelming_logit_gives_zero_entropy_and_full_confidence():
    z = np.zeros((1, VOCAB), np.float32)
    z[0, 123] = 100.0
    f = feats_of(z)
    assert 0.0 <= f[0, 0] < 1e-30 and f[0, 3] == 1.0


@pytest.mark.parametrize("k,a", [(1, 2.0), (7, 5.5), (1000, 1.0), (49151, -3.0)])
def test_k_logits_at_a_rest_zero_closed_form(k, a):
    z = np.zeros((1, VOCAB), np.float32)
    z[0, :k] = a
    Z = k * math.exp(a) + (VOCAB - k)
    H = math.log(Z) - a * k * math.exp(a) / Z
    C = max(math.exp(a), 1.0) / Z
    f = feats_of(z)
    assert f[0, 0] == pytest.approx(H, rel=2e-7) and f[0, 3] == pytest.approx(C, rel=2e-7)


def test_entropy_matches_library_routines_is_shift_invariant_and_bounded():
    rng = np.random.default_rng(1)
    z = (rng.standard_normal((6, VOCAB)) * 2.0).astype(np.float32)
    f = feats_of(z)
    p = scipy.special.softmax(z.astype(np.float64), axis=1)
    H_lib = scipy.stats.entropy(p, axis=1)
    H_logsm = -(p * scipy.special.log_softmax(z.astype(np.float64), axis=1)).sum(axis=1)
    np.testing.assert_array_equal(f[:, 0], H_lib.astype(np.float32))
    np.testing.assert_allclose(f[:, 0], H_logsm, rtol=1e-7)
    np.testing.assert_array_equal(f[:, 3], p.max(axis=1).astype(np.float32))
    shifted = feats_of((z.astype(np.float64) + 64.0).astype(np.float32))   # z+64 is re-rounded to fp32:
    np.testing.assert_allclose(shifted[:, 0], f[:, 0], rtol=1e-5)          # invariant up to that rounding only
    assert np.all(f[:, 0] >= 0) and np.all(f[:, 0] <= math.log(VOCAB))
    # N(0, sigma^2) logits: H ~ ln V - sigma^2/2
    assert abs(float(f[:, 0].mean()) - (math.log(VOCAB) - 2.0)) < 0.05


def test_entropy_is_exactly_shift_invariant_for_exactly_shifted_logits():
    rng = np.random.default_rng(2)
    z = rng.integers(-20, 20, (2, 512)).astype(np.float32) / 4
    a = oracle.features(z, np.zeros(2, np.int32), np.zeros(512, np.int64), 0, 0, np.full((2, 1, 2), 0.5), np.full(2, 2, np.int32))
    b = oracle.features(z + 32.0, np.zeros(2, np.int32), np.zeros(512, np.int64), 0, 0, np.full((2, 1, 2), 0.5), np.full(2, 2, np.int32))
    np.testing.assert_array_equal(a[:, [0, 3]], b[:, [0, 3]])


def test_underflowing_probabilities_contribute_zero_not_nan():
    z = np.zeros((1, 64), np.float32)
    z[0, 0] = 2000.0                      # every other p underflows to exactly 0 in fp64
    f = oracle.features(z, np.zeros(1, np.int32), np.zeros(64, np.int64), 0, 0, np.full((1, 1, 2), 0.5), np.full(1, 2, np.int32))
    assert f[0, 0] == 0.0 and f[0, 3] == 1.0


# ---------------------------------------------------------------- rarity R_t

def test_rarity_hand_table_empty_table_unseen_token_and_monotonicity():
    z = np.zeros((3, 8), np.float32)
    counts = np.array([5, 0, 1, 0, 0, 0, 0, 0], np.int64)            # N = 6, two distinct tokens observed
    f = feats_of(z, ids=[0, 1, 2], counts=counts, N=6, Vobs=2)
    assert f[0, 1] == np.float32(-math.log(6 / 9))
    assert f[1, 1] == np.float32(math.log(9))                        # unseen: ln(N + Vobs + 1)
    assert f[2, 1] == np.float32(-math.log(2 / 9))
    assert f[1, 1] > f[2, 1] > f[0, 1]
    f0 = feats_of(z[:1], ids=[4], counts=np.zeros(8, np.int64), N=0, Vobs=0)
    assert f0[0, 1] == 0.0                                           # -ln(1/1)


def test_counts_update_scores_first_then_counts_and_tracks_distinct_ids():
    counts = np.array([0, 3, 0, 0], np.int64)
    c2, N2, V2 = oracle.counts_update(np.array([0, 0, 1, 2], np.int32), counts, 3, 1)
    assert list(c2) == [2, 4, 1, 0] and N2 == 7 and V2 == 3
    assert list(counts) == [0, 3, 0, 0]


# ---------------------------------------------------------------- attention variance V_t

def test_variance_uniform_row_is_zero_one_hot_row_closed_form_and_matches_numpy():
    l, Hq = 50, 3
    z = np.zeros((1, 8), np.float32)
    uni = np.full((1, Hq, 64), 1.0 / 64)                              # power of two: the mean is exact
    assert feats_of(z, probs=uni, lens=[64])[0, 2] == 0.0
    assert feats_of(z, probs=np.full((1, Hq, l), 1.0 / l), lens=[l])[0, 2] < 1e-30
    hot = np.zeros((1, Hq, l))
    hot[0, :, 7] = 1.0
    assert feats_of(z, probs=hot, lens=[l])[0, 2] == np.float32((1 / l) * (1 - 1 / l))
    rng = np.random.default_rng(3)
    p = scipy.special.softmax(rng.standard_normal((2, Hq, 80)) * 3, axis=2)
    lens = np.array([80, 33], np.int32)
    p[1, :, 33:] = 7.0                                               # beyond the row length: must be ignored
    p[1, :, :33] /= p[1, :, :33].sum(axis=1, keepdims=True)
    f = feats_of(np.zeros((2, 8), np.float32), probs=p, lens=lens)
    for t in range(2):
        want = np.mean([np.var(p[t, i, : lens[t]]) for i in range(Hq)])
        assert f[t, 2] == np.float32(want)
        closed = np.mean([(p[t, i, : lens[t]] ** 2).sum() / lens[t] - 1.0 / lens[t] ** 2 for i in range(Hq)])
        assert f[t, 2] == pytest.approx(closed, rel=1e-6)


def test_variance_is_the_mean_over_heads_not_the_variance_of_the_pooled_rows():
    l = 10
    p = np.zeros((1, 2, l))
    p[0, 0] = 1.0 / l                      # var 0
    p[0, 1, 0] = 1.0                       # var (1/l)(1-1/l)
    f = feats_of(np.zeros((1, 8), np.float32), probs=p, lens=[l])
    assert f[0, 2] == np.float32(0.5 * (1 / l) * (1 - 1 / l))


def test_feature_vector_layout_is_H_R_V_C():
    z = np.zeros((1, 16), np.float32)
    z[0, 0] = 1.0
    p = np.zeros((1, 1, 4))
    p[0, 0, 0] = 1.0
    f = feats_of(z, ids=[2], counts=np.array([0, 0, 9] + [0] * 13), N=9, Vobs=1, probs=p, lens=[4])
    Z = math.e + 15
    assert f[0, 0] == pytest.approx(math.log(Z) - math.e / Z, rel=1e-6)
    assert f[0, 1] == pytest.approx(-math.log(10 / 11), rel=1e-6)
    assert f[0, 2] == pytest.approx(0.25 * 0.75, rel=1e-6)
    assert f[0, 3] == pytest.approx(math.e / Z, rel=1e-6)


# ---------------------------------------------------------------- controller

def xavier(out_f, in_f, rng):
    a = math.sqrt(6.0 / (in_f + out_f))
    return rng.uniform(-a, a, (out_f, in_f)).astype(np.float32)


@pytest.mark.parametrize("dims", [(4, 32, 32, 4), (4, 64, 4), (4, 128, 128, 4)])
def test_controller_equals_a_torch_linear_relu_stack_in_fp64(dims):
    rng = np.random.default_rng(sum(dims))
    Ws = [xavier(dims[i + 1], dims[i], rng) for i in range(len(dims) - 1)]
    bs = [rng.standard_normal(dims[i + 1]).astype(np.float32) * 0.1 for i in range(len(dims) - 1)]
    feats = rng.standard_normal((200, 4)).astype(np.float32) * np.array([3, 4, 1e-3, 0.3], np.float32)
    bits, logits = oracle.controller(feats, Ws, bs)
    x = torch.from_numpy(feats).double()
    for i, (W, b) in enumerate(zip(Ws, bs)):
        x = torch.nn.functional.linear(x, torch.from_numpy(W).double(), torch.from_numpy(b).double())
        if i + 1 < len(Ws):
            x = torch.relu(x)
    np.testing.assert_allclose(logits, x.numpy(), rtol=1e-12, atol=1e-13)
    want_bits = np.array([2, 4, 8, 16], np.uint8)[x.argmax(dim=1).numpy()]
    np.testing.assert_array_equal(bits, want_bits)
    assert len(set(bits.tolist())) >= 2


def test_controller_hand_built_weights_select_class_by_thresholds_on_one_feature():
    # hidden layer 1 copies feature 1 (and its negation), layer 2 copies; output k = -(x - k)^2-like ordering made
    # from piecewise linear pieces: logit_k = k*x - k^2/2 is maximal for the k nearest to x (k = 0..3)
    W1 = np.zeros((2, 4), np.float32)
    W1[0, 1], W1[1, 1] = 1.0, -1.0
    b1 = np.zeros(2, np.float32)
    W2 = np.eye(2, dtype=np.float32)
    b2 = np.zeros(2, np.float32)
    W3 = np.array([[0, 0], [1, -1], [2, -2], [3, -3]], np.float32)     # k * (relu(x) - relu(-x)) = k*x
    b3 = np.array([0, -0.5, -2.0, -4.5], np.float32)
    xs = np.array([-5.0, 0.2, 0.7, 1.4, 1.6, 2.4, 2.6, 9.0], np.float32)
    feats = np.zeros((len(xs), 4), np.float32)
    feats[:, 1] = xs
    feats[:, 0] = 100.0                                               # ignored by W1
    bits, logits = oracle.controller(feats, [W1, W2, W3], [b1, b2, b3])
    assert list(bits) == [2, 2, 4, 4, 8, 8, 16, 16]
    np.testing.assert_allclose(logits[3], [0, 1.4 - 0.5, 2.8 - 2.0, 4.2 - 4.5], rtol=1e-6)


def test_controller_zero_weights_follow_the_bias_and_ties_go_to_the_lowest_class():
    Ws = [np.zeros((8, 4), np.float32), np.zeros((4, 8), np.float32)]
    feats = np.random.default_rng(5).standard_normal((5, 4)).astype(np.float32)
    bits, _ = oracle.controller(feats, Ws, [np.zeros(8, np.float32), np.array([0.1, 0.7, 0.3, 0.2], np.float32)])
    assert list(bits) == [4] * 5
    bits, _ = oracle.controller(feats, Ws, [np.zeros(8, np.float32), np.array([0.5, 0.5, 0.5, 0.5], np.float32)])
    assert list(bits) == [2] * 5
    bits, _ = oracle.controller(feats, Ws, [np.zeros(8, np.float32), np.array([0.1, 0.2, 0.9, 0.9], np.float32)])
    assert list(bits) == [8] * 5


def test_controller_relu_is_applied_to_hidden_layers_only_and_hidden_permutation_is_irrelevant():
    rng = np.random.default_rng(6)
    Ws = [xavier(16, 4, rng), xavier(16, 16, rng), xavier(4, 16, rng)]
    bs = [rng.standard_normal(16).astype(np.float32), rng.standard_normal(16).astype(np.float32),
          -5.0 + rng.standard_normal(4).astype(np.float32)]
    feats = rng.standard_normal((50, 4)).astype(np.float32)
    bits, logits = oracle.controller(feats, Ws, bs)
    assert (logits < 0).any()                                         # no ReLU on the output layer
    perm = rng.permutation(16)
    Wp = [Ws[0][perm], Ws[1][:, perm], Ws[2]]
    bp = [bs[0][perm], bs[1], bs[2]]
    bits_p, logits_p = oracle.controller(feats, Wp, bp)
    np.testing.assert_allclose(logits_p, logits, rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(bits_p, bits)
    # dropping the ReLU would change the result: the network is not accidentally linear on these inputs
    lin = feats.astype(np.float64)
    for W, b in zip(Ws, bs):
        lin = lin @ W.astype(np.float64).T + b
    assert np.max(np.abs(lin - logits)) > 1e-2


def test_rule_policy_counts_the_thresholds_a_linear_score_exceeds():
    rng = np.random.default_rng(17)
    feats = (rng.standard_normal((500, 4)) * np.array([3, 4, 1e-3, 0.3])).astype(np.float32)
    w = np.array([0.25, 0.5, 100.0, -1.0], np.float32)
    thr = np.array([-0.5, 0.4, 1.7], np.float32)
    bits, score = oracle.rule_policy(feats, w, 0.125, thr)
    want_score = 0.125 + feats.astype(np.float64) @ w.astype(np.float64)
    np.testing.assert_allclose(score, want_score, rtol=1e-14, atol=1e-14)
    # class = number of thresholds strictly below the score: a library binary search gives the same count
    want_cls = np.searchsorted(thr.astype(np.float64), want_score, side="left")
    assert np.array_equal(bits, np.array([2, 4, 8, 16], np.uint8)[want_cls])
    # hand cases: a score equal to a threshold does not exceed it; only feature 1 matters with w = e_1
    f = np.zeros((5, 4), np.float32)
    f[:, 1] = [-1.0, 0.0, 0.5, 1.0, 2.5]
    b, _ = oracle.rule_policy(f, np.array([0, 1, 0, 0], np.float32), 0.0, np.array([0.0, 0.5, 2.0], np.float32))
    assert b.tolist() == [2, 2, 4, 8, 16]
    # monotone in the score: raising the bias never lowers a width
    b_hi, _ = oracle.rule_policy(feats, w, 1.0, thr)
    assert np.all(b_hi >= bits)
