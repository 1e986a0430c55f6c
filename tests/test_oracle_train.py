"""Pins of the training-step oracle (oracle/train.py; paper Sec. 3.8 and Algorithm 1) against things other than itself:
closed forms, central finite differences, and a library's cross-entropy, autograd and Adam in fp64 on the CPU."""
import math

import numpy as np
import pytest
import torch

from oracle import train as T


def make_net(dims, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    Ws = [rng.uniform(-1, 1, (dims[i + 1], dims[i])) * scale * math.sqrt(3.0 / dims[i]) for i in range(len(dims) - 1)]
    bs = [rng.uniform(-0.2, 0.2, dims[i + 1]) for i in range(len(dims) - 1)]
    return Ws, bs


def make_batch(n, seed):
    rng = np.random.default_rng(seed)
    feats = rng.standard_normal((n, 4)) * np.array([3.0, 4.0, 0.5, 0.5])
    bits = rng.choice([2, 4, 8, 16], n)
    return feats, bits


HP = T.Hyper(alpha=1.0, beta=0.3, gamma=0.7, c=[0.2, 0.35, 0.6, 1.0], q=[0.55, 0.8, 0.95, 1.0], lr=2e-3)


def test_label_map_is_the_one_of_algorithm_1():
    assert T.labels_to_classes([2, 4, 8, 16, 16, 2]).tolist() == [0, 1, 2, 3, 3, 0]


def test_loss_terms_closed_forms_for_uniform_and_one_hot_probabilities():
    n = 7
    y = np.array([0, 1, 2, 3, 0, 1, 2])
    # all logits equal: p = 1/4 everywhere
    L, ce, lat, qual = T.loss_terms(np.zeros((n, 4)), y, HP)
    assert ce == pytest.approx(math.log(4.0), rel=1e-14)
    assert lat == pytest.approx(np.mean(HP.c), rel=1e-14) and qual == pytest.approx(1 - np.mean(HP.q), rel=1e-14)
    assert L == pytest.approx(HP.alpha * ce + HP.beta * lat + HP.gamma * qual, rel=1e-14)
    # one logit far above the others, on the label: p -> one-hot(y)
    o = np.full((n, 4), -40.0)
    o[np.arange(n), y] = 40.0
    _, ce, lat, qual = T.loss_terms(o, y, HP)
    assert ce == pytest.approx(0.0, abs=1e-12)
    assert lat == pytest.approx(np.mean(np.array(HP.c)[y]), rel=1e-12)
    assert qual == pytest.approx(1 - np.mean(np.array(HP.q)[y]), rel=1e-12)
    # ... and off the label by one class: -log p_y = 80
    _, ce, _, _ = T.loss_terms(o, (y + 1) % 4, HP)
    assert ce == pytest.approx(80.0, rel=1e-12)


def test_cross_entropy_equals_the_library_routine():
    rng = np.random.default_rng(3)
    o = rng.standard_normal((50, 4)) * 3
    y = rng.integers(0, 4, 50)
    want = float(torch.nn.functional.cross_entropy(torch.from_numpy(o), torch.from_numpy(y)))
    assert T.loss_terms(o, y, HP)[1] == pytest.approx(want, rel=1e-13)


@pytest.mark.parametrize("dims", [(4, 5, 4), (4, 6, 7, 4)])
def test_gradients_equal_central_finite_differences(dims):
    Ws, bs = make_net(dims, 11)
    feats, bits = make_batch(9, 12)
    y = T.labels_to_classes(bits)
    gW, gb, _ = T.gradients(feats, y, Ws, bs, HP)
    h = 1e-6
    for l in range(len(Ws)):
        for arr, g in ((Ws[l], gW[l]), (bs[l], gb[l])):
            flat = arr.reshape(-1)
            for i in range(flat.size):
                old = flat[i]
                flat[i] = old + h
                lp = T.loss(feats, y, Ws, bs, HP)
                flat[i] = old - h
                lm = T.loss(feats, y, Ws, bs, HP)
                flat[i] = old
                assert g.reshape(-1)[i] == pytest.approx((lp - lm) / (2 * h), rel=2e-5, abs=2e-9)


def torch_net(Ws, bs):
    return [torch.tensor(W, dtype=torch.float64, requires_grad=True) for W in Ws], \
           [torch.tensor(b, dtype=torch.float64, requires_grad=True) for b in bs]


def torch_loss(x, y, tW, tb, hp):
    a = x
    for l, (W, b) in enumerate(zip(tW, tb)):
        a = a @ W.T + b
        if l + 1 < len(tW):
            a = torch.relu(a)
    p = torch.softmax(a, dim=1)
    ce = torch.nn.functional.cross_entropy(a, y)
    lat = (p @ torch.tensor(hp.c, dtype=torch.float64)).mean()
    qual = 1 - (p @ torch.tensor(hp.q, dtype=torch.float64)).mean()
    return hp.alpha * ce + hp.beta * lat + hp.gamma * qual


@pytest.mark.parametrize("dims", [(4, 64, 4), (4, 128, 128, 4)])
def test_gradients_equal_library_autograd(dims):
    Ws, bs = make_net(dims, 21)
    feats, bits = make_batch(200, 22)
    y = T.labels_to_classes(bits)
    gW, gb, terms = T.gradients(feats, y, Ws, bs, HP)
    tW, tb = torch_net(Ws, bs)
    L = torch_loss(torch.from_numpy(feats), torch.from_numpy(y), tW, tb, HP)
    L.backward()
    assert terms[0] == pytest.approx(float(L.detach()), rel=1e-13)
    for l in range(len(Ws)):
        np.testing.assert_allclose(gW[l], tW[l].grad.numpy(), rtol=1e-10, atol=1e-15)
        np.testing.assert_allclose(gb[l], tb[l].grad.numpy(), rtol=1e-10, atol=1e-15)


def test_train_steps_equal_library_adam_over_several_steps():
    dims = (4, 32, 32, 4)
    Ws, bs = make_net(dims, 31)
    tW, tb = torch_net(Ws, bs)
    opt = torch.optim.Adam(tW + tb, lr=HP.lr, betas=(HP.beta1, HP.beta2), eps=HP.eps)
    mW = [np.zeros_like(W) for W in Ws]; vW = [np.zeros_like(W) for W in Ws]
    mb = [np.zeros_like(b) for b in bs]; vb = [np.zeros_like(b) for b in bs]
    first = None
    for t in range(1, 9):
        feats, bits = make_batch(64, 100 + t)
        (Ws, bs, mW, mb, vW, vb), _, terms = T.train_step(feats, bits, Ws, bs, mW, mb, vW, vb, t, HP)
        opt.zero_grad()
        L = torch_loss(torch.from_numpy(feats), torch.from_numpy(T.labels_to_classes(bits)), tW, tb, HP)
        L.backward()
        opt.step()
        assert terms[0] == pytest.approx(float(L.detach()), rel=1e-10)
        first = first if first is not None else terms[0]
    for l in range(len(Ws)):
        np.testing.assert_allclose(Ws[l], tW[l].detach().numpy(), rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(bs[l], tb[l].detach().numpy(), rtol=1e-9, atol=1e-12)


def test_first_adam_step_moves_every_parameter_by_lr_against_the_gradient_sign():
    # t = 1: m_hat = g, v_hat = g^2, so the update is lr * g / (|g| + eps)
    hp = T.Hyper(1.0, 0.0, 0.0, [0] * 4, [0] * 4, lr=0.01, eps=1e-12)
    g = np.array([3.0, -2.0, 1e-3, -5e-6])
    th, m, v = T.adam_update(np.zeros(4), g, np.zeros(4), np.zeros(4), 1, hp)
    np.testing.assert_allclose(th, -0.01 * np.sign(g), rtol=1e-6)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-14)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)


def test_training_lowers_the_loss_on_a_learnable_labelling():
    rng = np.random.default_rng(5)
    feats = rng.standard_normal((512, 4))
    bits = np.array([2, 4, 8, 16])[np.clip(np.floor(feats[:, 0] + 2).astype(int), 0, 3)]
    Ws, bs = make_net((4, 16, 16, 4), 6)
    hp = T.Hyper(1.0, 0.05, 0.05, HP.c, HP.q, lr=1e-2)
    mW = [np.zeros_like(W) for W in Ws]; vW = [np.zeros_like(W) for W in Ws]
    mb = [np.zeros_like(b) for b in bs]; vb = [np.zeros_like(b) for b in bs]
    losses = []
    for t in range(1, 201):
        (Ws, bs, mW, mb, vW, vb), _, terms = T.train_step(feats, bits, Ws, bs, mW, mb, vW, vb, t, hp)
        losses.append(terms[1])
    assert losses[-1] < 0.5 * losses[0]
