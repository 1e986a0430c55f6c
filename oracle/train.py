"""CPU oracle of the controller's training step (paper Sec. 3.8 "Training Objective" and Algorithm 1).

TEST INFRASTRUCTURE ONLY, like the rest of this directory: imported by ``tests/`` only.  Plain numpy in fp64, one
statement per formula of the paper, no blocking or fusion.

What the paper fixes: the network (Sec. 3.6: Linear-ReLU-Linear-ReLU-Linear on s_t = [H, R, V, C]), the label map
{2,4,8,16} -> {0,1,2,3} (Algorithm 1), p = Softmax(o), L_ce = CrossEntropy(o, y), L_lat = mean_i sum_k p_ik c_k,
L_qual = 1 - mean_i sum_k p_ik q_k, L = alpha L_ce + beta L_lat + gamma L_qual, "update theta using Adam".
What it leaves open, and the reading taken here (all are inputs or standard choices):
  * c, q, alpha, beta, gamma and the Adam hyper-parameters are not given: they are arguments;
  * CrossEntropy is the mean over the mini-batch of -log p_{i,y_i} (the other two terms carry the same 1/B);
  * the derivative of ReLU at 0 is 0;
  * Adam is the published algorithm: m <- b1 m + (1-b1) g, v <- b2 v + (1-b2) g^2, theta <- theta - lr * (m / (1-b1^t)) /
    (sqrt(v / (1-b2^t)) + eps), t counted from 1, no weight decay.
Pins (tests/test_oracle_train.py): loss terms against closed forms and a library cross-entropy; gradients against central
finite differences of `loss` and against a library autograd in fp64; Adam against a library optimizer over several steps.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

BIT_TO_INDEX = {2: 0, 4: 1, 8: 2, 16: 3}


@dataclass
class Hyper:
    alpha: float
    beta: float
    gamma: float
    c: Sequence[float]          # latency cost of each class
    q: Sequence[float]          # quality score of each class
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8


def labels_to_classes(label_bits) -> np.ndarray:
    """Algorithm 1: bit-width labels {2,4,8,16} -> class indices {0,1,2,3}."""
    return np.array([BIT_TO_INDEX[int(b)] for b in np.asarray(label_bits).ravel()], np.int64)


def forward(feats, Ws: Sequence[np.ndarray], bs: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Sec. 3.6: activations [x, h1, (h2,) o], each [n, width], ReLU on the hidden layers only."""
    acts = [np.asarray(feats, np.float64)]
    for l, (W, b) in enumerate(zip(Ws, bs)):
        a = acts[-1] @ np.asarray(W, np.float64).T + np.asarray(b, np.float64)
        if l + 1 < len(Ws):
            a = np.maximum(a, 0.0)
        acts.append(a)
    return acts


def softmax(o: np.ndarray) -> np.ndarray:
    e = np.exp(o - o.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def loss_terms(o: np.ndarray, y: np.ndarray, hp: Hyper) -> Tuple[float, float, float, float]:
    """Sec. 3.8: (L, L_ce, L_lat, L_qual) of one mini-batch of logits o [n,4] and class labels y [n]."""
    p = softmax(o)
    n = o.shape[0]
    l_ce = float(-np.log(p[np.arange(n), y]).mean())
    l_lat = float((p @ np.asarray(hp.c, np.float64)).mean())
    l_qual = float(1.0 - (p @ np.asarray(hp.q, np.float64)).mean())
    return hp.alpha * l_ce + hp.beta * l_lat + hp.gamma * l_qual, l_ce, l_lat, l_qual


def loss(feats, y, Ws, bs, hp: Hyper) -> float:
    return loss_terms(forward(feats, Ws, bs)[-1], y, hp)[0]


def gradients(feats, y, Ws, bs, hp: Hyper):
    """dL/dW_l and dL/db_l by the chain rule, layer by layer.  Returns (gW list, gb list, loss terms)."""
    acts = forward(feats, Ws, bs)
    o = acts[-1]
    n = o.shape[0]
    p = softmax(o)
    onehot = np.zeros_like(p)
    onehot[np.arange(n), y] = 1.0
    # d/do_k of -log p_y is p_k - [k == y]; d/do_k of sum_j p_j w_j is p_k (w_k - sum_j p_j w_j)
    w = hp.beta * np.asarray(hp.c, np.float64) - hp.gamma * np.asarray(hp.q, np.float64)
    d = (hp.alpha * (p - onehot) + p * (w - (p @ w)[:, None])) / n
    gW, gb = [None] * len(Ws), [None] * len(Ws)
    for l in range(len(Ws) - 1, -1, -1):
        gW[l] = d.T @ acts[l]
        gb[l] = d.sum(axis=0)
        if l > 0:
            d = (d @ np.asarray(Ws[l], np.float64)) * (acts[l] > 0.0)
    return gW, gb, loss_terms(o, y, hp)


def adam_update(theta, g, m, v, t: int, hp: Hyper):
    """One Adam step on one tensor (t counted from 1).  Returns (theta', m', v')."""
    m = hp.beta1 * m + (1.0 - hp.beta1) * g
    v = hp.beta2 * v + (1.0 - hp.beta2) * g * g
    m_hat = m / (1.0 - hp.beta1 ** t)
    v_hat = v / (1.0 - hp.beta2 ** t)
    return theta - hp.lr * m_hat / (np.sqrt(v_hat) + hp.eps), m, v


def train_step(feats, label_bits, Ws, bs, mW, mb, vW, vb, t: int, hp: Hyper):
    """Algorithm 1, the body of the inner loop for one mini-batch.  All states are lists of fp64 arrays; returns the new
    (Ws, bs, mW, mb, vW, vb), the gradients (gW, gb) and the loss terms (L, L_ce, L_lat, L_qual) before the update."""
    y = labels_to_classes(label_bits)
    gW, gb, terms = gradients(feats, y, Ws, bs, hp)
    nW, nb, nmW, nmb, nvW, nvb = [], [], [], [], [], []
    for l in range(len(Ws)):
        th, m_, v_ = adam_update(np.asarray(Ws[l], np.float64), gW[l], mW[l], vW[l], t, hp)
        nW.append(th); nmW.append(m_); nvW.append(v_)
        th, m_, v_ = adam_update(np.asarray(bs[l], np.float64), gb[l], mb[l], vb[l], t, hp)
        nb.append(th); nmb.append(m_); nvb.append(v_)
    return (nW, nb, nmW, nmb, nvW, nvb), (gW, gb), terms
