"""GPU parity: kvq_controller_train_step against the fp64 training oracle (paper Sec. 3.8, Algorithm 1).

Tolerances.  Losses and gradients are fp32 sums of n (<= 4096) terms against fp64: relative 2e-5 of the largest
gradient entry of a tensor (+1e-9).  After an Adam step a parameter moves by lr * m_hat / (sqrt(v_hat) + eps), which
for t = 1 is lr * g / (|g| + eps): a gradient error dg moves the update by at most lr * dg / (|g| + eps), so entries whose
oracle gradient is below 1e-3 of the tensor's largest are only required to stay within 2 lr of the oracle (Adam turns
a tiny gradient of uncertain sign into a step of full size); all others within 1e-3 * lr + 2e-7 * |theta|."""
import math

import numpy as np
import pytest
import torch

from helpers import tuning, dev
from oracle import train as T
from paper_2604_04722_amd import binding as kvq

pytestmark = pytest.mark.gpu

HP = dict(alpha=1.0, beta=0.3, gamma=0.7, c=[0.2, 0.35, 0.6, 1.0], q=[0.55, 0.8, 0.95, 1.0], lr=2e-3)


def make_net(dims, seed):
    rng = np.random.default_rng(seed)
    Ws = [(rng.uniform(-1, 1, (dims[i + 1], dims[i])) * math.sqrt(3.0 / dims[i])).astype(np.float32) for i in range(len(dims) - 1)]
    bs = [rng.uniform(-0.2, 0.2, dims[i + 1]).astype(np.float32) for i in range(len(dims) - 1)]
    return Ws, bs


def make_batch(n, seed):
    rng = np.random.default_rng(seed)
    feats = (rng.standard_normal((n, 4)) * np.array([3.0, 4.0, 0.5, 0.5])).astype(np.float32)
    bits = rng.choice([2, 4, 8, 16], n).astype(np.uint8)
    return feats, bits


def flat(gW, gb):
    return np.concatenate([np.concatenate([w.reshape(-1), b.reshape(-1)]) for w, b in zip(gW, gb)])


def to_dev(arrs):
    return [torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev()) for a in arrs]


class GpuTrainer:
    def __init__(self, Ws, bs):
        self.mlp = kvq.MlpWeights(to_dev(Ws), to_dev(bs))
        self.m = kvq.MlpWeights(to_dev([np.zeros_like(w) for w in Ws]), to_dev([np.zeros_like(b) for b in bs]))
        self.v = kvq.MlpWeights(to_dev([np.zeros_like(w) for w in Ws]), to_dev([np.zeros_like(b) for b in bs]))
        self.P = kvq.kvq_controller_param_count(self.mlp)
        self.hp = kvq.make_train_hparams(**HP)

    def step(self, feats, bits, t):
        d = dev()
        ws = torch.empty(kvq.kvq_controller_train_workspace(self.mlp, feats.shape[0]), dtype=torch.uint8, device=d)
        losses = torch.zeros(4, dtype=torch.float32, device=d)
        grads = torch.zeros(self.P, dtype=torch.float32, device=d)
        kvq.kvq_controller_train_step(torch.from_numpy(feats).to(d), torch.from_numpy(bits).to(d), self.mlp, self.m, self.v,
                                      self.hp, t, ws, losses, grads)
        torch.cuda.synchronize()
        return losses.cpu().numpy(), grads.cpu().numpy()


def check_step(dims, n, seed):
    Ws, bs = make_net(dims, seed)
    feats, bits = make_batch(n, seed + 1)
    hp = T.Hyper(**HP)
    z = lambda arrs: [np.zeros(a.shape) for a in arrs]
    (oW, ob, omW, omb, ovW, ovb), (gW, gb), terms = T.train_step(feats, bits, Ws, bs, z(Ws), z(bs), z(Ws), z(bs), 1, hp)
    g = GpuTrainer(Ws, bs)
    losses, grads = g.step(feats, bits, 1)
    np.testing.assert_allclose(losses, np.array(terms), rtol=2e-5, atol=1e-6)
    # gradients, tensor by tensor
    off = 0
    for l in range(len(Ws)):
        for want, got_t, got_m, got_v, want_t, want_m, want_v, old in (
                (gW[l], g.mlp.W[l], g.m.W[l], g.v.W[l], oW[l], omW[l], ovW[l], Ws[l]),
                (gb[l], g.mlp.b[l], g.m.b[l], g.v.b[l], ob[l], omb[l], ovb[l], bs[l])):
            k = want.size
            got_g = grads[off:off + k].reshape(want.shape)
            off += k
            gmax = float(np.abs(want).max()) + 1e-30
            assert np.all(np.abs(got_g - want) <= 2e-5 * gmax + 1e-9), "gradient of layer %d" % l
            np.testing.assert_allclose(got_m.cpu().numpy(), want_m, rtol=0, atol=0.1 * (2e-5 * gmax + 1e-9))      # m = (1 - beta1) g
            np.testing.assert_allclose(got_v.cpu().numpy(), want_v, rtol=1e-4, atol=1e-10 * gmax * gmax + 1e-20)   # v = (1 - beta2) g^2
            th = got_t.cpu().numpy().astype(np.float64)
            big = np.abs(want) >= 1e-3 * gmax
            assert np.all(np.abs(th - want_t)[big] <= 1e-3 * hp.lr + 2e-7 * np.abs(want_t)[big])
            assert np.all(np.abs(th - want_t)[~big] <= 2.0 * hp.lr + 2e-7)
            # a dead unit has an exactly zero gradient and must not move at all
            dead = want == 0.0
            assert np.array_equal(th[dead].astype(np.float32), old[dead])
    assert off == g.P


# hidden widths of 32, 64 or 128 on both sides put the middle layer on the matrix cores (every tile mapping: equal and
# unequal widths, fewer tiles than wavefronts and more); other widths and two-layer networks stay on the vector ALU
@pytest.mark.parametrize("dims,n", [((4, 32, 32, 4), 64), ((4, 128, 128, 4), 1000), ((4, 64, 4), 333), ((4, 128, 128, 4), 1),
                                    ((4, 40, 24, 4), 4096), ((4, 128, 128, 4), 10000), ((4, 64, 128, 4), 777),
                                    ((4, 128, 32, 4), 2050), ((4, 32, 64, 4), 31), ((4, 128, 64, 4), 9000)])
def test_train_step_matches_the_oracle(dims, n):
    print("train step dims %s n=%d" % (dims, n), flush=True)
    check_step(dims, n, seed=sum(dims) + n)


def test_train_step_on_the_vector_alu_when_the_matrix_core_path_is_switched_off():
    print("train step 4-128-128-4, n=500, train_no_mfma=1", flush=True)
    with tuning(train_no_mfma=1):
        check_step((4, 128, 128, 4), 500, seed=99)


def test_training_run_follows_the_oracle_and_learns():
    print("200 training steps on a learnable labelling", flush=True)
    rng = np.random.default_rng(5)
    feats = rng.standard_normal((1024, 4)).astype(np.float32)
    bits = np.array([2, 4, 8, 16], np.uint8)[np.clip(np.floor(feats[:, 0] + 2).astype(int), 0, 3)]
    Ws, bs = make_net((4, 32, 32, 4), 6)
    hp = T.Hyper(**HP)
    g = GpuTrainer(Ws, bs)
    z = lambda arrs: [np.zeros(a.shape) for a in arrs]
    oW, ob, omW, omb, ovW, ovb = [w.astype(np.float64) for w in Ws], [b.astype(np.float64) for b in bs], z(Ws), z(bs), z(Ws), z(bs)
    gl, ol = [], []
    for t in range(1, 201):
        (oW, ob, omW, omb, ovW, ovb), _, terms = T.train_step(feats, bits, oW, ob, omW, omb, ovW, ovb, t, hp)
        losses, _ = g.step(feats, bits, t)
        gl.append(float(losses[0])); ol.append(terms[0])
    # the two trajectories stay together (the loss is a smooth function of the parameters) and the loss falls
    assert gl[-1] < 0.6 * gl[0] and ol[-1] < 0.6 * ol[0]
    np.testing.assert_allclose(gl[:20], ol[:20], rtol=1e-3)
    np.testing.assert_allclose(gl, ol, rtol=5e-2)
    # assignments of the trained networks agree on fresh features
    test_f = rng.standard_normal((4096, 4)).astype(np.float32)
    d = dev()
    got = torch.zeros(4096, dtype=torch.uint8, device=d)
    kvq.kvq_controller(torch.from_numpy(test_f).to(d), g.mlp, got)
    o = T.forward(test_f, oW, ob)[-1]
    want = np.array([2, 4, 8, 16])[o.argmax(axis=1)]
    assert (got.cpu().numpy() == want).mean() > 0.97


def test_train_step_argument_checks():
    Ws, bs = make_net((4, 32, 4), 1)
    g = GpuTrainer(Ws, bs)
    feats, bits = make_batch(8, 2)
    d = dev()
    small = torch.empty(16, dtype=torch.uint8, device=d)
    with pytest.raises(kvq.KvqError):
        kvq.kvq_controller_train_step(torch.from_numpy(feats).to(d), torch.from_numpy(bits).to(d), g.mlp, g.m, g.v, g.hp, 1, small)
    ws = torch.empty(kvq.kvq_controller_train_workspace(g.mlp, 8), dtype=torch.uint8, device=d)
    with pytest.raises(kvq.KvqError):
        kvq.kvq_controller_train_step(torch.from_numpy(feats).to(d), torch.from_numpy(bits).to(d), g.mlp, g.m, g.v, g.hp, 0, ws)
    other = GpuTrainer(*make_net((4, 16, 4), 3))
    with pytest.raises(kvq.KvqError):
        kvq.kvq_controller_train_step(torch.from_numpy(feats).to(d), torch.from_numpy(bits).to(d), g.mlp, other.m, g.v, g.hp, 1, ws)
    wide = GpuTrainer(*make_net((4, 200, 4), 4))
    with pytest.raises(kvq.KvqError):
        kvq.kvq_controller_train_step(torch.from_numpy(feats).to(d), torch.from_numpy(bits).to(d), wide.mlp, wide.m, wide.v, wide.hp, 1,
                                      torch.empty(1 << 20, dtype=torch.uint8, device=d))
    np.testing.assert_array_equal(g.mlp.W[0].cpu().numpy(), Ws[0])
