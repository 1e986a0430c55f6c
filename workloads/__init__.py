"""Seeded synthetic inputs shaped like the paper's workloads (SmolLM-135M/360M/1.7B decoding).

This module only draws random numbers and shapes them.  It contains none of the method's arithmetic
(no softmax, no entropy, no MLP forward, no quantizer, no attention), so that the HIP path and the
CPU oracle can both be fed from it without sharing any computation.  Every tensor is a pure function
of (config index, sub-stream key): the same call gives the same data in the tests and in the bench.

The paper evaluates on benchmark contexts (HellaSwag / OpenBookQA / ARC-Challenge) run through
SmolLM weights; neither is available here, so K/V/q/logits with the stated distributions stand in
for them.  No benchmark item is used or reproduced.
"""
from __future__ import annotations

import dataclasses
import math
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

VOCAB = 49152
HEAD_DIM = 64
BIT_CHOICES = (2, 4, 8, 16)


@dataclasses.dataclass(frozen=True)
class Config:
    index: int                 # 1..5
    name: str
    n_layers: int
    batch: int
    context: int               # tokens per sequence (maximum, for the ragged config)
    n_q_heads: int
    n_kv_heads: int
    kv_kind: str               # "outlier4x10" | "student_t3"
    bits_kind: str             # "uniform" | "controller" | "runs"
    mix: Tuple[float, float, float, float]   # target share of 2/4/8/16-bit tokens
    mlp_dims: Tuple[int, ...]
    logits_sigma: float
    min_context: int = 0       # ragged lower bound (config 5)


CONFIGS: Dict[int, Config] = {
    1: Config(1, "smollm135m-1layer-ctx512", 1, 1, 512, 9, 3, "outlier4x10", "uniform",
              (0.25, 0.25, 0.25, 0.25), (4, 32, 32, 4), 1.0),
    2: Config(2, "smollm135m-30layer-ctx2048", 30, 1, 2048, 9, 3, "outlier4x10", "controller",
              (0.25, 0.25, 0.25, 0.25), (4, 64, 4), 2.0),
    3: Config(3, "smollm360m-b16-ctx4096", 32, 16, 4096, 15, 5, "student_t3", "controller",
              (0.40, 0.30, 0.20, 0.10), (4, 128, 128, 4), 2.0),
    4: Config(4, "smollm1.7b-b32-ctx8192", 24, 32, 8192, 32, 32, "outlier4x10", "controller",
              (0.50, 0.25, 0.15, 0.10), (4, 128, 128, 4), 2.0),
    5: Config(5, "smollm1.7b-b64-ctx32768-ragged", 24, 64, 32768, 32, 32, "outlier4x10", "runs",
              (0.70, 0.20, 0.08, 0.02), (4, 128, 128, 4), 2.0, min_context=8192),
}

BYTES_PER_TOKEN_HEAD = {2: 40, 4: 72, 8: 136, 16: 256}    # K+V codes plus fp16 (scale, min) pairs


def seed_for(cfg_index: int, *key: int) -> int:
    """Seed of one sub-stream: 4722*10 + config index, mixed with the key (layer, tensor tag, ...)."""
    s = 4722 * 10 + cfg_index
    for k in key:
        s = (s * 1000003 + int(k) + 12345) % (2 ** 63 - 1)
    return s


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


# tensor tags for sub-streams
_TAG_K, _TAG_V, _TAG_Q, _TAG_CH, _TAG_LOGITS, _TAG_IDS, _TAG_BITS, _TAG_MLP, _TAG_FEAT, _TAG_LEN, _TAG_PERM = range(11)


def channel_multipliers(cfg: Config, layer: int, which: int, device="cpu") -> torch.Tensor:
    """[Hkv, 64] fp32 per-channel scale: four outlier channels x10, or |Student-t(3)| clipped to [0.1, 50]."""
    g = _gen("cpu", seed_for(cfg.index, _TAG_CH, layer, which))
    if cfg.kv_kind == "outlier4x10":
        m = torch.ones(cfg.n_kv_heads, HEAD_DIM)
        for h in range(cfg.n_kv_heads):
            idx = torch.randperm(HEAD_DIM, generator=g)[:4]
            m[h, idx] = 10.0
    elif cfg.kv_kind == "student_t3":
        # t_3 = z / sqrt(chi2_3 / 3)
        z = torch.randn(cfg.n_kv_heads, HEAD_DIM, generator=g)
        chi = (torch.randn(3, cfg.n_kv_heads, HEAD_DIM, generator=g) ** 2).sum(dim=0)
        m = (z / torch.sqrt(chi / 3.0)).abs().clamp_(0.1, 50.0)
    else:
        raise ValueError(cfg.kv_kind)
    return m.to(device)


def kv_chunk(cfg: Config, layer: int, seq0: int, n_seq: int, t0: int, T: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """K and V of tokens [t0, t0+T) of sequences [seq0, seq0+n_seq) at one layer: fp16 [n_seq, T, Hkv, 64].

    Drawn per (layer, sequence, 256-token window) so that any slice can be regenerated on its own;
    t0 and T must be multiples of 256 unless the chunk ends the context.
    """
    W = 256
    assert t0 % W == 0
    outs = []
    for which, tag in ((0, _TAG_K), (1, _TAG_V)):
        mult = channel_multipliers(cfg, layer, which, device)
        x = torch.empty((n_seq, T, cfg.n_kv_heads, HEAD_DIM), dtype=torch.float16, device=device)
        for s in range(n_seq):
            for w0 in range(0, T, W):
                w = min(W, T - w0)
                g = _gen(device, seed_for(cfg.index, tag, layer, seq0 + s, (t0 + w0) // W))
                blk = torch.randn((W, cfg.n_kv_heads, HEAD_DIM), generator=g, device=device, dtype=torch.float32)
                x[s, w0:w0 + w] = (blk[:w] * mult).to(torch.float16)
        outs.append(x)
    return outs[0], outs[1]


def kv_chunk_fast(cfg: Config, layer: int, chunk_id: int, n_seq: int, T: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Bulk variant for the full-size caches of the bench: one draw per (layer, chunk), fp16 [n_seq, T, Hkv, 64]."""
    outs = []
    for which, tag in ((0, _TAG_K), (1, _TAG_V)):
        mult = channel_multipliers(cfg, layer, which, device)
        g = _gen(device, seed_for(cfg.index, tag, layer, 1_000_000 + chunk_id))
        x = torch.randn((n_seq, T, cfg.n_kv_heads, HEAD_DIM), generator=g, device=device, dtype=torch.float32)
        outs.append((x * mult).to(torch.float16))
        del x
    return outs[0], outs[1]


def queries(cfg: Config, layer: int, step: int, n_seq: int, device) -> torch.Tensor:
    """fp16 [n_seq, Hq, 64] ~ N(0,1)."""
    g = _gen(device, seed_for(cfg.index, _TAG_Q, layer, step))
    return torch.randn((n_seq, cfg.n_q_heads, HEAD_DIM), generator=g, device=device, dtype=torch.float32).to(torch.float16)


def logits(cfg: Config, step: int, n: int, device, vocab: int = VOCAB) -> torch.Tensor:
    """fp32 [n, vocab] ~ N(0, sigma^2); "N(0,2)" in the config list is read as standard deviation 2."""
    g = _gen(device, seed_for(cfg.index, _TAG_LOGITS, step))
    return torch.randn((n, vocab), generator=g, device=device, dtype=torch.float32) * cfg.logits_sigma


def zipf_table(cfg: Config, vocab: int = VOCAB, draws: int = 1 << 20, a: float = 1.1):
    """Token statistics of a truncated Zipf stream: p(rank r) ~ r^-a over `vocab` ranks, ranks mapped to ids by a
    seeded permutation.  Returns (counts int64[vocab], N, Vobs, probs float64[vocab] indexed by id)."""
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_IDS, 0))
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    p = ranks ** (-a)
    p /= p.sum()
    perm = rng.permutation(vocab)
    probs = np.empty(vocab)
    probs[perm] = p
    ids = rng.choice(vocab, size=draws, p=probs)
    counts = np.bincount(ids, minlength=vocab).astype(np.int64)
    return counts, int(draws), int((counts > 0).sum()), probs


def zipf_ids(cfg: Config, probs: np.ndarray, step: int, n: int) -> np.ndarray:
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_IDS, 1 + step))
    return rng.choice(probs.shape[0], size=n, p=probs).astype(np.int32)


def xavier_mlp(cfg: Config, dims: Optional[Sequence[int]] = None):
    """Seeded Xavier-uniform weights U(+-sqrt(6/(in+out))), zero biases.  Returns (weights, biases) as numpy fp32."""
    dims = tuple(dims or cfg.mlp_dims)
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_MLP))
    Ws, bs = [], []
    for i in range(len(dims) - 1):
        a = math.sqrt(6.0 / (dims[i] + dims[i + 1]))
        Ws.append(rng.uniform(-a, a, (dims[i + 1], dims[i])).astype(np.float32))
        bs.append(np.zeros(dims[i + 1], np.float32))
    return Ws, bs


def bulk_features(cfg: Config, n: int, chunk: int = 0) -> np.ndarray:
    """Feature vectors for the tokens that build a cache, drawn directly instead of computed from a model's
    forward pass: H ~ U(0, ln V), R ~ U(0, 14) (the range of the rarity score for a 2^20-token stream),
    V ~ logN(-9, 1), C ~ U(0, 1).  fp32 [n, 4]."""
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_FEAT, chunk))
    f = np.empty((n, 4), np.float32)
    f[:, 0] = rng.uniform(0.0, math.log(VOCAB), n)
    f[:, 1] = rng.uniform(0.0, 14.0, n)
    f[:, 2] = rng.lognormal(-9.0, 1.0, n)
    f[:, 3] = rng.uniform(0.0, 1.0, n)
    return f


def uniform_bits(cfg: Config, n_seq: int, T: int) -> np.ndarray:
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_BITS))
    return rng.choice(np.array(BIT_CHOICES, np.uint8), size=(n_seq, T)).astype(np.uint8)


def run_bits(cfg: Config, seq: int, T: int, max_run: int = 64) -> np.ndarray:
    """Precisions clustered in runs of length U{1..max_run}, classes drawn with the config's mix."""
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_BITS, seq))
    out = np.empty(T, np.uint8)
    t = 0
    choices = np.array(BIT_CHOICES, np.uint8)
    while t < T:
        run = int(rng.integers(1, max_run + 1))
        out[t:t + run] = rng.choice(choices, p=np.array(cfg.mix))
        t += run
    return out


def ragged_lengths(cfg: Config) -> np.ndarray:
    rng = np.random.default_rng(seed_for(cfg.index, _TAG_LEN))
    if cfg.min_context <= 0:
        return np.full(cfg.batch, cfg.context, np.int32)
    return rng.integers(cfg.min_context, cfg.context + 1, cfg.batch).astype(np.int32)


def calibration_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "controller_calibration.json")


def calibrated_rule(cfg: Config):
    """(w, bias, thr) of the stand-in rule-based policy whose thresholds were set (offline, by the same script) at the
    score quantiles that give the config's precision mix on `bulk_features`."""
    import json
    with open(calibration_path()) as f:
        r = json.load(f)[str(cfg.index)]["rule"]
    return np.asarray(r["w"], np.float32), float(r["bias"]), np.asarray(r["thr"], np.float32)


def calibrated_mlp(cfg: Config):
    """Xavier weights with the output bias that was calibrated (offline, by a script next to the oracle) so that
    the controller's argmax reproduces the config's precision mix on `bulk_features`."""
    import json
    Ws, bs = xavier_mlp(cfg)
    with open(calibration_path()) as f:
        table = json.load(f)
    b3 = table[str(cfg.index)]["b_out"]
    bs[-1] = np.asarray(b3, np.float32)
    return Ws, bs
