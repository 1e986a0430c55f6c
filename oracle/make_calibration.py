"""Writes workloads/controller_calibration.json: the output-layer bias that makes the seeded Xavier
controller of each config reproduce that config's precision mix on the seeded bulk feature draw.

Also writes, per config, the thresholds of the stand-in rule-based policy that give the same mix.
Calls only the oracle (controller forward and rule score in fp64) and the input generators.  Run from the repository root:
    python oracle/make_calibration.py
The recipe: the oracle gives the logits of the sample with zero output bias; the bias then follows
b_out += step * (target - actual) with step = mean logit standard deviation, shrunk by 0.7 every 20 rounds,
until every class is within half a point of its target; the oracle is run once more with the rounded bias
and the mix it produces is recorded.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import oracle                                          # noqa: E402
import workloads as wl       # noqa: E402

N_SAMPLE = 200_000


def calibrate(cfg):
    Ws, bs = wl.xavier_mlp(cfg)
    feats = wl.bulk_features(cfg, N_SAMPLE, chunk=0)
    target = np.asarray(cfg.mix, np.float64)
    _, logits0 = oracle.controller(feats, Ws, bs)              # zero output bias
    b = np.zeros(4, np.float64)
    step = float(logits0.std(axis=0).mean())
    for rnd in range(400):
        mix = np.bincount((logits0 + b).argmax(axis=1), minlength=4) / float(N_SAMPLE)
        if np.max(np.abs(mix - target)) < 0.005:
            break
        b += step * (target - mix)
        if rnd % 20 == 19:
            step *= 0.7
    bs[-1] = b.astype(np.float32)
    bits, _ = oracle.controller(feats, Ws, bs)
    mix = np.array([(bits == w).mean() for w in (2, 4, 8, 16)])
    return {"b_out": [float(x) for x in bs[-1]], "mix_on_sample": [float(x) for x in mix], "rounds": rnd + 1,
            "target": list(cfg.mix), "n_sample": N_SAMPLE}


RULE_W = [1.0 / float(np.log(wl.VOCAB)), 1.0 / 14.0, 50.0, -1.0]    # uncertain, rare, spread-out attention: wider; confident: narrower


def calibrate_rule(cfg):
    """Thresholds of the stand-in rule-based policy at the quantiles of its score that give the config's mix."""
    feats = wl.bulk_features(cfg, N_SAMPLE, chunk=0)
    zero = np.zeros(3, np.float32)
    _, score = oracle.rule_policy(feats, np.asarray(RULE_W, np.float32), 0.0, zero)
    thr = np.quantile(score, np.cumsum(cfg.mix)[:3]).astype(np.float32)
    bits, _ = oracle.rule_policy(feats, np.asarray(RULE_W, np.float32), 0.0, thr)
    mix = np.array([(bits == w).mean() for w in (2, 4, 8, 16)])
    return {"w": [float(np.float32(x)) for x in RULE_W], "bias": 0.0, "thr": [float(x) for x in thr],
            "mix_on_sample": [float(x) for x in mix], "target": list(cfg.mix), "n_sample": N_SAMPLE}


def main():
    table = {}
    for idx in (2, 3, 4):
        table[str(idx)] = calibrate(wl.CONFIGS[idx])
        table[str(idx)]["rule"] = calibrate_rule(wl.CONFIGS[idx])
        print(idx, table[str(idx)])
    with open(wl.calibration_path(), "w") as f:
        json.dump(table, f, indent=1)


if __name__ == "__main__":
    main()
