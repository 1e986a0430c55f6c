"""Writes paper_2604_04722_amd/controller_calibration.json: the output-layer bias that makes the seeded Xavier
controller of each config reproduce that config's precision mix on the seeded bulk feature draw.

Calls only the oracle (controller forward in fp64) and the input generators.  Run from the repository root:
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
from paper_2604_04722_amd import workloads as wl       # noqa: E402

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


def main():
    table = {}
    for idx in (2, 3, 4):
        table[str(idx)] = calibrate(wl.CONFIGS[idx])
        print(idx, table[str(idx)])
    with open(wl.calibration_path(), "w") as f:
        json.dump(table, f, indent=1)


if __name__ == "__main__":
    main()
