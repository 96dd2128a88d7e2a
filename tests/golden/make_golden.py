"""Writes tests/golden/c1_oracle.json and astl_oracle.json: digests of the oracles' outputs on the
fp32 parity case (the attention layer, and the whole layer of Eq. 4-5 around it).

Calls only ``oracle/`` and the seeded input generator.  The values are the oracle's own
(the paper prints no worked example of the layer); the file guards the oracle against
silent changes, it does not pin it to the paper.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import astl_oracle, gswa_oracle  # noqa: E402
from paper_2409_06206_amd import synth  # noqa: E402


def digest(a):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    probe = np.linspace(0, a.size - 1, 7).astype(int)
    return {"sum": float(a.sum()), "abs_sum": float(np.abs(a).sum()),
            "probe_index": probe.tolist(), "probe": a[probe].tolist()}


def compute():
    cfg = synth.CONFIGS["c1"]
    G, s = cfg["groups"][0], cfg["layers"][0]
    p = synth.layer_params(cfg["C"], cfg["heads"], G, cfg["window"], synth.LAYER_SEED0)
    x, dy = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], synth.ACT_SEED)
    kw = dict(heads=cfg["heads"], groups=G, window=cfg["window"], shift=s)
    args = (p["w_qkv"], p["b_qkv"], p["w_proj"], p["b_proj"], p["table"])
    y = gswa_oracle.forward(x, *args, **kw)
    g = gswa_oracle.backward(x, dy, *args, **kw)
    names = ("dx", "dw_qkv", "db_qkv", "dw_proj", "db_proj", "dtable")
    out = {"case": "c1: B1 16x16 C60 heads6 groups2 window8 shift4, init regime, seeds 0/100",
           "y": digest(y)}
    out.update({n: digest(v) for n, v in zip(names, g)})
    return out


def compute_astl():
    cfg = synth.CONFIGS["c1"]
    G, s, hidden = cfg["groups"][0], cfg["layers"][0], 2 * cfg["C"]
    p = synth.astl_params(cfg["C"], cfg["heads"], G, cfg["window"], hidden, synth.LAYER_SEED0, "stress")
    x, dy = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], synth.ACT_SEED)
    kw = dict(heads=cfg["heads"], groups=G, window=cfg["window"], shift=s)
    dx, g = astl_oracle.backward(x, dy, p, **kw)
    out = {"case": "whole layer on c1: B1 16x16 C60 heads6 groups2 window8 shift4 hidden120 eps1e-5, "
                   "stress regime, seeds 0/100",
           "y": digest(astl_oracle.forward(x, p, **kw)), "dx": digest(dx)}
    out.update({"d" + k: digest(v) for k, v in g.items()})
    return out


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    for name, fn in (("c1_oracle.json", compute), ("astl_oracle.json", compute_astl)):
        with open(os.path.join(here, name), "w") as f:
            json.dump(fn(), f, indent=1)
        print("wrote", os.path.join(here, name))
