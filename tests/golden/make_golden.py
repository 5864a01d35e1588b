"""Writes tests/golden/config1_chain.json: the loss and the L2 norm of every gradient of the
tiny fp32 workload (configs[0]) as the CPU checker computes them in float64.

The paper prints no worked example for the module arithmetic (it schedules opaque modules),
so there is no value of the paper's to store; this file only freezes the checker's own
result, so that an unintended change to oracle/ shows up as a diff.  It calls nothing but
oracle/ and the seeded input generator.  Run from the repository root:
    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from oracle import layers as O                      # noqa: E402
from paper_2605_18710_amd import synth              # noqa: E402
from helpers import layer_params, projector_params  # noqa: E402


def compute():
    wl = synth.WORKLOADS[0]
    vit, proj, llm = (dict(m) for m in wl["modules"])
    out = {}
    # decoupled form: every module steps on its own staged input (seeded), MSE for the decoder,
    # a seeded upstream gradient for the others
    for name, cfg in (("vit", vit), ("llm", llm)):
        T, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
        layers = [layer_params(cfg, 40000 + 100 * l) for l in range(cfg["layers"])]
        x = synth.normal(40500, (T, h))
        y, saved = O.stack_fwd(x, layers, cfg)
        if cfg["kind"] == "decoder":
            target = synth.normal(40501, (T, h))
            out[name + ".loss"] = float(O.mse_fwd(y, target))
            dy = O.mse_bwd(y, target)
        else:
            dy = synth.normal(40502, (T, h), 0.0, 2.0 / (T * h))
        dx, grads = O.stack_bwd(dy, layers, saved, cfg)
        out[name + ".y"] = float(np.sqrt((y * y).sum()))
        out[name + ".dx"] = float(np.sqrt((dx * dx).sum()))
        for l, g in enumerate(grads):
            for k, v in sorted(g.items()):
                out[f"{name}.L{l}.{k}"] = float(np.sqrt((v * v).sum()))
    p = projector_params(proj["in_dim"], proj["out_dim"], 40600)
    x = synth.normal(40601, (proj["batch"] * proj["seq"], proj["in_dim"]))
    y, s = O.projector_fwd(x, p)
    dx, g = O.projector_bwd(synth.normal(40602, y.shape), p, s)
    out["proj.y"] = float(np.sqrt((y * y).sum()))
    out["proj.dx"] = float(np.sqrt((dx * dx).sum()))
    for k, v in sorted(g.items()):
        out["proj." + k] = float(np.sqrt((v * v).sum()))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_chain.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1, sort_keys=True)
    print("wrote", path)
