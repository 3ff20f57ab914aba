"""Writes tests/golden/tiny_seed0.json: a digest of the float64 oracle's results on the tiny workload
(seed 0, the benchmark's recipe).  Calls only oracle/ and the seeded input generators; nothing here
comes from the HIP path.  Run from the repository root:  python tests/golden/make_golden.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import adamw_oracle as A          # noqa: E402
from oracle import rev_oracle as O            # noqa: E402
from paper_2306_09342_amd import synth        # noqa: E402


def digest(a):
    a = np.asarray(a, np.float64).ravel()
    idx = np.linspace(0, a.size - 1, 5).astype(int)
    return {"sum": float(a.sum()), "abs_sum": float(np.abs(a).sum()), "max_abs": float(np.abs(a).max()),
            "samples": [float(a[i]) for i in idx]}


def main():
    cfg = dict(synth.CONFIGS["tiny"])
    flat = synth.make_params(cfg, seed=0)
    x, dy1, dy2 = synth.make_inputs(cfg, seed=0)
    blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
    H = cfg["n_heads"]
    x64 = x.astype(np.float64)
    y1, y2 = O.stack_forward(x64, x64, blocks, H, 1e-6)
    dx1, dx2, grads, rx1, rx2 = O.stack_backward_reversible(y1, y2, blocks, H, dy1.astype(np.float64), dy2.astype(np.float64))
    g = O.pack_params(grads)
    theta, m, v = A.adamw_step(flat.astype(np.float64), g, 0 * g, 0 * g, 1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                               weight_decay=0.01)
    out = {"_source": "float64 oracle (oracle/rev_oracle.py, oracle/adamw_oracle.py) on synth.CONFIGS['tiny'], seed 0; "
                      "written by tests/golden/make_golden.py",
           "Y1": digest(y1), "Y2": digest(y2), "dX1": digest(dx1), "dX2": digest(dx2), "dparams": digest(g),
           "X1_reconstructed": digest(rx1), "adamw_theta_step1": digest(theta)}
    for i, blk in enumerate(grads):
        for k, a in blk.items():
            out[f"block{i}.{k}"] = digest(a)
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_seed0.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main()
