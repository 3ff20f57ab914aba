"""Shared plumbing of the GPU parity tests: run the oracle on the CPU, the HIP
path through the C-ABI binding, and compare tensor by tensor.

Error measure (used for every tolerance in these tests): for each output tensor
(dX1, dX2, each reconstructed input, each parameter-gradient tensor of each
block) max|gpu - ref| / max|ref|.  Pure element-wise relative error is
undefined at the zeros every gradient tensor has.
Tolerances: 1e-4 in float32 mode, 3e-2 in bf16 mode.
"""
import numpy as np
import torch

from oracle import rev_oracle as O
from paper_2306_09342_amd import binding as B
from paper_2306_09342_amd import synth

TOL = {"fp32": 1e-4, "bf16": 3e-2}


def rel_err(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape
    assert np.isfinite(gpu).all(), "non-finite values from the GPU"
    return float(np.abs(gpu - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_case(cfg, seed=0, perturb=True):
    """Seeded inputs + the oracle's forward outputs (float32-rounded, fed to both sides)."""
    flat = synth.make_params(cfg, seed=seed, perturb=perturb)
    x, dy1, dy2 = synth.make_inputs(cfg, seed=seed)
    blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
    return flat, blocks, x, dy1, dy2


def oracle_forward(cfg, blocks, x1, x2, chunk=8):
    y1 = np.empty(x1.shape, np.float64)
    y2 = np.empty(x1.shape, np.float64)
    for s in range(0, x1.shape[0], chunk):
        sl = slice(s, s + chunk)
        y1[sl], y2[sl] = O.stack_forward(x1[sl].astype(np.float64), x2[sl].astype(np.float64), blocks,
                                         cfg["n_heads"], cfg.get("ln_eps", 1e-6))
    return y1, y2


def to_dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(dtype).contiguous()


def gpu_cfg(cfg):
    return B.make_cfg(**cfg)


def compare_backward(cfg, res, ref, tol, what=""):
    """res: dict of GPU tensors; ref: (dx1, dx2, grads(list of dict), x1, x2) from the oracle."""
    rdx1, rdx2, rgrads, rx1, rx2 = ref
    worst = {}
    worst["dX1"] = rel_err(res["dX1"].cpu().numpy(), rdx1)
    worst["dX2"] = rel_err(res["dX2"].cpu().numpy(), rdx2)
    if res.get("X1") is not None:
        worst["X1"] = rel_err(res["X1"].cpu().numpy(), rx1)
        worst["X2"] = rel_err(res["X2"].cpu().numpy(), rx2)
    g = O.unpack_params(res["dparams"].cpu().numpy(), cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
    for bi, (gb, rb) in enumerate(zip(g, rgrads)):
        for k in rb:
            worst[f"blk{bi}.{k}"] = rel_err(gb[k], rb[k])
    bad = {k: v for k, v in worst.items() if not v <= tol}
    assert not bad, f"{what}: over tolerance {tol}: {bad}"
    return worst
