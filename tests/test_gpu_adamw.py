"""GPU parity of the optimizer update (rev_adamw_step, through the C-ABI) against
the float64 oracle, element by element.

Tolerance: the kernel works in float32; each of m, v and theta comes out of a
handful of float32 operations on O(1)-conditioned expressions, so the error per
step is a few ulp (6e-8 relative) of the largest operand; 2e-6 of the tensor's
largest magnitude is asserted after 4 steps.  The bf16 copy of the weights is an
integer decision (a rounding): it must equal round-to-nearest-even of the
kernel's own float32 result, bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import adamw_oracle as A
from paper_2306_09342_amd import binding as B

from parity_util import rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-6


@pytest.mark.parametrize("n", [5, 4096, 1000003])
@pytest.mark.parametrize("with_bf16", [False, True])
def test_adamw_steps_match_the_oracle(n, with_bf16):
    print(f"[case] adamw n={n} bf16_copy={with_bf16}", flush=True)
    rng = np.random.default_rng([n, int(with_bf16)])
    theta = (0.02 * rng.standard_normal(n)).astype(np.float32)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05)
    # the float32 values of the hyper-parameters are what both sides use
    hp64 = {k: float(np.float32(x)) for k, x in hp.items()}
    master = torch.from_numpy(theta.copy()).cuda()
    m = torch.zeros_like(master)
    v = torch.zeros_like(master)
    pb = torch.empty(n, dtype=torch.bfloat16, device="cuda") if with_bf16 else None
    r_theta, r_m, r_v = theta.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, 5):
        g = rng.standard_normal(n).astype(np.float32) * np.float32(10.0 ** rng.integers(-4, 2))
        g[rng.random(n) < 0.1] = 0.0                        # exact zeros, as bias gradients of unused units have
        gd = torch.from_numpy(g).cuda()
        before = gd.clone()
        B.rev_adamw_step(master, gd, m, v, step, params_bf16=pb, **hp)
        torch.cuda.synchronize()
        assert torch.equal(gd, before), "the gradient must not be modified"
        r_theta, r_m, r_v = A.adamw_step(r_theta, g, r_m, r_v, step, lr=hp64["lr"], beta1=hp64["beta1"],
                                         beta2=hp64["beta2"], eps=hp64["eps"], weight_decay=hp64["weight_decay"])
        e = (rel_err(master.cpu().numpy(), r_theta), rel_err(m.cpu().numpy(), r_m), rel_err(v.cpu().numpy(), r_v))
        print(f"[ok] step {step}: theta {e[0]:.2e} m {e[1]:.2e} v {e[2]:.2e}", flush=True)
        assert max(e) <= TOL, (step, e)
        if with_bf16:
            assert torch.equal(pb, master.to(torch.bfloat16)), "bf16 copy is not the rounded master"


def test_adamw_rejects_bad_arguments():
    t = torch.zeros(8, device="cuda")
    with pytest.raises(B.RevError):
        B.rev_adamw_step(t, t.clone(), t.clone(), t.clone(), 0, 1e-3)          # step counter starts at 1
    with pytest.raises(B.RevError):
        B.rev_adamw_step(t, t.clone(), t.clone(), t.clone(), 1, 1e-3, beta1=1.0)


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
def test_three_training_steps_match_the_oracle_pipeline(mode):
    """Forward, reversible backward (PaReprop) and AdamW chained for three steps, each side feeding
    on its own previous step: the GPU path against oracle forward -> oracle reversible backward ->
    oracle AdamW.  In bf16 mode the oracle's stack reads the bf16-rounded copy of its float64 master
    weights, as the GPU's does of its float32 ones; the comparison is on the master weights."""
    from oracle import rev_oracle as O
    from paper_2306_09342_amd import synth
    from parity_util import TOL, make_case, to_dev, gpu_cfg

    cfg = dict(n_blocks=2, d_model=64, n_heads=2, d_mlp=128, seq_len=24, batch=3, mode=mode)
    print(f"[case] three training steps mode={mode} cfg={cfg}", flush=True)
    flat, _, x, dy1, dy2 = make_case(cfg, seed=11)
    # eps = 1e-4: the key bias has an exactly zero gradient (softmax is shift invariant), which both
    # sides reach only up to their own rounding noise (1e-9 in float32, 1e-17 in float64); AdamW divides by
    # |g| + eps, so with eps at that noise level it would turn the noise into a step of its own
    hp = dict(lr=1e-2, beta1=0.9, beta2=0.99, eps=1e-4, weight_decay=0.1)
    hp64 = {k: float(np.float32(v)) for k, v in hp.items()}
    c = gpu_cfg(cfg)
    master = to_dev(flat)                                           # float32 master weights
    params = master.clone() if mode == "fp32" else master.to(torch.bfloat16)
    m = torch.zeros_like(master)
    v = torch.zeros_like(master)
    ws = B.alloc_workspace(c)
    side = torch.cuda.Stream()
    X, dY1, dY2 = to_dev(x), to_dev(dy1), to_dev(dy2)

    r_master = flat.astype(np.float64)
    r_m, r_v = np.zeros_like(r_master), np.zeros_like(r_master)
    N, D, Dm, H = cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"], cfg["n_heads"]
    for step in range(1, 4):
        Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws)
        g = B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws)
        B.rev_adamw_step(master, g["dparams"], m, v, step, params_bf16=params if mode == "bf16" else None, **hp)
        if mode == "fp32":
            params.copy_(master)
        torch.cuda.synchronize()

        r_params = r_master if mode == "fp32" else synth.to_bf16_grid(r_master.astype(np.float32)).astype(np.float64)
        blocks = O.unpack_params(r_params, N, D, Dm)
        y1, y2 = O.stack_forward(x.astype(np.float64), x.astype(np.float64), blocks, H, 1e-6)
        _, _, grads, _, _ = O.stack_backward_reversible(y1, y2, blocks, H, dy1.astype(np.float64), dy2.astype(np.float64))
        r_g = O.pack_params(grads)
        r_master, r_m, r_v = A.adamw_step(r_master, r_g, r_m, r_v, step, lr=hp64["lr"], beta1=hp64["beta1"],
                                          beta2=hp64["beta2"], eps=hp64["eps"], weight_decay=hp64["weight_decay"])
        e = rel_err(master.cpu().numpy(), r_master)
        print(f"[ok] step {step}: master weights {e:.2e}", flush=True)
        # AdamW normalises the gradient, so a relative gradient error eps moves a weight by about lr * eps
        # of a full step; the bound is the backward tolerance of the mode
        assert e <= TOL[mode], (step, e)


@pytest.mark.parametrize("n", [7, 4096, 1000003])
@pytest.mark.parametrize("with_bf16", [False, True])
def test_sgd_steps_match_the_oracle(n, with_bf16):
    print(f"[case] sgd n={n} bf16_copy={with_bf16}", flush=True)
    rng = np.random.default_rng([n, 9, int(with_bf16)])
    theta = (0.02 * rng.standard_normal(n)).astype(np.float32)
    lr = float(np.float32(3e-2))
    master = torch.from_numpy(theta.copy()).cuda()
    pb = torch.empty(n, dtype=torch.bfloat16, device="cuda") if with_bf16 else None
    ref = theta.astype(np.float64)
    for step in range(3):
        g = rng.standard_normal(n).astype(np.float32)
        gd = torch.from_numpy(g).cuda()
        B.rev_sgd_step(master, gd, lr, params_bf16=pb)
        torch.cuda.synchronize()
        ref = A.sgd_step(ref, g, lr)
        e = rel_err(master.cpu().numpy(), ref)
        assert e <= TOL, (step, e)
        if with_bf16:
            assert torch.equal(pb, master.to(torch.bfloat16)), "bf16 copy is not the rounded master"
    t = torch.zeros(8, device="cuda")
    with pytest.raises(B.RevError):
        B.rev_sgd_step(t, t.clone(), -1.0)
