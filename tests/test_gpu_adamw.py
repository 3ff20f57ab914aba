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
