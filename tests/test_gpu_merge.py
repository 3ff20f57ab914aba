"""GPU parity of the stage transition (rev_merge_forward / rev_merge_backward, through the C-ABI)
against the float64 oracle, tensor by tensor, on the same seeded inputs.

Error measure and tolerances as for the stack: max|gpu - ref| / max|ref| per tensor, 1e-4 in float32
mode, 3e-2 in bf16 mode (the oracle then runs on the bf16-rounded parameters, so only compute error
is measured).  The case list spans one and several windows per image side, non-square grids, widths
with 2, 3, 6 and 12 register chunks per lane, and a ragged last block of the backward kernel; the
full first transition of the smallest hierarchy runs at its real size with per-row spot checks.
"""
import numpy as np
import pytest
import torch

from oracle import merge_oracle as MO
from paper_2306_09342_amd import binding as B
from paper_2306_09342_amd import synth

from parity_util import TOL, rel_err, to_dev

pytestmark = pytest.mark.gpu

CASES = {
    "tiny_fp32": dict(batch=2, grid_h=8, grid_w=4, window=2, d_in=8, mode="fp32", ln_eps=1e-5),
    "one_window_fp32": dict(batch=3, grid_h=14, grid_w=14, window=7, d_in=32, mode="fp32", ln_eps=1e-5),
    "windows7_bf16": dict(batch=2, grid_h=28, grid_w=14, window=7, d_in=96, mode="bf16", ln_eps=1e-5),
    "wide_bf16": dict(batch=1, grid_h=14, grid_w=14, window=7, d_in=768, mode="bf16", ln_eps=1e-5),
    "width192_bf16": dict(batch=5, grid_h=28, grid_w=28, window=7, d_in=192, mode="bf16", ln_eps=1e-6),
    "width384_fp32": dict(batch=1, grid_h=14, grid_w=28, window=7, d_in=384, mode="fp32", ln_eps=1e-5),
}


def _run(mcfg, seed):
    flat = synth.make_merge_params(mcfg, seed=seed, perturb=True)
    X1, X2, dA, dB = synth.make_merge_inputs(mcfg, seed=seed)
    c = B.make_merge_cfg(**mcfg)
    params = to_dev(flat, B.param_dtype(c))
    args = [to_dev(a) for a in (X1, X2, dA, dB)]
    keep = [a.clone() for a in args]
    out = B.rev_merge_forward(c, params, args[0], args[1])
    res = B.rev_merge_backward(c, params, *args)
    torch.cuda.synchronize()
    for a, k in zip(args, keep):
        assert torch.equal(a, k), "inputs must not be modified"
    return flat, (X1, X2, dA, dB), out, res


@pytest.mark.parametrize("name", list(CASES))
def test_merge_matches_the_oracle(name):
    mcfg = CASES[name]
    print(f"[case] merge {name} {mcfg}", flush=True)
    flat, (X1, X2, dA, dB), out, res = _run(mcfg, seed=11)
    g = (mcfg["batch"], mcfg["grid_h"], mcfg["grid_w"], mcfg["window"])
    r_out = MO.merge_forward(X1, X2, flat, *g, eps=mcfg["ln_eps"])
    r_dX1, r_dX2, r_dp = MO.merge_backward(X1, X2, dA, dB, flat, *g, eps=mcfg["ln_eps"])
    tol = TOL[mcfg["mode"]]
    got_dp = MO.unpack_params(res["dparams"].cpu().numpy(), mcfg["d_in"])
    errs = {"out": rel_err(out.cpu().numpy(), r_out), "dX1": rel_err(res["dX1"].cpu().numpy(), r_dX1),
            "dX2": rel_err(res["dX2"].cpu().numpy(), r_dX2)}
    for k in r_dp:
        errs["d" + k] = rel_err(got_dp[k], r_dp[k])
    print("[ok] " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (name, bad)
    assert torch.equal(res["dX1"], res["dX2"]), "both streams receive the same cotangent"


def test_two_calls_give_the_same_bits():
    mcfg = CASES["windows7_bf16"]
    _, _, out_a, res_a = _run(mcfg, seed=3)
    _, _, out_b, res_b = _run(mcfg, seed=3)
    assert torch.equal(out_a, out_b)
    for k in res_a:
        assert torch.equal(res_a[k], res_b[k]), k


def test_first_transition_of_the_smallest_hierarchy_at_full_size():
    """64 images, 56x56 tokens of width 96 -> 28x28 of width 192, the launch configuration the benchmark
    times.  The oracle finishes this size in seconds, so every tensor is compared."""
    mcfg = synth.merge_cfgs(synth.HIERARCHIES["swin_t"])[0]
    print(f"[case] merge full size {mcfg}", flush=True)
    flat, (X1, X2, dA, dB), out, res = _run(mcfg, seed=5)
    g = (mcfg["batch"], mcfg["grid_h"], mcfg["grid_w"], mcfg["window"])
    r_out = MO.merge_forward(X1, X2, flat, *g, eps=mcfg["ln_eps"])
    r_dX1, _, r_dp = MO.merge_backward(X1, X2, dA, dB, flat, *g, eps=mcfg["ln_eps"])
    tol = TOL[mcfg["mode"]]
    got_dp = MO.unpack_params(res["dparams"].cpu().numpy(), mcfg["d_in"])
    errs = {"out": rel_err(out.cpu().numpy(), r_out), "dX1": rel_err(res["dX1"].cpu().numpy(), r_dX1)}
    for k in r_dp:
        errs["d" + k] = rel_err(got_dp[k], r_dp[k])
    print("[ok] " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= tol for v in errs.values()), errs


def test_merge_rejects_bad_arguments():
    c = B.make_merge_cfg(1, 14, 14, 7, 32, "fp32")
    p = torch.zeros(B.rev_merge_param_count(c), device="cuda")
    x = torch.zeros(14 * 14, 32, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.RevError):
        B.rev_merge_forward(c, p, x, x.clone(), workspace=small)
    bad = B.make_merge_cfg(1, 14, 21, 7, 32, "fp32")           # 21 is not a multiple of 2*7
    assert B.rev_merge_check_cfg(bad) < 0
