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


# the small-MLP choice of the stream fusion: narrow and wide, both modes, K of the hidden layer not a multiple of 64
MLP_CASES = {
    "mlp_tiny_fp32": dict(batch=2, grid_h=8, grid_w=4, window=2, d_in=8, mode="fp32", ln_eps=1e-5, fusion="mlp"),
    "mlp_windows7_bf16": dict(batch=2, grid_h=28, grid_w=14, window=7, d_in=96, mode="bf16", ln_eps=1e-5, fusion="mlp"),
    "mlp_width192_bf16": dict(batch=5, grid_h=28, grid_w=28, window=7, d_in=192, mode="bf16", ln_eps=1e-6, fusion="mlp"),
    "mlp_width384_fp32": dict(batch=1, grid_h=14, grid_w=28, window=7, d_in=384, mode="fp32", ln_eps=1e-5, fusion="mlp"),
    "mlp_wide_bf16": dict(batch=1, grid_h=14, grid_w=14, window=7, d_in=768, mode="bf16", ln_eps=1e-5, fusion="mlp"),
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


@pytest.mark.parametrize("name", list(MLP_CASES))
def test_merge_with_mlp_fusion_matches_the_oracle(name):
    mcfg = MLP_CASES[name]
    print(f"[case] merge {name} {mcfg}", flush=True)
    flat, (X1, X2, dA, dB), out, res = _run(mcfg, seed=21)
    g = (mcfg["batch"], mcfg["grid_h"], mcfg["grid_w"], mcfg["window"])
    C = mcfg["d_in"]
    assert flat.size == 8 * C + 8 * C * C + 3 * C * C + 2 * C
    r_out = MO.merge_forward(X1, X2, flat, *g, eps=mcfg["ln_eps"])
    r_dX1, r_dX2, r_dp = MO.merge_backward(X1, X2, dA, dB, flat, *g, eps=mcfg["ln_eps"])
    assert set(r_dp) == {"ln_g", "ln_b", "w", "fa_w", "fa_b", "fb_w", "fb_b"}
    tol = TOL[mcfg["mode"]]
    got_dp = MO.unpack_params(res["dparams"].cpu().numpy(), C)
    errs = {"out": rel_err(out.cpu().numpy(), r_out), "dX1": rel_err(res["dX1"].cpu().numpy(), r_dX1),
            "dX2": rel_err(res["dX2"].cpu().numpy(), r_dX2)}
    for k in r_dp:
        errs["d" + k] = rel_err(got_dp[k], r_dp[k])
    print("[ok] " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (name, bad)
    assert not torch.equal(res["dX1"], res["dX2"]), "the MLP treats the two streams differently"


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


def test_two_stage_hierarchy_backward_matches_the_oracle_end_to_end():
    """Stage 1 stack -> transition -> stage 2 stack, forward then the whole backward (reversible
    backward of stage 2, backward of the transition fed with its two input cotangents, reversible
    backward of stage 1), every call through the C-ABI, against the same chain of oracle calls."""
    from oracle import rev_oracle as O
    images, w = 2, 2
    s1 = dict(n_blocks=2, d_model=16, n_heads=2, d_mlp=64, seq_len=w * w, batch=images * 4, mode="fp32")
    s2 = dict(n_blocks=1, d_model=32, n_heads=4, d_mlp=128, seq_len=w * w, batch=images * 1, mode="fp32")
    mcfg = dict(batch=images, grid_h=4, grid_w=4, window=w, d_in=16, mode="fp32", ln_eps=1e-5)
    p1, p2 = synth.make_params(s1, seed=1, perturb=True), synth.make_params(s2, seed=2, perturb=True)
    pm = synth.make_merge_params(mcfg, seed=3, perturb=True)
    x, _, _ = synth.make_inputs(s1, seed=1)
    _, dy1, dy2 = synth.make_inputs(s2, seed=2)
    print("[case] two-stage hierarchy, fp32", flush=True)

    # ---- oracle
    b1 = O.unpack_params(p1, s1["n_blocks"], s1["d_model"], s1["d_mlp"])
    b2 = O.unpack_params(p2, s2["n_blocks"], s2["d_model"], s2["d_mlp"])
    x64 = x.astype(np.float64)
    y1, y2 = O.stack_forward(x64, x64, b1, s1["n_heads"], 1e-6)
    rows = images * 16
    merged = MO.merge_forward(y1.reshape(rows, -1), y2.reshape(rows, -1), pm, images, 4, 4, w, eps=1e-5)
    xin2 = merged.reshape(s2["batch"], s2["seq_len"], s2["d_model"])
    z1, z2 = O.stack_forward(xin2, xin2, b2, s2["n_heads"], 1e-6)
    r_dx1, r_dx2, r_g2, _, _ = O.stack_backward_reversible(z1, z2, b2, s2["n_heads"], dy1.astype(np.float64),
                                                          dy2.astype(np.float64), 1e-6)
    m_dx1, m_dx2, r_gm = MO.merge_backward(y1.reshape(rows, -1), y2.reshape(rows, -1), r_dx1.reshape(rows // 4, -1),
                                           r_dx2.reshape(rows // 4, -1), pm, images, 4, 4, w, eps=1e-5)
    f_dx1, f_dx2, r_g1, _, _ = O.stack_backward_reversible(y1, y2, b1, s1["n_heads"], m_dx1.reshape(y1.shape),
                                                          m_dx2.reshape(y1.shape), 1e-6)

    # ---- HIP path
    c1, c2, cm = B.make_cfg(**s1), B.make_cfg(**s2), B.make_merge_cfg(**mcfg)
    P1, P2, PM = to_dev(p1), to_dev(p2), to_dev(pm)
    X = to_dev(x)
    Y1, Y2 = B.rev_stack_forward(c1, P1, X, X.clone())
    merged_g = B.rev_merge_forward(cm, PM, Y1.view(rows, -1), Y2.view(rows, -1))
    Xin2 = merged_g.view(s2["batch"], s2["seq_len"], s2["d_model"])
    Z1, Z2 = B.rev_stack_forward(c2, P2, Xin2, Xin2.clone())
    side = torch.cuda.Stream()
    res2 = B.rev_stack_backward_pareprop(c2, P2, Z1, Z2, to_dev(dy1), to_dev(dy2), side)
    resm = B.rev_merge_backward(cm, PM, Y1.view(rows, -1), Y2.view(rows, -1), res2["dX1"].view(rows // 4, -1),
                                res2["dX2"].view(rows // 4, -1))
    res1 = B.rev_stack_backward_pareprop(c1, P1, Y1, Y2, resm["dX1"].view(Y1.shape), resm["dX2"].view(Y1.shape), side)
    torch.cuda.synchronize()

    tol = TOL["fp32"]
    errs = {"merged": rel_err(merged_g.cpu().numpy(), merged), "dX1": rel_err(res1["dX1"].cpu().numpy(), f_dx1),
            "dX2": rel_err(res1["dX2"].cpu().numpy(), f_dx2)}
    gm = MO.unpack_params(resm["dparams"].cpu().numpy(), 16)
    for k in r_gm:
        errs["merge.d" + k] = rel_err(gm[k], r_gm[k])
    for name, res, ref, s in (("s1", res1, r_g1, s1), ("s2", res2, r_g2, s2)):
        g = O.unpack_params(res["dparams"].cpu().numpy(), s["n_blocks"], s["d_model"], s["d_mlp"])
        for bi, (gb, rb) in enumerate(zip(g, ref)):
            for k in rb:
                errs[f"{name}.blk{bi}.{k}"] = rel_err(gb[k], rb[k])
    worst = max(errs, key=errs.get)
    print(f"[ok] worst {worst} {errs[worst]:.2e} over {len(errs)} tensors", flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
