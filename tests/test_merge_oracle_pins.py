"""Pins of the stage-transition oracle (fusion by averaging + patch merging; paper Sec. 3.4 and the
panel (b) of its architecture figure) against things other than itself: explicit per-token loops
for the window-ordered 2x2 gather, central finite differences for every gradient, locality, the
adjoint identity of gather and scatter, and closed-form special cases."""
import numpy as np
import pytest

from oracle import merge_oracle as MO

B, GH, GW, W, C = 2, 8, 4, 2, 8          # windows of 2x2 tokens on an 8x4 grid; merged grid 4x2
EPS = 1e-5


def _row(b, y, x, Gh, Gw, w):
    """Row of grid token (y, x) of image b in window order -- written out, not via reshapes."""
    return ((b * (Gh // w) + y // w) * (Gw // w) + x // w) * w * w + (y % w) * w + (x % w)


def _inputs(seed=0):
    rng = np.random.default_rng(seed)
    M = B * GH * GW
    X1 = rng.standard_normal((M, C))
    X2 = rng.standard_normal((M, C))
    p = {"ln_g": 1.0 + 0.1 * rng.standard_normal(4 * C), "ln_b": 0.1 * rng.standard_normal(4 * C),
         "w": 0.3 * rng.standard_normal((2 * C, 4 * C))}
    dA = rng.standard_normal((M // 4, 2 * C))
    dB = rng.standard_normal((M // 4, 2 * C))
    return X1, X2, p, dA, dB


def test_gather_matches_per_token_loops():
    rng = np.random.default_rng(1)
    rows = rng.standard_normal((B * GH * GW, C))
    got = MO.gather_2x2(rows, B, GH, GW, W)
    want = np.zeros_like(got)
    for b in range(B):
        for yo in range(GH // 2):
            for xo in range(GW // 2):
                o = _row(b, yo, xo, GH // 2, GW // 2, W)
                for dy in range(2):
                    for dx in range(2):
                        q = 2 * dy + dx
                        want[o, q * C:(q + 1) * C] = rows[_row(b, 2 * yo + dy, 2 * xo + dx, GH, GW, W)]
    assert np.array_equal(got, want)


def test_window_order_round_trip_and_known_positions():
    rows = np.arange(B * GH * GW, dtype=np.float64)[:, None] * np.ones((1, 1))
    grid = MO.windows_to_grid(rows, B, GH, GW, W)
    for b, y, x in [(0, 0, 0), (0, 1, 1), (0, 2, 0), (1, 7, 3), (1, 3, 2), (0, 0, 2)]:
        assert grid[b, y, x, 0] == _row(b, y, x, GH, GW, W)
    assert np.array_equal(MO.grid_to_windows(grid, W), rows)


def test_scatter_is_the_inverse_and_the_adjoint_of_gather():
    rng = np.random.default_rng(2)
    a = rng.standard_normal((B * GH * GW, C))
    b4 = rng.standard_normal((B * GH * GW // 4, 4 * C))
    assert np.array_equal(MO.scatter_2x2(MO.gather_2x2(a, B, GH, GW, W), B, GH, GW, W), a)
    lhs = np.sum(MO.gather_2x2(a, B, GH, GW, W) * b4)
    rhs = np.sum(a * MO.scatter_2x2(b4, B, GH, GW, W))
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)


def test_forward_written_out_for_one_output_token():
    X1, X2, p, _, _ = _inputs()
    out = MO.merge_forward(X1, X2, p, B, GH, GW, W, EPS)
    b, yo, xo = 1, 2, 1
    feats = []
    for dy in range(2):
        for dx in range(2):
            r = _row(b, 2 * yo + dy, 2 * xo + dx, GH, GW, W)
            feats.append(0.5 * (X1[r] + X2[r]))
    z = np.concatenate(feats)
    mu = z.mean()
    var = ((z - mu) ** 2).mean()
    n = (z - mu) / np.sqrt(var + EPS) * p["ln_g"] + p["ln_b"]
    want = p["w"] @ n
    got = out[_row(b, yo, xo, GH // 2, GW // 2, W)]
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_one_input_token_reaches_exactly_one_output_row():
    X1, X2, p, _, _ = _inputs()
    base = MO.merge_forward(X1, X2, p, B, GH, GW, W, EPS)
    b, y, x = 0, 5, 2
    X1b = X1.copy()
    X1b[_row(b, y, x, GH, GW, W)] += 1.0
    diff = np.abs(MO.merge_forward(X1b, X2, p, B, GH, GW, W, EPS) - base).max(axis=1)
    changed = np.nonzero(diff > 0)[0]
    assert list(changed) == [_row(b, y // 2, x // 2, GH // 2, GW // 2, W)]


def _loss(X1, X2, p, dA, dB):
    out = MO.merge_forward(X1, X2, p, B, GH, GW, W, EPS)
    return float(np.sum(out * (dA + dB)))


@pytest.mark.parametrize("which", ["X1", "X2", "ln_g", "ln_b", "w"])
def test_gradients_match_central_finite_differences(which):
    X1, X2, p, dA, dB = _inputs(3)
    dX1, dX2, dp = MO.merge_backward(X1, X2, dA, dB, p, B, GH, GW, W, EPS)
    grads = {"X1": dX1, "X2": dX2, **dp}
    rng = np.random.default_rng(4)
    h = 1e-6

    def perturbed(direction, step):
        X1p, X2p, pp = X1, X2, dict(p)
        if which == "X1":
            X1p = X1 + step * direction
        elif which == "X2":
            X2p = X2 + step * direction
        else:
            pp[which] = p[which] + step * direction
        return _loss(X1p, X2p, pp, dA, dB)

    # random directions and single coordinates
    for trial in range(6):
        d = rng.standard_normal(grads[which].shape)
        if trial >= 3:
            d = np.zeros(grads[which].shape)
            d.flat[rng.integers(d.size)] = 1.0
        fd = (perturbed(d, h) - perturbed(d, -h)) / (2 * h)
        an = float(np.sum(grads[which] * d))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (which, trial, fd, an)


def test_both_streams_get_the_same_cotangent_and_half_the_fused_one():
    X1, X2, p, dA, dB = _inputs(5)
    dX1, dX2, _ = MO.merge_backward(X1, X2, dA, dB, p, B, GH, GW, W, EPS)
    assert np.array_equal(dX1, dX2)
    # the cotangent of the fused map, by differentiating with respect to a common shift of both streams
    rng = np.random.default_rng(6)
    d = rng.standard_normal(X1.shape)
    h = 1e-6
    fd = (_loss(X1 + h * d, X2 + h * d, p, dA, dB) - _loss(X1 - h * d, X2 - h * d, p, dA, dB)) / (2 * h)
    assert abs(fd - float(np.sum((dX1 + dX2) * d))) <= 1e-6 * max(1.0, abs(fd))


def test_layernorm_rows_have_the_closed_form_moments():
    X1, X2, p, _, _ = _inputs(7)
    p = dict(p, ln_g=np.ones(4 * C), ln_b=np.zeros(4 * C), w=np.eye(2 * C, 4 * C))
    _, (n, _, _) = MO.merge_forward(X1, X2, p, B, GH, GW, W, EPS, want_cache=True)
    z = MO.gather_2x2(0.5 * (X1 + X2), B, GH, GW, W)
    var = z.var(axis=1)
    assert np.allclose(n.mean(axis=1), 0.0, atol=1e-12)
    assert np.allclose(n.var(axis=1), var / (var + EPS), rtol=1e-10)


def test_input_cotangent_is_orthogonal_to_constants_per_output_row():
    # LayerNorm's backward annihilates the row mean: the four source tokens of an output row get
    # cotangents that sum to zero over their 4C features
    X1, X2, p, dA, dB = _inputs(8)
    dX1, _, _ = MO.merge_backward(X1, X2, dA, dB, p, B, GH, GW, W, EPS)
    per_row = MO.gather_2x2(dX1, B, GH, GW, W).sum(axis=1)
    assert np.allclose(per_row, 0.0, atol=1e-10)


def test_pack_unpack_round_trip():
    _, _, p, _, _ = _inputs(9)
    flat = MO.pack_params(p)
    assert flat.size == 8 * C + 8 * C * C
    q = MO.unpack_params(flat, C)
    for k in p:
        assert np.array_equal(p[k], q[k])


# ---- the small-MLP choice of the stream fusion (Sec. 3.4 names it next to averaging) -----------------------
def _mlp_inputs(seed=0):
    X1, X2, p, dA, dB = _inputs(seed)
    rng = np.random.default_rng(100 + seed)
    p = dict(p, fa_w=0.4 * rng.standard_normal((C, 2 * C)), fa_b=0.3 * rng.standard_normal(C),
             fb_w=0.4 * rng.standard_normal((C, C)), fb_b=0.3 * rng.standard_normal(C))
    return X1, X2, p, dA, dB


def test_mlp_fusion_reduces_to_averaging_for_weights_that_make_it_the_mean():
    """Hidden layer = the mean of the two streams pushed 30 up, where the GELU is the identity to 1e-190,
    output layer = identity minus 30: the fused map is the average, so everything downstream of the fusion and
    the input cotangents must agree with the averaging variant."""
    X1, X2, p, dA, dB = _inputs(11)
    half = 0.5 * np.concatenate([np.eye(C), np.eye(C)], axis=1)
    pm = dict(p, fa_w=half, fa_b=np.full(C, 30.0), fb_w=np.eye(C), fb_b=np.full(C, -30.0))
    assert np.allclose(MO.merge_forward(X1, X2, pm, B, GH, GW, W, EPS), MO.merge_forward(X1, X2, p, B, GH, GW, W, EPS),
                       rtol=1e-11, atol=1e-11)
    a1, a2, ga = MO.merge_backward(X1, X2, dA, dB, p, B, GH, GW, W, EPS)
    m1, m2, gm = MO.merge_backward(X1, X2, dA, dB, pm, B, GH, GW, W, EPS)
    assert np.allclose(m1, a1, rtol=1e-10, atol=1e-11) and np.allclose(m2, a2, rtol=1e-10, atol=1e-11)
    for k in ("ln_g", "ln_b", "w"):
        assert np.allclose(gm[k], ga[k], rtol=1e-10, atol=1e-10)
    # the output bias of the fusion shifts every fused feature by the same amount: its gradient is the column
    # sum of the fused map's cotangent, i.e. of twice the averaging variant's input cotangent
    assert np.allclose(gm["fb_b"], 2.0 * a1.sum(axis=0), rtol=1e-10, atol=1e-10)


def test_mlp_fusion_written_out_for_one_token():
    from math import erf, sqrt
    X1, X2, p, _, _ = _mlp_inputs(12)
    z0, _ = MO.fuse(X1, X2, p)
    r = 37
    cat = list(X1[r]) + list(X2[r])
    hid = []
    for i in range(C):
        hsum = p["fa_b"][i] + sum(p["fa_w"][i, k] * cat[k] for k in range(2 * C))
        hid.append(0.5 * hsum * (1.0 + erf(hsum / sqrt(2.0))))
    want = [p["fb_b"][o] + sum(p["fb_w"][o, i] * hid[i] for i in range(C)) for o in range(C)]
    assert np.allclose(z0[r], want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("which", ["X1", "X2", "ln_g", "ln_b", "w", "fa_w", "fa_b", "fb_w", "fb_b"])
def test_mlp_fusion_gradients_match_central_finite_differences(which):
    X1, X2, p, dA, dB = _mlp_inputs(13)
    dX1, dX2, dp = MO.merge_backward(X1, X2, dA, dB, p, B, GH, GW, W, EPS)
    grads = {"X1": dX1, "X2": dX2, **dp}
    rng = np.random.default_rng(14)
    h = 1e-6

    def perturbed(direction, step):
        X1p, X2p, pp = X1, X2, dict(p)
        if which == "X1":
            X1p = X1 + step * direction
        elif which == "X2":
            X2p = X2 + step * direction
        else:
            pp[which] = p[which] + step * direction
        return _loss(X1p, X2p, pp, dA, dB)

    for trial in range(6):
        d = rng.standard_normal(grads[which].shape)
        if trial >= 3:
            d = np.zeros(grads[which].shape)
            d.flat[rng.integers(d.size)] = 1.0
        fd = (perturbed(d, h) - perturbed(d, -h)) / (2 * h)
        an = float(np.sum(grads[which] * d))
        assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (which, trial, fd, an)


def test_mlp_fusion_against_a_library_autodiff_evaluation():
    """The same transition from a library's own layers (linear, gelu, layer_norm) and reverse-mode autodiff in
    float64; the gather is done by explicit index lists built from the per-token row formula."""
    import torch
    import torch.nn.functional as F
    X1, X2, p, dA, dB = _mlp_inputs(15)
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    x1 = torch.tensor(X1, dtype=torch.float64, requires_grad=True)
    x2 = torch.tensor(X2, dtype=torch.float64, requires_grad=True)
    z0 = F.linear(F.gelu(F.linear(torch.cat([x1, x2], dim=1), t["fa_w"], t["fa_b"])), t["fb_w"], t["fb_b"])
    idx = np.zeros((B * GH * GW // 4, 4), dtype=np.int64)
    for b in range(B):
        for yo in range(GH // 2):
            for xo in range(GW // 2):
                o = _row(b, yo, xo, GH // 2, GW // 2, W)
                for dy in range(2):
                    for dx in range(2):
                        idx[o, 2 * dy + dx] = _row(b, 2 * yo + dy, 2 * xo + dx, GH, GW, W)
    z = torch.cat([z0[torch.from_numpy(idx[:, q])] for q in range(4)], dim=1)
    out = F.linear(F.layer_norm(z, (4 * C,), t["ln_g"], t["ln_b"], EPS), t["w"])
    assert np.allclose(out.detach().numpy(), MO.merge_forward(X1, X2, p, B, GH, GW, W, EPS), rtol=1e-11, atol=1e-11)
    (out * torch.tensor(dA + dB)).sum().backward()
    dX1, dX2, dp = MO.merge_backward(X1, X2, dA, dB, p, B, GH, GW, W, EPS)
    assert np.allclose(x1.grad.numpy(), dX1, rtol=1e-9, atol=1e-10) and np.allclose(x2.grad.numpy(), dX2, rtol=1e-9, atol=1e-10)
    for k in dp:
        assert np.allclose(t[k].grad.numpy(), dp[k], rtol=1e-9, atol=1e-10), k


def test_mlp_fusion_pack_unpack_round_trip():
    _, _, p, _, _ = _mlp_inputs(16)
    flat = MO.pack_params(p)
    assert flat.size == 8 * C + 8 * C * C + 3 * C * C + 2 * C
    q = MO.unpack_params(flat, C)
    assert list(q) == ["ln_g", "ln_b", "w", "fa_w", "fa_b", "fb_w", "fb_b"]
    for k in p:
        assert np.array_equal(p[k], q[k])
