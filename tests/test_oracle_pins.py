"""Pins for the CPU oracle: facts fixed by the paper and by mathematics, none by the oracle itself.

The paper prints no worked numeric example, so the pins are invariants (exact
inversion, Sec. 3.1/3.2), finite differences of the scalar <Y1,dY1>+<Y2,dY2>,
equality of the reversible and stored-activation routes (Sec. 3.2), an
independent autograd evaluation with library routines, closed forms and special
cases.  Each test names the mistake it is meant to catch.
"""
import math

import numpy as np
import pytest
import torch

from oracle import rev_oracle as O
from paper_2306_09342_amd import synth

EPS = 1e-6


def _setup(name="tiny", seed=0, perturb=True, **over):
    cfg = dict(synth.CONFIGS[name])
    cfg.update(over)
    cfg["mode"] = "fp32"
    flat = synth.make_params(cfg, seed=seed, perturb=perturb).astype(np.float64)
    blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
    x, dy1, dy2 = (a.astype(np.float64) for a in synth.make_inputs(cfg, seed=seed))
    return cfg, blocks, x, dy1, dy2


def _scale_weights(blocks, s):
    for p in blocks:
        for k in p:
            if k.startswith("w_"):
                p[k] = p[k] * s
    return blocks


def _rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


# ---------------------------------------------------------------- inversion
@pytest.mark.parametrize("wscale", [1.0, 8.0])
def test_inverse_reconstructs_inputs(wscale):
    """Sec. 3.1/3.2: inputs are recovered exactly from outputs.  Catches a wrong
    inverse order (X1 must use the reconstructed X2) or a sign slip."""
    cfg, blocks, x, _, _ = _setup()
    _scale_weights(blocks, wscale)
    x1 = x
    x2 = x[::-1].copy()                     # different streams, so a swap shows
    y1, y2 = O.stack_forward(x1, x2, blocks, cfg["n_heads"], EPS)
    assert _rel(y1, x1) > 1e-3              # the stack is not the identity
    r1, r2 = O.stack_inverse(y1, y2, blocks, cfg["n_heads"], EPS)
    assert np.abs(r1 - x1).max() < 1e-12
    assert np.abs(r2 - x2).max() < 1e-12


def test_inverse_per_depth_and_big_shape_sample():
    cfg, blocks, x, _, _ = _setup()
    H = cfg["n_heads"]
    a, b = x, x
    for p in blocks:
        y1, y2 = O.block_forward(a, b, p, H, EPS)
        r1, r2 = O.block_inverse(y1, y2, p, H, EPS)
        assert np.abs(r1 - a).max() < 1e-13 and np.abs(r2 - b).max() < 1e-13
        a, b = y1, y2
    # one sample of a ViT-S-shaped stack, two blocks deep
    cfg, blocks, x, _, _ = _setup("vit_s", n_blocks=2, batch=1)
    y1, y2 = O.stack_forward(x, x, blocks, cfg["n_heads"], EPS)
    r1, r2 = O.stack_inverse(y1, y2, blocks, cfg["n_heads"], EPS)
    assert np.abs(r1 - x).max() < 1e-12 and np.abs(r2 - x).max() < 1e-12


def test_inverse_costs_one_F_and_one_G():
    """Sec. 3.1: the inverse needs exactly one call of F and one of G per block,
    and the reversible backward adds no further branch evaluation."""
    cfg, blocks, x, dy1, dy2 = _setup()
    H = cfg["n_heads"]
    y1, y2 = O.stack_forward(x, x, blocks, H, EPS)
    O.CALLS.update(F=0, G=0)
    O.stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, EPS)
    assert O.CALLS == {"F": cfg["n_blocks"], "G": cfg["n_blocks"]}


# ------------------------------------------------------- finite differences
def _loss(x1, x2, blocks, H, dy1, dy2):
    y1, y2 = O.stack_forward(x1, x2, blocks, H, EPS)
    return float((y1 * dy1).sum() + (y2 * dy2).sum())


@pytest.mark.parametrize("wscale", [1.0, 10.0])
def test_backward_matches_central_finite_differences(wscale):
    """Independent of every hand-derived backward formula: random directional
    derivatives and single coordinates of L = <Y1,dY1> + <Y2,dY2>."""
    cfg, blocks, x, dy1, dy2 = _setup(n_blocks=2, batch=2, seq_len=5)
    _scale_weights(blocks, wscale)
    H = cfg["n_heads"]
    rng = np.random.default_rng(123)
    x1 = x
    x2 = x + 0.3 * rng.standard_normal(x.shape)
    dx1, dx2, grads = O.stack_backward_stored(x1, x2, blocks, H, dy1, dy2, EPS)
    h = 1e-5

    def check(fd, an, what):
        # absolute floor: rounding noise of the two loss values (|L| ~ 1e2..1e3) over 2h
        assert abs(fd - an) <= 2e-7 * max(abs(an), abs(fd)) + 3e-8, (what, fd, an)

    # inputs: directional + coordinates
    for which, g in (("x1", dx1), ("x2", dx2)):
        for trial in range(3):
            d = rng.standard_normal(x.shape)
            if trial == 2:                      # a single coordinate
                d = np.zeros(x.shape)
                d.flat[rng.integers(d.size)] = 1.0
            a1, a2 = (x1 + h * d, x2) if which == "x1" else (x1, x2 + h * d)
            b1, b2 = (x1 - h * d, x2) if which == "x1" else (x1, x2 - h * d)
            fd = (_loss(a1, a2, blocks, H, dy1, dy2) - _loss(b1, b2, blocks, H, dy1, dy2)) / (2 * h)
            check(fd, float((g * d).sum()), which)
    # every parameter tensor of every block
    for bi, p in enumerate(blocks):
        for name in list(p):
            for trial in range(2):
                d = rng.standard_normal(p[name].shape)
                if trial == 1:
                    d = np.zeros(p[name].shape)
                    d.flat[rng.integers(d.size)] = 1.0
                keep = p[name]
                p[name] = keep + h * d
                lp = _loss(x1, x2, blocks, H, dy1, dy2)
                p[name] = keep - h * d
                lm = _loss(x1, x2, blocks, H, dy1, dy2)
                p[name] = keep
                check((lp - lm) / (2 * h), float((grads[bi][name] * d).sum()), (bi, name))


# ----------------------------------------------- reversible == stored route
@pytest.mark.parametrize("wscale", [1.0, 8.0])
def test_reversible_route_equals_stored_route(wscale):
    """Sec. 3.2: recomputing activations changes nothing about the gradients."""
    cfg, blocks, x, dy1, dy2 = _setup()
    _scale_weights(blocks, wscale)
    H = cfg["n_heads"]
    x2 = x[:, ::-1].copy()
    sdx1, sdx2, sg = O.stack_backward_stored(x, x2, blocks, H, dy1, dy2, EPS)
    y1, y2 = O.stack_forward(x, x2, blocks, H, EPS)
    rdx1, rdx2, rg, r1, r2 = O.stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, EPS)
    assert _rel(rdx1, sdx1) < 1e-10 and _rel(rdx2, sdx2) < 1e-10
    assert np.abs(r1 - x).max() < 1e-12 and np.abs(r2 - x2).max() < 1e-12
    for a, b in zip(rg, sg):
        for k in b:
            assert _rel(a[k], b[k]) < 1e-10, k
    # the chunked walk is the same sum over samples
    cdx1, cdx2, cg, _, _ = O.stack_backward_reversible_chunked(y1, y2, blocks, H, dy1, dy2, EPS, chunk=3)
    assert _rel(cdx1, sdx1) < 1e-10 and _rel(cdx2, sdx2) < 1e-10
    for a, b in zip(cg, sg):
        for k in b:
            assert _rel(a[k], b[k]) < 1e-10, k


# ------------------------------------- independent autograd with library ops
def _torch_stack(x1, x2, tb, H):
    Fn = torch.nn.functional
    for p in tb:
        D = x1.shape[-1]
        n = Fn.layer_norm(x2, (D,), p["ln1_g"], p["ln1_b"], EPS)
        qkv = Fn.linear(n, p["w_qkv"], p["b_qkv"])
        B, T, _ = qkv.shape
        q, k, v = (t.reshape(B, T, H, D // H).transpose(1, 2) for t in qkv.split(D, dim=-1))
        o = Fn.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, T, D)
        x1 = x1 + Fn.linear(o, p["w_proj"], p["b_proj"])
        n = Fn.layer_norm(x1, (D,), p["ln2_g"], p["ln2_b"], EPS)
        x2 = x2 + Fn.linear(Fn.gelu(Fn.linear(n, p["w_fc1"], p["b_fc1"])), p["w_fc2"], p["b_fc2"])
    return x1, x2


@pytest.mark.parametrize("wscale", [1.0, 10.0])
def test_against_library_autograd(wscale):
    """The whole map is a composition of textbook layers, so a library's own
    layer_norm / linear / attention / gelu with reverse-mode autodiff must agree.
    Catches transposed operands, head-split order, scale and GELU-form slips."""
    cfg, blocks, x, dy1, dy2 = _setup(seq_len=7, batch=3)
    _scale_weights(blocks, wscale)
    H = cfg["n_heads"]
    x2 = x[::-1].copy()
    tb = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in blocks]
    t1 = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    t2 = torch.tensor(x2, dtype=torch.float64, requires_grad=True)
    y1, y2 = _torch_stack(t1, t2, tb, H)
    oy1, oy2 = O.stack_forward(x, x2, blocks, H, EPS)
    assert _rel(oy1, y1.detach().numpy()) < 1e-12 and _rel(oy2, y2.detach().numpy()) < 1e-12
    ((y1 * torch.tensor(dy1)).sum() + (y2 * torch.tensor(dy2)).sum()).backward()
    dx1, dx2, grads, _, _ = O.stack_backward_reversible(oy1, oy2, blocks, H, dy1, dy2, EPS)
    assert _rel(dx1, t1.grad.numpy()) < 1e-10 and _rel(dx2, t2.grad.numpy()) < 1e-10
    for g, p in zip(grads, tb):
        for k in p:
            assert _rel(g[k], p[k].grad.numpy()) < 1e-10, k


# --------------------------------------------------------- closed-form facts
def test_layer_norm_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 5, 32)) * 3 + 1
    y, cache = O.layer_norm(x, np.ones(32), np.zeros(32), EPS)
    var = x.var(axis=-1)
    assert np.abs(y.mean(-1)).max() < 1e-14
    assert np.abs(y.var(-1) - var / (var + EPS)).max() < 1e-12
    g = rng.standard_normal(32)
    dy = rng.standard_normal(x.shape)
    dx, dg, db = O.layer_norm_vjp(dy, cache, g)
    # the output is invariant to shifting and (up to eps) scaling a token, so dx
    # is orthogonal to the all-ones vector and to x-hat
    assert np.abs(dx.sum(-1)).max() < 1e-12
    assert np.abs((dx * cache[0]).sum(-1)).max() < 1e-5
    assert np.allclose(db, dy.sum((0, 1))) and np.allclose(dg, (dy * cache[0]).sum((0, 1)))


def test_softmax_and_attention_facts():
    rng = np.random.default_rng(2)
    H, D, T = 2, 16, 6
    qkv = rng.standard_normal((2, T, 3 * D))
    o, cache = O.attention(qkv, H)
    P = cache[3]
    assert np.abs(P.sum(-1) - 1).max() < 1e-14 and (P > 0).all()
    # brute force, one head, python loops
    b, h, dh = 1, 1, D // H
    for t in range(T):
        q = qkv[b, t, h * dh:(h + 1) * dh]
        s = np.array([q @ qkv[b, u, D + h * dh:D + (h + 1) * dh] for u in range(T)]) / math.sqrt(dh)
        w = np.exp(s - s.max())
        w /= w.sum()
        ref = sum(w[u] * qkv[b, u, 2 * D + h * dh:2 * D + (h + 1) * dh] for u in range(T))
        assert np.abs(o[b, t, h * dh:(h + 1) * dh] - ref).max() < 1e-14
    # rows of dS sum to zero: shifting a row of scores does not change softmax
    do = rng.standard_normal(o.shape)
    dqkv = O.attention_vjp(do, cache)
    shift = qkv.copy()
    # adding a constant vector c to every key of a head shifts each score row by q.c: no change in o
    shift[..., D:D + dh] += 0.7
    o2, _ = O.attention(shift, H)
    assert np.abs(o2 - o).max() < 1e-13
    assert np.abs(dqkv[..., D:D + dh].sum(axis=1)).max() < 1e-12   # hence dk sums to zero over keys


def test_single_token_attention_is_value_passthrough():
    """T = 1: P = 1, so the attention output is v and F is LN followed by two linear maps."""
    cfg, blocks, x, _, _ = _setup(seq_len=1)
    p, D = blocks[0], cfg["d_model"]
    out, _ = O.F_forward(x, p, cfg["n_heads"], EPS)
    mu = x.mean(-1, keepdims=True)
    n = (x - mu) / np.sqrt(x.var(-1, keepdims=True) + EPS) * p["ln1_g"] + p["ln1_b"]
    v = n @ p["w_qkv"][2 * D:].T + p["b_qkv"][2 * D:]
    assert np.abs(out - (v @ p["w_proj"].T + p["b_proj"])).max() < 1e-13


def test_uniform_scores_average_the_values():
    """W_q = 0, b_q = 0: every score is 0, P = 1/T, each head outputs the mean value."""
    cfg, blocks, x, _, _ = _setup()
    p, D = blocks[0], cfg["d_model"]
    p["w_qkv"][:D] = 0
    p["b_qkv"][:D] = 0
    n, _ = O.layer_norm(x, p["ln1_g"], p["ln1_b"], EPS)
    qkv = O.linear(n, p["w_qkv"], p["b_qkv"])
    o, _ = O.attention(qkv, cfg["n_heads"])
    ref = np.broadcast_to(qkv[..., 2 * D:].mean(axis=1, keepdims=True), o.shape)
    assert np.abs(o - ref).max() < 1e-14


def test_gelu_facts():
    x = np.linspace(-6, 6, 241)
    assert O.gelu(np.array(0.0)) == 0.0 and O.gelu_grad(np.array(0.0)) == 0.5
    assert np.abs(O.gelu(x) - O.gelu(-x) - x).max() < 1e-14        # Phi(x) + Phi(-x) = 1
    h = 1e-5
    fd = (O.gelu(x + h) - O.gelu(x - h)) / (2 * h)
    assert np.abs(fd - O.gelu_grad(x)).max() < 1e-9
    # exact form, not the tanh approximation: x * Phi(x) with Phi from math.erf
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x])
    assert np.abs(O.gelu(x) - ref).max() < 1e-15
    assert abs(O.gelu(np.array(1.0)) - 0.8413447460685429) < 1e-15  # Phi(1), a table value


def test_zero_output_weights_case():
    """W_proj = b_proj = W_fc2 = b_fc2 = 0: F = G = 0, so Y = X and dX = dY; the
    gradients of those two output maps are plain outer products and every other
    parameter gradient vanishes."""
    cfg, blocks, x, dy1, dy2 = _setup(n_blocks=1)
    p, H = blocks[0], cfg["n_heads"]
    for k in ("w_proj", "b_proj", "w_fc2", "b_fc2"):
        p[k] = np.zeros_like(p[k])
    x2 = x[::-1].copy()
    y1, y2 = O.stack_forward(x, x2, blocks, H, EPS)
    assert np.array_equal(y1, x) and np.array_equal(y2, x2)
    dx1, dx2, grads, _, _ = O.stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, EPS)
    assert np.array_equal(dx1, dy1) and np.array_equal(dx2, dy2)
    g = grads[0]
    D = cfg["d_model"]
    # a = gelu(LN2(y1) W1^T + b1), O = attention output, both recomputed here by hand
    n2 = (y1 - y1.mean(-1, keepdims=True)) / np.sqrt(y1.var(-1, keepdims=True) + EPS) * p["ln2_g"] + p["ln2_b"]
    hpre = n2 @ p["w_fc1"].T + p["b_fc1"]
    a = np.vectorize(lambda v: 0.5 * v * (1 + math.erf(v / math.sqrt(2))))(hpre)
    assert _rel(g["w_fc2"], np.einsum("btd,btm->dm", dy2, a)) < 1e-12
    assert _rel(g["b_fc2"], dy2.sum((0, 1))) < 1e-12
    assert _rel(g["b_proj"], dy1.sum((0, 1))) < 1e-12      # gY1 = dY1 since J_G = 0
    assert np.abs(g["w_proj"]).max() > 0
    for k in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "ln2_g", "ln2_b", "w_fc1", "b_fc1"):
        assert np.abs(g[k]).max() == 0.0, k


def test_token_permutation_equivariance_and_batch_linearity():
    """No mask and no positional term inside the stack: permuting tokens permutes
    Y and dX and leaves parameter gradients unchanged.  Samples never interact:
    parameter gradients add over samples, dX of a sample ignores the others."""
    cfg, blocks, x, dy1, dy2 = _setup(n_blocks=2)
    _scale_weights(blocks, 6.0)
    H = cfg["n_heads"]
    perm = np.random.default_rng(5).permutation(cfg["seq_len"])
    y1, y2 = O.stack_forward(x, x, blocks, H, EPS)
    dx1, dx2, grads, _, _ = O.stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, EPS)
    py1, py2 = O.stack_forward(x[:, perm], x[:, perm], blocks, H, EPS)
    assert np.abs(py1 - y1[:, perm]).max() < 1e-12
    pdx1, pdx2, pgrads, _, _ = O.stack_backward_reversible(py1, py2, blocks, H, dy1[:, perm], dy2[:, perm], EPS)
    assert _rel(pdx1, dx1[:, perm]) < 1e-11 and _rel(pdx2, dx2[:, perm]) < 1e-11
    for a, b in zip(pgrads, grads):
        for k in b:
            assert _rel(a[k], b[k]) < 1e-10, k
    acc = None
    for b in range(cfg["batch"]):
        sl = slice(b, b + 1)
        s1, s2, sg, _, _ = O.stack_backward_reversible(y1[sl], y2[sl], blocks, H, dy1[sl], dy2[sl], EPS)
        assert _rel(s1, dx1[sl]) < 1e-12 and _rel(s2, dx2[sl]) < 1e-12
        acc = O.add_grads(acc, sg)
    for a, b in zip(acc, grads):
        for k in b:
            assert _rel(a[k], b[k]) < 1e-11, k


def test_pack_unpack_roundtrip_and_layout():
    cfg = synth.CONFIGS["tiny"]
    flat = synth.make_params(cfg, seed=3, perturb=True)
    blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"], dtype=np.float32)
    assert np.array_equal(O.pack_params(blocks), flat)
    D, Dm = cfg["d_model"], cfg["d_mlp"]
    assert flat.size == cfg["n_blocks"] * (4 * D * D + 2 * D * Dm + 9 * D + Dm)
    # the generator and the oracle agree on the storage order
    assert [n for n, _ in synth.block_tensors(D, Dm)] == list(O.tensor_shapes(D, Dm))


def test_synth_recipe():
    cfg = synth.CONFIGS["tiny"]
    flat = synth.make_params(cfg, seed=0)
    p = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])[1]
    assert np.all(p["ln1_g"] == 1) and np.all(p["ln2_b"] == 0) and np.all(p["b_fc1"] == 0)
    w = p["w_fc1"]
    assert np.abs(w).max() <= 0.04 + 1e-9 and 0.015 < w.std() < 0.02
    x, dy1, dy2 = synth.make_inputs(cfg, seed=0)
    assert x.shape == (4, 16, 64) and abs(x.std() - 1) < 0.05
    assert not np.array_equal(dy1, dy2)
    # a smaller batch is a prefix of the full one
    xs, _, _ = synth.make_inputs(cfg, seed=0, batch=2)
    assert np.array_equal(xs, x[:2])
    # bf16 grid: low 16 bits are zero and rounding is to nearest
    v = np.array([1.0, 1.00390625, 1.005859375, 3.1415927], dtype=np.float32)
    r = synth.to_bf16_grid(v)
    assert np.all(r.view(np.uint32) & 0xFFFF == 0)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0078125     # tie -> even, then up
    assert np.array_equal(r, torch.tensor(v).to(torch.bfloat16).float().numpy())


# ---------------------------------------------------------------- key-padding mask
KEY_LEN = np.array([16, 9, 1, 12])          # tiny config: 4 samples of 16 tokens


def test_masked_attention_equals_attention_on_the_truncated_sequence():
    """Valid query rows see exactly what they would see if the padded keys did not exist; padded query
    rows are a softmax over the valid keys only (brute-force loop); masked probabilities are exactly 0.
    Catches masking the wrong axis (queries instead of keys), an off-by-one in the length and a finite
    'large negative' stand-in that leaks probability."""
    rng = np.random.default_rng(0)
    B, T, H, dh = 4, 16, 2, 8
    D = H * dh
    qkv = rng.standard_normal((B, T, 3 * D))
    o, (q, k, v, P, scale) = O.attention(qkv, H, KEY_LEN)
    for b, n in enumerate(KEY_LEN):
        assert np.all(P[b, :, :, n:] == 0.0)
        assert np.allclose(P[b].sum(axis=-1), 1.0, atol=1e-14)
        o_trunc, _ = O.attention(qkv[b:b + 1, :n], H)
        assert np.abs(o[b, :n] - o_trunc[0]).max() < 1e-13
        # a padded query row, by hand
        i = T - 1
        for h in range(H):
            s = np.array([q[b, h, i] @ k[b, h, j] for j in range(n)]) * scale
            w = np.exp(s - s.max())
            w /= w.sum()
            want = sum(w[j] * v[b, h, j] for j in range(n))
            assert np.abs(o[b, i, h * dh:(h + 1) * dh] - want).max() < 1e-13


def test_masked_keys_and_values_get_exactly_zero_gradient():
    rng = np.random.default_rng(1)
    B, T, H, dh = 4, 16, 2, 8
    D = H * dh
    qkv = rng.standard_normal((B, T, 3 * D))
    do = rng.standard_normal((B, T, D))
    _, cache = O.attention(qkv, H, KEY_LEN)
    dqkv = O.attention_vjp(do, cache)
    for b, n in enumerate(KEY_LEN):
        assert np.all(dqkv[b, n:, D:] == 0.0)            # dK and dV of padded positions
        if 1 < n < T:                                    # (one valid key: the softmax is constant, dQ = 0)
            assert np.abs(dqkv[b, n:, :D]).max() > 0     # padded queries still have a dQ


def test_masked_stack_equals_the_stack_on_truncated_sequences():
    """With cotangents that vanish on the padded positions, every valid-position output and every
    parameter gradient equals the computation on the truncated sequences, sample by sample."""
    cfg, blocks, x, dy1, dy2 = _setup()
    H = cfg["n_heads"]
    for b, n in enumerate(KEY_LEN):
        dy1[b, n:] = 0.0
        dy2[b, n:] = 0.0
    y1, y2 = O.stack_forward(x, x, blocks, H, EPS, key_len=KEY_LEN)
    dx1, dx2, grads, rx1, rx2 = O.stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, EPS, key_len=KEY_LEN)
    assert np.abs(rx1 - x).max() < 1e-12 and np.abs(rx2 - x).max() < 1e-12      # inversion holds under the mask
    acc = None
    for b, n in enumerate(KEY_LEN):
        xs = x[b:b + 1, :n]
        t1, t2 = O.stack_forward(xs, xs, blocks, H, EPS)
        assert np.abs(t1[0] - y1[b, :n]).max() < 1e-12 and np.abs(t2[0] - y2[b, :n]).max() < 1e-12
        a1, a2, g, _, _ = O.stack_backward_reversible(t1, t2, blocks, H, dy1[b:b + 1, :n], dy2[b:b + 1, :n], EPS)
        assert _rel(dx1[b, :n], a1[0]) < 1e-10 and _rel(dx2[b, :n], a2[0]) < 1e-10
        assert np.all(dx1[b, n:] == 0.0) and np.all(dx2[b, n:] == 0.0)
        acc = O.add_grads(acc, g)
    for gb, ab in zip(grads, acc):
        for name in gb:
            assert _rel(gb[name], ab[name]) < 1e-9, name


def test_masked_backward_matches_finite_differences_and_the_stored_route():
    cfg, blocks, x, dy1, dy2 = _setup()
    H = cfg["n_heads"]
    x2 = x[::-1].copy()
    y1, y2 = O.stack_forward(x, x2, blocks, H, EPS, key_len=KEY_LEN)
    dx1, dx2, grads, _, _ = O.stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, EPS, key_len=KEY_LEN)
    s1, s2, sg = O.stack_backward_stored(x, x2, blocks, H, dy1, dy2, EPS, key_len=KEY_LEN)
    assert _rel(dx1, s1) < 1e-10 and _rel(dx2, s2) < 1e-10

    def loss(a1, a2, bl):
        o1, o2 = O.stack_forward(a1, a2, bl, H, EPS, key_len=KEY_LEN)
        return float(np.sum(o1 * dy1) + np.sum(o2 * dy2))

    rng = np.random.default_rng(2)
    h = 1e-6
    for trial in range(3):
        d = rng.standard_normal(x.shape)
        fd = (loss(x, x2 + h * d, blocks) - loss(x, x2 - h * d, blocks)) / (2 * h)
        assert abs(fd - float(np.sum(dx2 * d))) <= 1e-6 * max(1.0, abs(fd))
    for name in ("w_qkv", "b_qkv", "w_proj", "ln1_g"):
        d = rng.standard_normal(blocks[1][name].shape)
        plus = [dict(p) for p in blocks]
        minus = [dict(p) for p in blocks]
        plus[1][name] = blocks[1][name] + h * d
        minus[1][name] = blocks[1][name] - h * d
        fd = (loss(x, x2, plus) - loss(x, x2, minus)) / (2 * h)
        an = float(np.sum(grads[1][name] * d))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), name
