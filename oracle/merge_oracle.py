"""CPU oracle for the stage transition of a hierarchical reversible model -- TEST INFRASTRUCTURE ONLY.

Between two stages of the reversible Swin model the paper places a "downsample
block" (Sec. 3.4; the architecture figure, panel b): the two residual streams
are first fused -- by averaging, or by a small MLP -- and the fused map then
goes through the usual patch merging.  The paper gives no formula; the readings
taken here:

  fusion         z0 = (X1 + X2) / 2                          (the averaging choice), or
                 z0 = fb_w . gelu(fa_w . [X1 | X2] + fa_b) + fb_b   (the small-MLP choice: the two
                 streams concatenated along the features, one hidden layer as wide as a stream,
                 the erf GELU of the blocks, output as wide as a stream; fa_w [C, 2C], fb_w [C, C])
  patch merging  the published one of the window-attention model the paper
                 builds on: each 2x2 neighbourhood of the token grid is
                 concatenated along the feature axis (C -> 4C), normalised by a
                 LayerNorm over the 4C features and reduced by a bias-free
                 linear map 4C -> 2C
  next stage     both streams of the next stage start from the merged map (as
                 the first stage starts from two copies of its input), so the
                 cotangent of the merged map is the sum of the cotangents of
                 the two copies.

Order of the four neighbours inside the 4C features: q = 2*dy + dx for the token
at grid position (2y' + dy, 2x' + dx); another order only permutes the columns
of the linear map.

Token storage: a stage keeps its tokens window by window (the windows are the
attention sequences): row = ((b * Hw + wy) * Ww + wx) * w*w + iy * w + ix for
the token at grid (wy*w + iy, wx*w + ix), Hw x Ww windows of w x w tokens.  The
merged map is stored the same way on the (Gh/2) x (Gw/2) grid.  Here this is
written with reshapes/transposes of whole arrays (the definition); the tests pin
it against explicit per-token loops.

float64 throughout.  Only the tests, the smoke check and the benchmark may
import this module; it shares no code with the HIP path.  Pins
(tests/test_merge_oracle_pins.py): central finite differences of every input and
parameter, per-token loops for the gather, locality (one input token reaches
exactly one output row), the adjoint identity of gather/scatter, and the
equal-streams special case; for the MLP fusion additionally a setting of its weights under which it
must reproduce the averaging variant, a hand-written token, and a library autodiff evaluation.
Not "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from .rev_oracle import gelu, gelu_grad, layer_norm, layer_norm_vjp, linear, linear_vjp

F64 = np.float64


def param_shapes(C: int, fusion: str = "average") -> dict:
    """Packed order: the patch-merging parameters, then (MLP fusion only) the fusion MLP's."""
    shapes = {"ln_g": (4 * C,), "ln_b": (4 * C,), "w": (2 * C, 4 * C)}
    if fusion == "mlp":
        shapes.update({"fa_w": (C, 2 * C), "fa_b": (C,), "fb_w": (C, C), "fb_b": (C,)})
    return shapes


def unpack_params(flat, C: int, fusion: str | None = None) -> dict:
    flat = np.asarray(flat, F64)
    if fusion is None:                                    # told apart by the length of the packed vector
        fusion = "mlp" if flat.size == 8 * C + 8 * C * C + 3 * C * C + 2 * C else "average"
    out, pos = {}, 0
    for name, shape in param_shapes(C, fusion).items():
        n = int(np.prod(shape))
        out[name] = flat[pos:pos + n].reshape(shape)
        pos += n
    assert pos == flat.size
    return out


def pack_params(p: dict) -> np.ndarray:
    keys = [k for k in ("ln_g", "ln_b", "w", "fa_w", "fa_b", "fb_w", "fb_b") if k in p]
    return np.concatenate([np.asarray(p[k], F64).ravel() for k in keys])


def fuse(X1, X2, p: dict):
    """The fused map z0 [M, C] and what its backward needs.  MLP fusion iff the MLP's parameters are in p."""
    if "fa_w" not in p:
        return 0.5 * (X1 + X2), None
    cat = np.concatenate([X1, X2], axis=-1)
    h = linear(cat, p["fa_w"], p["fa_b"])
    a = gelu(h)
    return linear(a, p["fb_w"], p["fb_b"]), (cat, h, a)


def fuse_vjp(dz0, cache, p: dict):
    """Cotangent of the fused map -> (dX1, dX2, gradients of the fusion parameters)."""
    if cache is None:
        return 0.5 * dz0, 0.5 * dz0, {}
    cat, h, a = cache
    da, dfb_w, dfb_b = linear_vjp(dz0, a, p["fb_w"])
    dh = da * gelu_grad(h)
    dcat, dfa_w, dfa_b = linear_vjp(dh, cat, p["fa_w"])
    C = dz0.shape[-1]
    return dcat[:, :C], dcat[:, C:], {"fa_w": dfa_w, "fa_b": dfa_b, "fb_w": dfb_w, "fb_b": dfb_b}


def windows_to_grid(rows, B, Gh, Gw, w):
    """[B * Gh*Gw, C] rows in window order -> [B, Gh, Gw, C]."""
    C = rows.shape[-1]
    t = rows.reshape(B, Gh // w, Gw // w, w, w, C)        # b, wy, wx, iy, ix, c
    return t.transpose(0, 1, 3, 2, 4, 5).reshape(B, Gh, Gw, C)


def grid_to_windows(grid, w):
    B, Gh, Gw, C = grid.shape
    t = grid.reshape(B, Gh // w, w, Gw // w, w, C)        # b, wy, iy, wx, ix, c
    return t.transpose(0, 1, 3, 2, 4, 5).reshape(B * Gh * Gw, C)


def gather_2x2(rows, B, Gh, Gw, w):
    """Concatenate every 2x2 neighbourhood: [B*Gh*Gw, C] -> [B*(Gh/2)*(Gw/2), 4C], both in window order."""
    C = rows.shape[-1]
    g = windows_to_grid(rows, B, Gh, Gw, w)
    t = g.reshape(B, Gh // 2, 2, Gw // 2, 2, C)           # b, y', dy, x', dx, c
    t = t.transpose(0, 1, 3, 2, 4, 5).reshape(B, Gh // 2, Gw // 2, 4 * C)   # feature = (2*dy + dx) * C + c
    return grid_to_windows(t, w)


def scatter_2x2(rows4, B, Gh, Gw, w):
    """The transpose (and inverse) of gather_2x2: [B*(Gh/2)*(Gw/2), 4C] -> [B*Gh*Gw, C]."""
    C = rows4.shape[-1] // 4
    t = windows_to_grid(rows4, B, Gh // 2, Gw // 2, w)    # b, y', x', (dy, dx, c)
    t = t.reshape(B, Gh // 2, Gw // 2, 2, 2, C).transpose(0, 1, 3, 2, 4, 5).reshape(B, Gh, Gw, C)
    return grid_to_windows(t, w)


def merge_forward(X1, X2, params, B, Gh, Gw, w, eps=1e-5, want_cache=False):
    """X1, X2: [B*Gh*Gw, C].  Returns the merged map [B*(Gh/2)*(Gw/2), 2C]."""
    X1 = np.asarray(X1, F64)
    X2 = np.asarray(X2, F64)
    C = X1.shape[-1]
    p = params if isinstance(params, dict) else unpack_params(params, C)
    z0, fuse_cache = fuse(X1, X2, p)
    z = gather_2x2(z0, B, Gh, Gw, w)
    n, ln_cache = layer_norm(z, p["ln_g"], p["ln_b"], eps)
    out = n @ p["w"].T
    if want_cache:
        return out, (n, ln_cache, fuse_cache)
    return out


def merge_backward(X1, X2, dOutA, dOutB, params, B, Gh, Gw, w, eps=1e-5):
    """Cotangents of the two copies of the merged map -> (dX1, dX2, dparams dict)."""
    C = np.asarray(X1).shape[-1]
    p = params if isinstance(params, dict) else unpack_params(params, C)
    _, (n, ln_cache, fuse_cache) = merge_forward(X1, X2, p, B, Gh, Gw, w, eps, want_cache=True)
    dout = np.asarray(dOutA, F64) + np.asarray(dOutB, F64)
    dw = dout.T @ n
    dn = dout @ p["w"]
    dz, dg, db = layer_norm_vjp(dn, ln_cache, p["ln_g"])
    dfused = scatter_2x2(dz, B, Gh, Gw, w)
    dX1, dX2, gfuse = fuse_vjp(dfused, fuse_cache, p)
    grads = {"ln_g": dg, "ln_b": db, "w": dw}
    grads.update(gfuse)
    return dX1, dX2.copy(), grads
