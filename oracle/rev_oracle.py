"""CPU oracle for the reversible transformer stack -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the HIP path computes.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product path never does.  It shares no code with the HIP kernels.

What is computed (paper Sec. 3.1, Eq. 1; Sec. 3.2):

  forward   Y1 = X1 + F(X2),  Y2 = X2 + G(Y1)           (Eq. 1, with the
            relabelling I1->X2, I2->X1, O2->Y1, O1->Y2)
  inverse   X2 = Y2 - G(Y1),  X1 = Y1 - F(X2)           (one F and one G call,
            Sec. 3.1 last paragraph)
  backward  the vector-Jacobian product of the N-block forward map with the
            cotangents (dY1, dY2): gradients of <Y1,dY1> + <Y2,dY2> with
            respect to X1, X2 and every parameter, reached either by storing
            all block inputs (ordinary backprop) or, as in Sec. 3.2, block by
            block from the top: recompute the block's inputs from its outputs,
            backpropagate through the block, drop the activations, repeat.

F is the attention branch and G the MLP branch (Sec. 3.2).  The paper does not
spell out their internals; the readings taken here: pre-LayerNorm inside each
branch (biased variance, eps a parameter, default 1e-6), multi-head softmax
attention scaled by head_dim**-0.5 with no dropout, exact (erf-based) GELU,
biases on every linear map.  No mask by default; optionally a key-padding mask
(one valid length per sample, for the variable-length text batches of the
Sec. 4.1 language experiments, which the paper does not describe): keys beyond
a sample's length get probability exactly 0 in every softmax of that sample.

Every function works on float64 arrays shaped [B, T, D] (any leading batch).
Pins (tests/test_oracle_pins.py): exact inversion, central finite differences,
reversible == stored-activation gradients, an independent autograd evaluation,
closed-form LayerNorm / softmax / GELU facts, the T=1 and uniform-attention
special cases, the zero-output-weights case, token-permutation equivariance,
batch linearity and the one-F-one-G call count; the key-padding mask against
the same computation on the truncated sequences, finite differences under the
mask and the exactly-zero key/value gradients of masked positions.  No
function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

F64 = np.float64

# number of branch evaluations, for the cost-model check (Sec. 3.1: the inverse
# needs exactly one call of F and one of G)
CALLS = {"F": 0, "G": 0}

_TENSORS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
            "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def tensor_shapes(D: int, Dm: int) -> dict:
    return {"ln1_g": (D,), "ln1_b": (D,), "w_qkv": (3 * D, D), "b_qkv": (3 * D,),
            "w_proj": (D, D), "b_proj": (D,), "ln2_g": (D,), "ln2_b": (D,),
            "w_fc1": (Dm, D), "b_fc1": (Dm,), "w_fc2": (D, Dm), "b_fc2": (D,)}


def unpack_params(flat, n_blocks: int, D: int, Dm: int, dtype=F64):
    """Split a packed parameter (or parameter-gradient) vector into per-block dicts."""
    flat = np.asarray(flat).ravel()
    shapes = tensor_shapes(D, Dm)
    blocks, off = [], 0
    for _ in range(n_blocks):
        p = {}
        for name in _TENSORS:
            n = int(np.prod(shapes[name]))
            p[name] = flat[off:off + n].reshape(shapes[name]).astype(dtype)
            off += n
        blocks.append(p)
    assert off == flat.size, "packed vector has the wrong length"
    return blocks


def pack_params(blocks) -> np.ndarray:
    return np.concatenate([b[name].ravel() for b in blocks for name in _TENSORS])


# ----------------------------------------------------------------------------
# elementary maps and their transposed Jacobians
# ----------------------------------------------------------------------------
def layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)      # biased, divides by D
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layer_norm_vjp(dy, cache, g):
    xhat, rstd = cache
    lead = tuple(range(dy.ndim - 1))
    dg = (dy * xhat).sum(axis=lead)
    db = dy.sum(axis=lead)
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True)
                 - xhat * (dxh * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def gelu_grad(x):
    cdf = 0.5 * (1.0 + erf(x / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    return cdf + x * pdf


def linear(x, w, b):
    return x @ w.T + b


def linear_vjp(dy, x, w):
    lead = tuple(range(dy.ndim - 1))
    dx = dy @ w
    dw = dy.reshape(-1, dy.shape[-1]).T @ x.reshape(-1, x.shape[-1])
    db = dy.sum(axis=lead)
    return dx, dw, db


def softmax_rows(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def _split_heads(t, H):           # [B,T,D] -> [B,H,T,dh]
    B, T, D = t.shape
    return t.reshape(B, T, H, D // H).transpose(0, 2, 1, 3)


def _merge_heads(t):              # [B,H,T,dh] -> [B,T,D]
    B, H, T, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B, T, H * dh)


def attention(qkv, H, key_len=None):
    """qkv [B,T,3D], feature order (q|k|v) then head then head_dim.

    key_len (optional, one integer per sample, 1 <= key_len[b] <= T): key-padding mask -- the keys at
    positions >= key_len[b] of sample b take no part in any softmax of that sample (score -inf, i.e.
    probability exactly 0); every query row is still computed.
    """
    D = qkv.shape[-1] // 3
    q, k, v = (_split_heads(qkv[..., i * D:(i + 1) * D], H) for i in range(3))
    scale = (D // H) ** -0.5
    S = (q @ k.transpose(0, 1, 3, 2)) * scale
    if key_len is not None:
        S = S.copy()
        for b, n in enumerate(key_len):
            S[b, :, :, int(n):] = -np.inf
    P = softmax_rows(S)
    o = _merge_heads(P @ v)
    return o, (q, k, v, P, scale)


def attention_vjp(do, cache):
    q, k, v, P, scale = cache
    H = q.shape[1]
    do = _split_heads(do, H)
    dv = P.transpose(0, 1, 3, 2) @ do
    dP = do @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dq = (dS @ k) * scale
    dk = (dS.transpose(0, 1, 3, 2) @ q) * scale
    return np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)


# ----------------------------------------------------------------------------
# the two branches (Sec. 3.2: F = attention block, G = MLP block)
# ----------------------------------------------------------------------------
def F_forward(x, p, H, eps, key_len=None):
    CALLS["F"] += 1
    n, ln = layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = linear(n, p["w_qkv"], p["b_qkv"])
    o, att = attention(qkv, H, key_len)
    return linear(o, p["w_proj"], p["b_proj"]), (n, ln, att, o)


def F_vjp(dout, cache, p):
    n, ln, att, o = cache
    do, dw_proj, db_proj = linear_vjp(dout, o, p["w_proj"])
    dqkv = attention_vjp(do, att)
    dn, dw_qkv, db_qkv = linear_vjp(dqkv, n, p["w_qkv"])
    dx, dg, db = layer_norm_vjp(dn, ln, p["ln1_g"])
    return dx, {"ln1_g": dg, "ln1_b": db, "w_qkv": dw_qkv, "b_qkv": db_qkv,
                "w_proj": dw_proj, "b_proj": db_proj}


def G_forward(x, p, eps):
    CALLS["G"] += 1
    n, ln = layer_norm(x, p["ln2_g"], p["ln2_b"], eps)
    h = linear(n, p["w_fc1"], p["b_fc1"])
    a = gelu(h)
    return linear(a, p["w_fc2"], p["b_fc2"]), (n, ln, h, a)


def G_vjp(dout, cache, p):
    n, ln, h, a = cache
    da, dw_fc2, db_fc2 = linear_vjp(dout, a, p["w_fc2"])
    dh = da * gelu_grad(h)
    dn, dw_fc1, db_fc1 = linear_vjp(dh, n, p["w_fc1"])
    dx, dg, db = layer_norm_vjp(dn, ln, p["ln2_g"])
    return dx, {"ln2_g": dg, "ln2_b": db, "w_fc1": dw_fc1, "b_fc1": db_fc1,
                "w_fc2": dw_fc2, "b_fc2": db_fc2}


# ----------------------------------------------------------------------------
# one reversible block (Eq. 1) and its inverse
# ----------------------------------------------------------------------------
def block_forward(x1, x2, p, H, eps, want_cache=False, key_len=None):
    f, cf = F_forward(x2, p, H, eps, key_len)
    y1 = x1 + f
    g, cg = G_forward(y1, p, eps)
    y2 = x2 + g
    return (y1, y2, (cf, cg)) if want_cache else (y1, y2)


def block_inverse(y1, y2, p, H, eps, want_cache=False, key_len=None):
    g, cg = G_forward(y1, p, eps)
    x2 = y2 - g
    f, cf = F_forward(x2, p, H, eps, key_len)       # uses the *reconstructed* x2
    x1 = y1 - f
    return (x1, x2, (cf, cg)) if want_cache else (x1, x2)


def block_vjp(cache, p, dy1, dy2):
    """Transposed Jacobian of one block applied to (dy1, dy2).

    From Y1 = X1 + F(X2), Y2 = X2 + G(Y1):
      gY1 = dY1 + J_G(Y1)^T dY2;  dX1 = gY1;  dX2 = dY2 + J_F(X2)^T gY1.
    """
    cf, cg = cache
    dg_in, grads_g = G_vjp(dy2, cg, p)
    gy1 = dy1 + dg_in
    df_in, grads_f = F_vjp(gy1, cf, p)
    dx1 = gy1
    dx2 = dy2 + df_in
    grads = dict(grads_f)
    grads.update(grads_g)
    return dx1, dx2, grads


# ----------------------------------------------------------------------------
# the stack
# ----------------------------------------------------------------------------
def stack_forward(x1, x2, blocks, H, eps=1e-6, key_len=None):
    for p in blocks:
        x1, x2 = block_forward(x1, x2, p, H, eps, key_len=key_len)
    return x1, x2


def stack_inverse(y1, y2, blocks, H, eps=1e-6, key_len=None):
    for p in reversed(blocks):
        y1, y2 = block_inverse(y1, y2, p, H, eps, key_len=key_len)
    return y1, y2


def stack_backward_stored(x1, x2, blocks, H, dy1, dy2, eps=1e-6, key_len=None):
    """Ordinary backprop: forward keeps every block's intermediates, then reverse mode."""
    caches = []
    for p in blocks:
        x1, x2, c = block_forward(x1, x2, p, H, eps, want_cache=True, key_len=key_len)
        caches.append(c)
    grads = [None] * len(blocks)
    for i in reversed(range(len(blocks))):
        dy1, dy2, grads[i] = block_vjp(caches[i], blocks[i], dy1, dy2)
    return dy1, dy2, grads


def stack_backward_reversible(y1, y2, blocks, H, dy1, dy2, eps=1e-6, key_len=None):
    """Sec. 3.2 (Reprop): top block first -- invert, backpropagate, drop, repeat.

    Returns (dX1, dX2, per-block grads, X1, X2) where X1, X2 are the
    reconstructed stack inputs.  PaReprop (Sec. 3.3) reorders this work in time
    only, so it has the same result.
    """
    grads = [None] * len(blocks)
    for i in reversed(range(len(blocks))):
        x1, x2, cache = block_inverse(y1, y2, blocks[i], H, eps, want_cache=True, key_len=key_len)
        dy1, dy2, grads[i] = block_vjp(cache, blocks[i], dy1, dy2)
        y1, y2 = x1, x2
    return dy1, dy2, grads, y1, y2


def add_grads(acc, grads):
    """acc += grads over a list of per-block dicts (parameter gradients sum over samples)."""
    if acc is None:
        return [{k: v.copy() for k, v in g.items()} for g in grads]
    for a, g in zip(acc, grads):
        for k in a:
            a[k] += g[k]
    return acc


def stack_backward_reversible_chunked(y1, y2, blocks, H, dy1, dy2, eps=1e-6, chunk=8, key_len=None):
    """Same result as stack_backward_reversible, walking the batch in chunks to bound memory."""
    B = y1.shape[0]
    dx1 = np.empty_like(y1, dtype=F64)
    dx2 = np.empty_like(y1, dtype=F64)
    x1 = np.empty_like(y1, dtype=F64)
    x2 = np.empty_like(y1, dtype=F64)
    acc = None
    for s in range(0, B, chunk):
        sl = slice(s, min(B, s + chunk))
        a, b, g, c, d = stack_backward_reversible(
            np.asarray(y1[sl], F64), np.asarray(y2[sl], F64), blocks, H,
            np.asarray(dy1[sl], F64), np.asarray(dy2[sl], F64), eps,
            key_len=None if key_len is None else key_len[sl])
        dx1[sl], dx2[sl], x1[sl], x2[sl] = a, b, c, d
        acc = add_grads(acc, g)
    return dx1, dx2, acc, x1, x2
