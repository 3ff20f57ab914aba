"""Seeded synthetic inputs for the reversible-stack backward path.

This module only draws random arrays and places them in the packed parameter
vector; it holds none of the method's arithmetic, so both the CPU oracle's
tests and the HIP path's tests/bench may feed from it.  The workloads stand in
for the paper's 224x224 image-classification batches (Rev-ViT shapes) and its
text-classification batches (Rev-RoBERTa shape): only the shapes matter for the
backward path, no dataset item is reproduced.

Recipe (all configs): X ~ N(0,1) [B,T,D], copied to both residual streams;
every weight matrix truncated-normal(0, 0.02) cut at +-2 sigma by rejection;
LayerNorm gamma = 1, beta = 0; linear biases 0; dY1, dY2 ~ N(0,1) independent.
``perturb=True`` (parity tests only) additionally draws non-trivial gammas,
betas and biases so that a dropped bias or affine term cannot hide.
In bf16 mode every value is rounded (nearest-even) onto the bf16 grid at
generation time, so both consumers read identical, exactly representable data.
"""
from __future__ import annotations

import numpy as np

# name -> (n_blocks, d_model, n_heads, d_mlp, seq_len, batch, mode)
CONFIGS = {
    "tiny": dict(n_blocks=4, d_model=64, n_heads=2, d_mlp=256, seq_len=16, batch=4, mode="fp32"),
    "vit_s": dict(n_blocks=12, d_model=384, n_heads=6, d_mlp=1536, seq_len=197, batch=128, mode="bf16"),
    "vit_b": dict(n_blocks=12, d_model=768, n_heads=12, d_mlp=3072, seq_len=197, batch=64, mode="bf16"),
    "roberta_base": dict(n_blocks=12, d_model=768, n_heads=12, d_mlp=3072, seq_len=512, batch=32, mode="bf16"),
    "vit_h": dict(n_blocks=32, d_model=1280, n_heads=16, d_mlp=5120, seq_len=257, batch=32, mode="bf16"),
    # further text-model points of the paper's sequence-length / model-size comparison (Sec. 4.1, NLP):
    # the base width at 1024 tokens and the large width (24 blocks, 1024 wide, 16 heads) at 512 and 1024
    "roberta_base_t1024": dict(n_blocks=12, d_model=768, n_heads=12, d_mlp=3072, seq_len=1024, batch=16, mode="bf16"),
    "roberta_large": dict(n_blocks=24, d_model=1024, n_heads=16, d_mlp=4096, seq_len=512, batch=16, mode="bf16"),
    "roberta_large_t1024": dict(n_blocks=24, d_model=1024, n_heads=16, d_mlp=4096, seq_len=1024, batch=8, mode="bf16"),
}

# Hierarchical (window-attention) workloads, Sec. 3.4 / Sec. 4.1: a list of stages, each a homogeneous
# reversible stack whose "samples" are the attention windows of the images.  224 x 224 inputs, 4 x 4
# patches, 7 x 7 windows: 49 tokens per window and 64 / 16 / 4 / 1 windows per image in the four
# stages, width doubling and head count doubling from stage to stage (head_dim 32), MLP ratio 4.
# Only these shapes are modelled; what sits between the stages (fusion of the two streams, patch
# merging) and inside the attention of the original architecture beyond plain softmax attention
# (window shifts, position bias) is outside the reversible blocks' backward path.
def _window_stages(width, heads, depths, images):
    return [dict(n_blocks=d, d_model=width << s, n_heads=heads << s, d_mlp=4 * (width << s), seq_len=49,
                 batch=images * (64 >> (2 * s)), mode="bf16") for s, d in enumerate(depths)]


HIERARCHIES = {
    "swin_t": dict(images=64, stages=_window_stages(96, 3, (2, 2, 6, 2), 64)),
    "swin_b": dict(images=64, stages=_window_stages(128, 4, (2, 2, 18, 2), 64)),
    "swin_l": dict(images=32, stages=_window_stages(192, 6, (2, 2, 18, 2), 32)),
}

# Per-block tensors of the packed parameter vector, in storage order.
# Linear weights are [out_features, in_features], row-major.
def block_tensors(d_model: int, d_mlp: int):
    D, Dm = d_model, d_mlp
    return [
        ("ln1_g", (D,)), ("ln1_b", (D,)),
        ("w_qkv", (3 * D, D)), ("b_qkv", (3 * D,)),
        ("w_proj", (D, D)), ("b_proj", (D,)),
        ("ln2_g", (D,)), ("ln2_b", (D,)),
        ("w_fc1", (Dm, D)), ("b_fc1", (Dm,)),
        ("w_fc2", (D, Dm)), ("b_fc2", (D,)),
    ]


def params_per_block(d_model: int, d_mlp: int) -> int:
    return sum(int(np.prod(s)) for _, s in block_tensors(d_model, d_mlp))


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def _trunc_normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float64)
    filled = 0
    while filled < n:
        draw = rng.standard_normal(int((n - filled) * 1.1) + 16)
        draw = draw[np.abs(draw) <= 2.0]
        take = min(draw.size, n - filled)
        out[filled:filled + take] = draw[:take]
        filled += take
    return (out * std).reshape(shape)


def make_params(cfg: dict, seed: int = 0, perturb: bool = False) -> np.ndarray:
    """Packed float32 parameter vector for the whole stack."""
    D, Dm, N = cfg["d_model"], cfg["d_mlp"], cfg["n_blocks"]
    per = params_per_block(D, Dm)
    flat = np.empty(N * per, dtype=np.float32)
    for blk in range(N):
        off = blk * per
        for tid, (name, shape) in enumerate(block_tensors(D, Dm)):
            rng = np.random.default_rng([seed, 1000 + blk, tid])
            n = int(np.prod(shape))
            if name.startswith("w_"):
                v = _trunc_normal(rng, shape, 0.02)
            elif name.endswith("_g"):
                v = 1.0 + (0.1 * rng.standard_normal(shape) if perturb else np.zeros(shape))
            elif name.startswith("ln"):
                v = 0.1 * rng.standard_normal(shape) if perturb else np.zeros(shape)
            else:
                v = 0.02 * rng.standard_normal(shape) if perturb else np.zeros(shape)
            flat[off:off + n] = np.asarray(v, dtype=np.float32).ravel()
            off += n
    if cfg.get("mode", "fp32") == "bf16":
        flat = to_bf16_grid(flat)
    return flat


def make_inputs(cfg: dict, seed: int = 0, batch: int | None = None):
    """Returns (X, dY1, dY2), each float32 [B, T, D]; X feeds both streams."""
    B = cfg["batch"] if batch is None else batch
    T, D = cfg["seq_len"], cfg["d_model"]
    out = []
    for tid in range(3):
        rng = np.random.default_rng([seed, 7, tid])
        out.append(rng.standard_normal((B, T, D), dtype=np.float32))
    return tuple(out)


# Stage transitions of the hierarchical workloads (Sec. 3.4): between stage s and s+1 of a hierarchy the
# token grid halves per side and the width doubles.  Seeded inputs only; no arithmetic of the block here.
def merge_cfgs(hier: dict, image: int = 224, patch: int = 4, window: int = 7, fusion: str = "average"):
    """One dict per transition of HIERARCHIES[...]: batch (images), grid_h, grid_w, window, d_in, mode, fusion."""
    out = []
    for s, st in enumerate(hier["stages"][:-1]):
        side = image // patch >> s
        out.append(dict(batch=hier["images"], grid_h=side, grid_w=side, window=window, d_in=st["d_model"],
                        mode=st["mode"], ln_eps=1e-5, fusion=fusion))
    return out


def make_merge_params(mcfg: dict, seed: int = 0, perturb: bool = False) -> np.ndarray:
    """Packed float32 parameters of one transition: ln_gamma[4C], ln_beta[4C], W[2C, 4C], and for
    mcfg["fusion"] == "mlp" the fusion MLP's Wa[C, 2C], ba[C], Wb[C, C], bb[C] behind them."""
    C = mcfg["d_in"]
    rng = np.random.default_rng([seed, 31, C])
    g = 1.0 + (0.1 * rng.standard_normal(4 * C) if perturb else np.zeros(4 * C))
    b = 0.1 * rng.standard_normal(4 * C) if perturb else np.zeros(4 * C)
    w = _trunc_normal(rng, (2 * C, 4 * C), 0.02)
    parts = [g, b, w.ravel()]
    if mcfg.get("fusion", "average") == "mlp":
        # fusion MLP (Sec. 3.4): Wa[C, 2C], ba[C], Wb[C, C], bb[C], drawn like the blocks' linear maps
        parts += [_trunc_normal(rng, (C, 2 * C), 0.02).ravel(), 0.02 * rng.standard_normal(C) if perturb else np.zeros(C),
                  _trunc_normal(rng, (C, C), 0.02).ravel(), 0.02 * rng.standard_normal(C) if perturb else np.zeros(C)]
    flat = np.concatenate(parts).astype(np.float32)
    if mcfg.get("mode", "fp32") == "bf16":
        flat = to_bf16_grid(flat)
    return flat


def make_merge_inputs(mcfg: dict, seed: int = 0):
    """Returns (X1, X2, dOutA, dOutB): float32 [B*Gh*Gw, C] twice and [B*Gh*Gw/4, 2C] twice."""
    M = mcfg["batch"] * mcfg["grid_h"] * mcfg["grid_w"]
    C = mcfg["d_in"]
    shapes = [(M, C), (M, C), (M // 4, 2 * C), (M // 4, 2 * C)]
    return tuple(np.random.default_rng([seed, 33, tid]).standard_normal(shp, dtype=np.float32)
                 for tid, shp in enumerate(shapes))


def make_key_lengths(cfg: dict, seed: int = 0) -> np.ndarray:
    """Valid lengths of a padded batch (int32 [batch]): uniform on [T/8, T], the first sample full length."""
    T, Bn = cfg["seq_len"], cfg["batch"]
    rng = np.random.default_rng([seed, 41])
    lens = rng.integers(max(1, T // 8), T + 1, size=Bn).astype(np.int32)
    lens[0] = T
    return lens
