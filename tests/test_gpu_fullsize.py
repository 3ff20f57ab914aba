"""GPU parity at the benchmark's full sizes and in its launch configuration.

Every bf16 workload is run on the GPU at its FULL batch, with the tile shapes
and grids the benchmark times, and compared with the fp64 oracle:
  * Rev-ViT-B (the headline), Rev-ViT-S and Rev-RoBERTa-base: the oracle's
    reversible backward of the whole batch (every sample's dX1/dX2 and
    reconstructed inputs, every parameter gradient of every block, summed over
    all samples), tens of seconds on the machine's host cores;
  * Rev-ViT-H (32 blocks, the oracle manages a third of a sample per second):
    the stack outputs Y of every sample, dX1/dX2 and the reconstructed inputs of
    sampled samples through all 32 blocks (samples never interact, so a
    sample's rows depend on that sample alone), and every parameter gradient
    of the TOP block over the full batch (one block of inversion and VJP);
and two properties that hold at any size are checked on the GPU results:
PaReprop == Reprop bit for bit, and parameter gradients add over sub-batches.
The reduced-batch runs below them keep the deep shapes cheap to re-run.
Tolerance: 3e-2 (bf16 mode), max-abs error over max-abs reference per tensor.
"""
import numpy as np
import pytest
import torch

from oracle import rev_oracle as O
from paper_2306_09342_amd import binding as B
from paper_2306_09342_amd import synth

from parity_util import TOL, compare_backward, gpu_cfg, oracle_forward, rel_err, to_dev

pytestmark = pytest.mark.gpu
TOLB = TOL["bf16"]


def _bench_inputs(name, batch=None):
    cfg = dict(synth.CONFIGS[name])
    if batch is not None:
        cfg["batch"] = batch
    flat = synth.make_params(cfg, seed=0)                 # the benchmark's recipe: unit gains, zero biases
    x, dy1, dy2 = synth.make_inputs(cfg, seed=0, batch=cfg["batch"])
    blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
    return cfg, flat, blocks, x, dy1, dy2


def _gpu_both_schedules(cfg, flat, y1f, y2f, dy1, dy2):
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    ws = B.alloc_workspace(c)
    Y1, Y2, dY1, dY2 = to_dev(y1f), to_dev(y2f), to_dev(dy1), to_dev(dy2)
    side = torch.cuda.Stream()
    par = B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    rep = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams", "X1", "X2"):
        assert torch.isfinite(par[k]).all(), k
        assert torch.equal(par[k], rep[k]), f"PaReprop differs from Reprop in {k}"
    return c, params, ws, (Y1, Y2, dY1, dY2), par


@pytest.mark.parametrize("name", ["vit_b", "vit_s", "roberta_base"])
def test_full_batch_every_tensor_against_the_oracle(name):
    """The benchmark's own launch configuration (full batch, hence its tile shapes and grids): every
    output of the backward pass against the oracle's reversible backward of the whole batch."""
    cfg, flat, blocks, x, dy1, dy2 = _bench_inputs(name)
    H, N = cfg["n_heads"], cfg["n_blocks"]
    print(f"[case] {name} full batch {cfg['batch']}: oracle forward of all samples", flush=True)
    y1, y2 = oracle_forward(cfg, blocks, x, x, chunk=4)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)

    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    X = to_dev(x)
    gy1, gy2 = B.rev_stack_forward(c, params, X, X)
    torch.cuda.synchronize()
    assert rel_err(gy1.cpu().numpy(), y1) <= TOLB and rel_err(gy2.cpu().numpy(), y2) <= TOLB
    del gy1, gy2, X

    print(f"[case] {name} full batch: GPU PaReprop + Reprop", flush=True)
    c, params, ws, (Y1, Y2, dY1, dY2), par = _gpu_both_schedules(cfg, flat, y1f, y2f, dy1, dy2)
    print(f"[case] {name} full batch: oracle reversible backward of all {cfg['batch']} samples", flush=True)
    ref = O.stack_backward_reversible_chunked(y1f, y2f, blocks, H, dy1, dy2, chunk=4)
    worst = compare_backward(cfg, par, ref, TOLB, what=f"{name} full batch")
    print(f"[ok] {name} full batch: worst {max(worst.values()):.3e} at {max(worst, key=worst.get)}", flush=True)
    # the reconstructed inputs are the true inputs, for every sample
    assert rel_err(par["X1"].cpu().numpy(), x) <= TOLB and rel_err(par["X2"].cpu().numpy(), x) <= TOLB

    if name != "vit_b":
        return
    # parameter gradients add over samples: four quarter-batch runs sum to the full-batch result
    q = cfg["batch"] // 4
    cq = gpu_cfg(dict(cfg, batch=q))
    wsq = B.alloc_workspace(cq)
    total = torch.zeros_like(par["dparams"], dtype=torch.float64)
    for i in range(4):
        sl = slice(i * q, (i + 1) * q)
        r = B.rev_stack_backward_reprop(cq, params, Y1[sl].contiguous(), Y2[sl].contiguous(),
                                        dY1[sl].contiguous(), dY2[sl].contiguous(), workspace=wsq)
        torch.cuda.synchronize()
        total += r["dparams"].double()
        assert rel_err(r["dX1"].cpu().numpy(), par["dX1"][sl].cpu().numpy()) <= 1e-6   # dX ignores other samples
    full = O.unpack_params(par["dparams"].cpu().numpy(), N, cfg["d_model"], cfg["d_mlp"])
    parts = O.unpack_params(total.cpu().numpy(), N, cfg["d_model"], cfg["d_mlp"])
    lin = max(rel_err(parts[i][k], full[i][k]) for i in range(N) for k in full[i])
    print(f"[ok] batch linearity of dparams: {lin:.2e}", flush=True)
    assert lin <= 1e-3


def test_vit_h_full_batch_sampled_against_the_oracle():
    """32 blocks, head_dim 80, full batch 32 in the benchmark's launch configuration.  The oracle is evaluated
    where it finishes in about a minute: Y of every sample, dX and reconstructed inputs of two samples through
    all 32 blocks, every parameter gradient of the top block over the whole batch."""
    name = "vit_h"
    cfg, flat, blocks, x, dy1, dy2 = _bench_inputs(name)
    H, N = cfg["n_heads"], cfg["n_blocks"]
    print(f"[case] {name} full batch {cfg['batch']}: oracle forward of all samples", flush=True)
    y1, y2 = oracle_forward(cfg, blocks, x, x, chunk=4)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    X = to_dev(x)
    gy1, gy2 = B.rev_stack_forward(c, params, X, X)
    torch.cuda.synchronize()
    e1, e2 = rel_err(gy1.cpu().numpy(), y1), rel_err(gy2.cpu().numpy(), y2)
    print(f"[ok] {name} forward of all samples: Y1 {e1:.2e} Y2 {e2:.2e}", flush=True)
    assert e1 <= TOLB and e2 <= TOLB
    del gy1, gy2, X
    c, params, ws, _, par = _gpu_both_schedules(cfg, flat, y1f, y2f, dy1, dy2)
    assert rel_err(par["X1"].cpu().numpy(), x) <= TOLB and rel_err(par["X2"].cpu().numpy(), x) <= TOLB
    for b in (0, 21):
        sl = slice(b, b + 1)
        rdx1, rdx2, _, rx1, rx2 = O.stack_backward_reversible(
            y1f[sl].astype(np.float64), y2f[sl].astype(np.float64), blocks, H,
            dy1[sl].astype(np.float64), dy2[sl].astype(np.float64))
        e1 = rel_err(par["dX1"][sl].cpu().numpy(), rdx1)
        e2 = rel_err(par["dX2"][sl].cpu().numpy(), rdx2)
        print(f"[ok] sample {b}: dX1 {e1:.2e} dX2 {e2:.2e}", flush=True)
        assert e1 <= TOLB and e2 <= TOLB, (b, e1, e2)
    acc = None
    top = blocks[N - 1]
    for s in range(0, cfg["batch"], 8):
        sl = slice(s, s + 8)
        _, _, cache = O.block_inverse(y1f[sl].astype(np.float64), y2f[sl].astype(np.float64), top, H, 1e-6,
                                      want_cache=True)
        _, _, g = O.block_vjp(cache, top, dy1[sl].astype(np.float64), dy2[sl].astype(np.float64))
        acc = O.add_grads(acc, [g])
    gpu_top = O.unpack_params(par["dparams"].cpu().numpy(), N, cfg["d_model"], cfg["d_mlp"])[N - 1]
    worst = {k: rel_err(gpu_top[k], acc[0][k]) for k in acc[0]}
    print(f"[ok] top-block parameter gradients over the full batch: worst {max(worst.values()):.2e}", flush=True)
    assert max(worst.values()) <= TOLB, worst


@pytest.mark.parametrize("name,batch", [("vit_s", 6), ("roberta_base", 2), ("vit_h", 2), ("roberta_large", 1)])
def test_full_depth_full_width_reduced_batch(name, batch):
    """All blocks at full width (32 blocks and head_dim 80 for vit_h, T = 512 for
    roberta_base), batch reduced to what the oracle finishes in seconds."""
    cfg, flat, blocks, x, dy1, dy2 = _bench_inputs(name, batch=batch)
    print(f"[case] {name} batch={batch} cfg={cfg}", flush=True)
    H = cfg["n_heads"]
    y1, y2 = oracle_forward(cfg, blocks, x, x, chunk=2)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)
    ref = O.stack_backward_reversible_chunked(y1f, y2f, blocks, H, dy1, dy2, chunk=2)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    ws = B.alloc_workspace(c)
    side = torch.cuda.Stream()
    par = B.rev_stack_backward_pareprop(c, params, to_dev(y1f), to_dev(y2f), to_dev(dy1), to_dev(dy2), side,
                                        workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    rep = B.rev_stack_backward_reprop(c, params, to_dev(y1f), to_dev(y2f), to_dev(dy1), to_dev(dy2),
                                      workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams", "X1", "X2"):
        assert torch.equal(par[k], rep[k]), f"PaReprop differs from Reprop in {k}"
    worst = compare_backward(cfg, par, ref, TOLB, what=name)
    print(f"[ok] {name}: worst {max(worst.values()):.3e} at {max(worst, key=worst.get)}", flush=True)


def test_full_batch_shapes_run_and_agree_between_schedules():
    """The widening text shapes at their full batch: finite outputs, exact reconstruction
    tolerance on the inputs (known without the oracle: Y comes from the GPU forward
    of X here, so only self-consistency is claimed), PaReprop == Reprop."""
    for name in ("roberta_large", "roberta_large_t1024", "roberta_base_t1024"):
        cfg = dict(synth.CONFIGS[name])
        print(f"[case] {name} full batch", flush=True)
        flat = synth.make_params(cfg, seed=0)
        x, dy1, dy2 = synth.make_inputs(cfg, seed=0)
        c = gpu_cfg(cfg)
        params = to_dev(flat, B.param_dtype(c))
        ws = B.alloc_workspace(c)
        X = to_dev(x)
        Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws)
        dY1, dY2 = to_dev(dy1), to_dev(dy2)
        side = torch.cuda.Stream()
        par = B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws, want_inputs=True)
        torch.cuda.synchronize()
        rep = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws, want_inputs=True)
        torch.cuda.synchronize()
        for k in ("dX1", "dX2", "dparams", "X1", "X2"):
            assert torch.isfinite(par[k]).all(), (name, k)
            assert torch.equal(par[k], rep[k]), (name, k)
        # inversion undoes the GPU's own forward up to bf16 rounding of the branch outputs
        err = (par["X1"] - X).abs().max().item() / X.abs().max().item()
        print(f"[ok] {name}: reconstruction error after {cfg['n_blocks']} blocks {err:.2e}", flush=True)
        assert err <= TOLB
        del ws, par, rep, Y1, Y2, dY1, dY2, X, params
        torch.cuda.empty_cache()
