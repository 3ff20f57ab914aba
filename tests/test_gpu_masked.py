"""GPU parity of the key-padding-mask entry points (rev_stack_*_masked, through the C-ABI) against the
float64 oracle run with the same per-sample key lengths: forward outputs at every position (padded
ones included: they are well defined), input cotangents, reconstructed inputs and every parameter
gradient; same error measure and tolerances as the unmasked parity tests.  Lengths cover full, ragged
inside a 32-key tile, a single valid key, and lengths that end before the last 64-row tile of the
streamed attention kernels.  PaReprop must equal Reprop bit for bit under the mask, and a mask of
full lengths must reproduce the unmasked call bit for bit."""
import numpy as np
import pytest
import torch

from oracle import rev_oracle as O
from paper_2306_09342_amd import binding as B

from parity_util import TOL, compare_backward, gpu_cfg, make_case, rel_err, to_dev

pytestmark = pytest.mark.gpu

CASES = {
    # name: (shape, key lengths)
    "tiny": (dict(n_blocks=4, d_model=64, n_heads=2, d_mlp=256, seq_len=16, batch=4), [16, 9, 1, 12]),
    "ragged_dh64": (dict(n_blocks=2, d_model=128, n_heads=2, d_mlp=512, seq_len=77, batch=3), [77, 40, 33]),
    "vit_s_slice": (dict(n_blocks=2, d_model=384, n_heads=6, d_mlp=1536, seq_len=197, batch=3), [150, 197, 64]),
    "window": (dict(n_blocks=2, d_model=96, n_heads=3, d_mlp=384, seq_len=49, batch=5), [49, 1, 32, 31, 48]),
    "dh80_T300": (dict(n_blocks=1, d_model=160, n_heads=2, d_mlp=160, seq_len=300, batch=2), [300, 130]),
    "dh64_T256": (dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=128, seq_len=256, batch=3), [256, 100, 193]),
    "dh32_T130": (dict(n_blocks=1, d_model=64, n_heads=2, d_mlp=128, seq_len=130, batch=4), [130, 1, 64, 97]),
    "T1024": (dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=128, seq_len=1024, batch=2), [700, 65]),
}


def _oracle_forward(cfg, blocks, x1, x2, lens):
    y1 = np.empty(x1.shape, np.float64)
    y2 = np.empty(x1.shape, np.float64)
    for b in range(x1.shape[0]):
        sl = slice(b, b + 1)
        y1[sl], y2[sl] = O.stack_forward(x1[sl].astype(np.float64), x2[sl].astype(np.float64), blocks, cfg["n_heads"],
                                         cfg.get("ln_eps", 1e-6), key_len=lens[sl])
    return y1, y2


def _run(name, mode):
    shape, lens = CASES[name]
    cfg = dict(shape, mode=mode)
    lens = np.asarray(lens, dtype=np.int32)
    print(f"[case] masked {name} mode={mode} key_len={lens.tolist()}", flush=True)
    flat, blocks, x, dy1, dy2 = make_case(cfg, seed=2)
    x2 = x[:, ::-1].copy()
    y1, y2 = _oracle_forward(cfg, blocks, x, x2, lens)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)
    ref = O.stack_backward_reversible_chunked(y1f, y2f, blocks, cfg["n_heads"], dy1, dy2, chunk=1, key_len=lens)

    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    klen = torch.from_numpy(lens).cuda()
    ws = B.alloc_workspace(c)
    tol = TOL[mode]
    gy1, gy2 = B.rev_stack_forward_masked(c, params, to_dev(x), to_dev(x2), klen, workspace=ws)
    torch.cuda.synchronize()
    assert rel_err(gy1.cpu().numpy(), y1) <= tol and rel_err(gy2.cpu().numpy(), y2) <= tol
    dY1, dY2, Y1, Y2 = to_dev(dy1), to_dev(dy2), to_dev(y1f), to_dev(y2f)
    rep = B.rev_stack_backward_reprop_masked(c, params, Y1, Y2, klen, dY1, dY2, workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    worst = compare_backward(cfg, rep, ref, tol, what=f"masked {name}/{mode}/reprop")
    side = torch.cuda.Stream()
    par = B.rev_stack_backward_pareprop_masked(c, params, Y1, Y2, klen, dY1, dY2, side, workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams", "X1", "X2"):
        assert torch.equal(rep[k], par[k]), f"PaReprop differs from Reprop in {k}"
    assert klen.cpu().numpy().tolist() == lens.tolist(), "key_len must not be modified"
    print(f"[ok] masked {name}/{mode}: worst {max(worst.values()):.3e} at {max(worst, key=worst.get)}", flush=True)


@pytest.mark.parametrize("name", list(CASES))
def test_masked_fp32_matches_oracle(name):
    _run(name, "fp32")


@pytest.mark.parametrize("name", list(CASES))
def test_masked_bf16_matches_oracle(name):
    _run(name, "bf16")


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
def test_full_lengths_reproduce_the_unmasked_call_bit_for_bit(mode):
    shape, _ = CASES["vit_s_slice"]
    cfg = dict(shape, mode=mode)
    flat, _, x, dy1, dy2 = make_case(cfg, seed=4)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    full = torch.full((cfg["batch"],), cfg["seq_len"], dtype=torch.int32, device="cuda")
    over = full + 1000                                      # values beyond seq_len are clamped to it
    X = to_dev(x)
    a1, a2 = B.rev_stack_forward(c, params, X, X.clone())
    b1, b2 = B.rev_stack_forward_masked(c, params, X, X.clone(), full)
    c1, c2 = B.rev_stack_forward_masked(c, params, X, X.clone(), over)
    assert torch.equal(a1, b1) and torch.equal(a2, b2) and torch.equal(a1, c1) and torch.equal(a2, c2)
    dY1, dY2 = to_dev(dy1), to_dev(dy2)
    ra = B.rev_stack_backward_reprop(c, params, a1, a2, dY1, dY2)
    rb = B.rev_stack_backward_reprop_masked(c, params, a1, a2, full, dY1, dY2)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams"):
        assert torch.equal(ra[k], rb[k]), k


def test_masked_calls_reject_a_missing_or_misshapen_mask():
    shape, _ = CASES["tiny"]
    cfg = dict(shape, mode="fp32")
    flat, _, x, dy1, dy2 = make_case(cfg, seed=0)
    c = gpu_cfg(cfg)
    X = to_dev(x)
    with pytest.raises(AssertionError):
        B.rev_stack_forward_masked(c, to_dev(flat), X, X.clone(), torch.ones(3, dtype=torch.int32, device="cuda"))
    import ctypes
    ws = B.alloc_workspace(c)
    Y = torch.empty_like(X)
    rc = B.lib().rev_stack_forward_masked(ctypes.byref(c), ctypes.c_void_p(to_dev(flat).data_ptr()),
                                          ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(X.data_ptr()), None,
                                          ctypes.c_void_p(Y.data_ptr()), ctypes.c_void_p(Y.data_ptr()),
                                          ctypes.c_void_p(ws.data_ptr()), ws.numel(), None)
    assert rc == -1 and "key_len" in B.rev_last_error()
