"""The allocation-free entry point (rev_stack_backward_reprop_static: the sequential schedule in the
library's built-in workspace) against the entry point it is a variant of, rev_stack_backward_reprop with a
caller-provided workspace.  Both run the same kernels with the same grids, so the bar is bit-identity.
Two calls in a row, the second on a smaller input, so stale contents of the shared buffer would show."""
import ctypes

import pytest
import torch

from paper_2306_09342_amd import binding as B

from parity_util import gpu_cfg, make_case, to_dev

KEYS = ("dX1", "dX2", "dparams", "X1", "X2")


def _one_call(cfg, seed):
    flat, _, x, dy1, dy2 = make_case(cfg, seed=seed)
    c = gpu_cfg(cfg)
    assert B.rev_stack_workspace_bytes_reprop(c) <= B.STATIC_WORKSPACE_BYTES
    params = to_dev(flat, B.param_dtype(c))
    X, dY1, dY2 = to_dev(x), to_dev(dy1), to_dev(dy2)
    Y1, Y2 = B.rev_stack_forward(c, params, X, X)
    ref = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, want_inputs=True)
    torch.cuda.synchronize()
    out = {"dX1": torch.empty_like(Y1), "dX2": torch.empty_like(Y1), "X1": torch.empty_like(Y1),
           "X2": torch.empty_like(Y1), "dparams": torch.empty(params.numel(), dtype=torch.float32, device="cuda")}
    for v in out.values():
        v.fill_(float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.rev_stack_backward_reprop_static(c, params, Y1, Y2, dY1, dY2, out)
    assert torch.cuda.memory_allocated() == before        # nothing allocated through torch either
    torch.cuda.synchronize()
    for k in KEYS:
        assert torch.isfinite(out[k]).all(), k
        assert torch.equal(out[k], ref[k]), f"{k} differs from rev_stack_backward_reprop"


@pytest.mark.gpu
def test_static_workspace_call_equals_the_workspace_call_twice_in_a_row():
    big = dict(n_blocks=3, d_model=384, n_heads=6, d_mlp=1536, seq_len=197, batch=3, mode="bf16")
    small = dict(n_blocks=2, d_model=128, n_heads=2, d_mlp=512, seq_len=77, batch=3, mode="bf16")
    print("[case] static workspace: vit_s_slice bf16, then ragged_dh64 bf16, then tiny fp32", flush=True)
    _one_call(big, seed=31)
    _one_call(small, seed=32)
    _one_call(dict(n_blocks=4, d_model=64, n_heads=2, d_mlp=256, seq_len=16, batch=4, mode="fp32"), seed=0)


def test_static_workspace_call_rejects_a_shape_beyond_its_buffer_on_the_host():
    c = B.make_cfg(n_blocks=12, d_model=768, n_heads=12, d_mlp=3072, seq_len=197, batch=64, mode="bf16")
    assert B.rev_stack_workspace_bytes_reprop(c) > B.STATIC_WORKSPACE_BYTES
    fake = ctypes.c_void_p(0x10000)      # never dereferenced: the size check comes first
    rc = B.lib().rev_stack_backward_reprop_static(ctypes.byref(c), fake, fake, fake, fake, fake, fake, fake, None, None,
                                                  fake, None)
    assert rc == -2 and "static workspace too small" in B.rev_last_error()
    bad = B.make_cfg(n_blocks=0, d_model=64, n_heads=2, d_mlp=256, seq_len=16, batch=4, mode="fp32")
    assert B.lib().rev_stack_backward_reprop_static(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, fake, None, None,
                                                    fake, None) == -1
