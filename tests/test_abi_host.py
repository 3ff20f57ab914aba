"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, sizes the packed parameters as the layout
says, and rejects bad arguments before enqueuing anything."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2306_09342_amd import binding as B
from paper_2306_09342_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    text = open(os.path.join(ROOT, "include", "rev_stack.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rev_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _header_functions()
    assert "rev_stack_forward" in names and "rev_stack_backward_pareprop" in names
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_param_count_and_offsets_match_the_layout(name):
    cfg = synth.CONFIGS[name]
    c = B.make_cfg(**cfg)
    D, Dm, N = cfg["d_model"], cfg["d_mlp"], cfg["n_blocks"]
    per = 4 * D * D + 2 * D * Dm + 9 * D + Dm
    assert B.rev_stack_param_count(c) == N * per == N * synth.params_per_block(D, Dm)
    off = 0
    for t, (tname, shape) in enumerate(synth.block_tensors(D, Dm)):
        o, cnt = B.rev_stack_param_offset(c, N - 1, t)
        assert o == (N - 1) * per + off and cnt == int(np.prod(shape)), tname
        off += cnt
    ws = B.rev_stack_workspace_bytes(c)
    assert ws > 0 and ws % 256 == 0


def _up(n):
    return (n + 255) // 256 * 256


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_workspace_sizes_of_the_two_schedules(name):
    """One activation slot holds n2, h, a, n1, qkv, o (activation type), the softmax row
    statistics and the two LayerNorm statistics (float32); the sequential schedule's workspace is
    smaller than the parallel one's by one slot, one residual level and the second copies of the
    per-block gradient temporaries (gY1 copy, dh, dqkv)."""
    cfg = synth.CONFIGS[name]
    c = B.make_cfg(**cfg)
    D, Dm, T, Bsz, H = cfg["d_model"], cfg["d_mlp"], cfg["seq_len"], cfg["batch"], cfg["n_heads"]
    M = Bsz * T
    es = 2 if cfg["mode"] == "bf16" else 4
    slot = (_up(M * D * es) * 3 + _up(M * Dm * es) * 2 + _up(M * 3 * D * es) + _up(Bsz * H * T * 4) + 2 * _up(M * 8))
    assert B.rev_stack_slot_bytes(c) == slot
    full, small = B.rev_stack_workspace_bytes(c), B.rev_stack_workspace_bytes_reprop(c)
    extra = slot + 2 * _up(M * D * 4) + _up(M * Dm * es) + _up(M * 3 * D * es) + (_up(M * D * es) if es == 2 else 0)
    assert full - small == extra and small % 256 == 0


def test_bad_configs_are_rejected():
    good = dict(synth.CONFIGS["tiny"])
    assert B.rev_stack_check_cfg(B.make_cfg(**good)) == 0
    for key, val in (("n_blocks", 0), ("d_model", 60), ("n_heads", 3), ("d_mlp", 100), ("seq_len", -1),
                     ("batch", 0), ("mode", 7), ("n_heads", 16), ("ln_eps", -1.0), ("d_model", 16384)):
        bad = dict(good)
        bad[key] = val
        c = B.make_cfg(**bad)
        assert B.rev_stack_check_cfg(c) == -1, (key, val)
        assert B.rev_last_error() != ""
        with pytest.raises(B.RevError):
            B.rev_stack_workspace_bytes(c)
    assert B.lib().rev_stack_check_cfg(None) == -1
    # head_dim above 128
    c = B.make_cfg(n_blocks=1, d_model=512, n_heads=2, d_mlp=512, seq_len=4, batch=1)
    assert B.rev_stack_check_cfg(c) == -1


def test_shapes_beyond_the_launch_grid_limits_are_rejected_on_the_host():
    """(sample, head) pairs and 64-token strips sit on a launch-grid axis that holds 65535 entries: a shape
    beyond that is refused by the validation, before anything is enqueued, not by a failing launch in mid-pass."""
    # a window-attention shaped stage: 4096 windows x 24 heads = 98304 (sample, head) pairs
    c = B.make_cfg(n_blocks=1, d_model=768, n_heads=24, d_mlp=3072, seq_len=49, batch=4096)
    assert B.rev_stack_check_cfg(c) == -1 and "batch*n_heads" in B.rev_last_error()
    c = B.make_cfg(n_blocks=1, d_model=768, n_heads=24, d_mlp=3072, seq_len=49, batch=2730)     # 65520 pairs
    assert B.rev_stack_check_cfg(c) == 0
    # tokens: 65535 strips of 64
    c = B.make_cfg(n_blocks=1, d_model=64, n_heads=1, d_mlp=64, seq_len=64, batch=65535)
    assert B.rev_stack_check_cfg(c) == 0
    c = B.make_cfg(n_blocks=1, d_model=64, n_heads=1, d_mlp=64, seq_len=65, batch=65535)
    assert B.rev_stack_check_cfg(c) == -1 and "batch*seq_len" in B.rev_last_error()
    L = B.lib()
    fake = ctypes.c_void_p(0x10000)
    assert L.rev_stack_forward(ctypes.byref(c), fake, fake, fake, fake, fake, fake, 1 << 40, None) == -1


def test_null_pointers_and_short_workspace_fail_before_any_gpu_work():
    L = B.lib()
    c = B.make_cfg(**synth.CONFIGS["tiny"])
    need = B.rev_stack_workspace_bytes_reprop(c)
    full = B.rev_stack_workspace_bytes(c)
    fake = ctypes.c_void_p(0x10000)          # never dereferenced: validation comes first
    vp = ctypes.c_void_p
    # null workspace
    assert L.rev_stack_forward(ctypes.byref(c), fake, fake, fake, fake, fake, None, need, None) == -1
    # short workspace
    assert L.rev_stack_forward(ctypes.byref(c), fake, fake, fake, fake, fake, fake, need - 1, None) == -2
    assert "workspace too small" in B.rev_last_error()
    # null tensors
    assert L.rev_stack_forward(ctypes.byref(c), None, fake, fake, fake, fake, fake, need, None) == -1
    args = [ctypes.byref(c), fake, fake, fake, fake, fake, fake, fake, None, None, None, fake, need]
    assert L.rev_stack_backward_reprop(*args, None) == -1            # dparams null
    args[10] = fake
    args[2] = vp(0x10004)                                             # misaligned Y1
    assert L.rev_stack_backward_reprop(*args, None) == -1
    args[2] = fake
    args[12] = need - 1
    assert L.rev_stack_backward_reprop(*args, None) == -2            # short for the sequential schedule
    args[12] = need
    s = vp(0x1234)
    assert L.rev_stack_backward_pareprop(*args, s, vp(0x5678)) == -2  # enough for Reprop only
    args[12] = full
    assert L.rev_stack_backward_pareprop(*args, s, s) == -1           # same stream twice
    assert "different streams" in B.rev_last_error()
    assert L.rev_stack_backward_chain(*args, None, 5) == -1
    assert L.rev_profile_kinds() >= 6
    assert L.rev_profile_name(0) == b"gemm_nt"


def test_adamw_arguments_are_validated_before_any_gpu_work():
    L = B.lib()
    fake = ctypes.c_void_p(0x10000)
    ok = [1024, fake, None, fake, fake, fake, 1, 1e-3, 0.9, 0.999, 1e-8, 0.01, None]
    for idx, val in ((0, 0), (1, None), (3, None), (4, None), (5, None), (6, 0), (7, -1.0), (8, 1.0), (9, -0.1),
                     (10, -1e-8), (11, -0.5), (1, ctypes.c_void_p(0x10004)), (2, ctypes.c_void_p(0x10002))):
        args = list(ok)
        args[idx] = val
        assert L.rev_adamw_step(*args) == -1, (idx, val)
        assert "adamw" in B.rev_last_error()


def test_merge_cfg_validation_and_sizes():
    ok = B.make_merge_cfg(4, 56, 56, 7, 96, "bf16")
    assert B.rev_merge_check_cfg(ok) == 0
    assert B.rev_merge_param_count(ok) == 8 * 96 + 8 * 96 * 96
    mlp = B.make_merge_cfg(4, 56, 56, 7, 96, "bf16", fusion="mlp")
    assert B.rev_merge_check_cfg(mlp) == 0
    assert B.rev_merge_param_count(mlp) == 8 * 96 + 8 * 96 * 96 + 3 * 96 * 96 + 2 * 96
    assert B.rev_merge_workspace_bytes(mlp) > B.rev_merge_workspace_bytes(ok)
    assert B.rev_merge_check_cfg(B.make_merge_cfg(4, 56, 56, 7, 96, "bf16", fusion=2)) < 0
    # the workspace holds at least the normalised rows, the statistics and the two activation-typed cotangents
    mo = 4 * 28 * 28
    assert B.rev_merge_workspace_bytes(ok) >= mo * (4 * 96 * 2 * 2 + 2 * 96 * 2 + 8)
    for bad in (B.make_merge_cfg(4, 56, 49, 7, 96), B.make_merge_cfg(4, 56, 56, 7, 100), B.make_merge_cfg(0, 56, 56, 7, 96),
                B.make_merge_cfg(4, 56, 56, 7, 96, 7), B.make_merge_cfg(4, 56, 56, 7, 4096)):
        assert B.rev_merge_check_cfg(bad) < 0
        assert B.rev_last_error() != ""
        with pytest.raises(B.RevError):
            B.rev_merge_param_count(bad)


def test_merge_calls_validate_before_touching_the_device():
    c = B.make_merge_cfg(1, 14, 14, 7, 32, "fp32")
    L = B.lib()
    import ctypes
    # null pointers and a short workspace are refused on the host
    assert L.rev_merge_forward(ctypes.byref(c), None, None, None, None, None, 0, None) < 0
    assert L.rev_merge_backward(ctypes.byref(c), None, None, None, None, None, None, None, None, None, 0, None) < 0
    fake = ctypes.c_void_p(256)
    assert L.rev_merge_forward(ctypes.byref(c), fake, fake, fake, fake, fake, 16, None) == -2


def test_masked_calls_refuse_a_null_or_misaligned_mask_on_the_host():
    import ctypes
    c = B.make_cfg(n_blocks=1, d_model=64, n_heads=2, d_mlp=128, seq_len=8, batch=2, mode="fp32")
    L = B.lib()
    fake = ctypes.c_void_p(4096)
    ws_bytes = B.rev_stack_workspace_bytes(c)
    rc = L.rev_stack_forward_masked(ctypes.byref(c), fake, fake, fake, None, fake, fake, fake, ws_bytes, None)
    assert rc == -1 and "key_len" in B.rev_last_error()
    rc = L.rev_stack_backward_reprop_masked(ctypes.byref(c), fake, fake, fake, None, fake, fake, fake, fake, None, None,
                                            fake, fake, ws_bytes, None)
    assert rc == -1 and "key_len" in B.rev_last_error()
    s1, s2 = ctypes.c_void_p(8), ctypes.c_void_p(16)
    rc = L.rev_stack_backward_pareprop_masked(ctypes.byref(c), fake, fake, fake, None, fake, fake, fake, fake, None, None,
                                              fake, fake, ws_bytes, s1, s2)
    assert rc == -1 and "key_len" in B.rev_last_error()
    odd = ctypes.c_void_p(4098)
    rc = L.rev_stack_forward_masked(ctypes.byref(c), fake, fake, fake, odd, fake, fake, fake, ws_bytes, None)
    assert rc == -1 and "aligned" in B.rev_last_error()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
