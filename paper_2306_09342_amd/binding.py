"""ctypes binding of librevstack.so: argument marshalling only.

Every function has the name of the C entry point it calls (``include/rev_stack.h``)
and takes torch CUDA tensors, whose ``data_ptr()`` and whose streams' raw
handles are handed through.  Nothing here computes; if the library is missing
the import of the symbols fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librevstack.so")

REV_MODE_FP32 = 0
REV_MODE_BF16 = 1
MODES = {"fp32": REV_MODE_FP32, "bf16": REV_MODE_BF16}

EXPORTS = (
    "rev_stack_check_cfg", "rev_stack_param_count", "rev_stack_param_offset", "rev_stack_workspace_bytes",
    "rev_stack_workspace_bytes_reprop", "rev_stack_slot_bytes",
    "rev_stack_forward", "rev_stack_backward_reprop", "rev_stack_backward_pareprop", "rev_stack_backward_chain",
    "rev_stack_backward_reprop_static",
    "rev_stack_forward_masked", "rev_stack_backward_reprop_masked", "rev_stack_backward_pareprop_masked",
    "rev_adamw_step", "rev_sgd_step",
    "rev_merge_check_cfg", "rev_merge_param_count", "rev_merge_workspace_bytes", "rev_merge_forward", "rev_merge_backward",
    "rev_profile_begin", "rev_profile_end", "rev_profile_kinds", "rev_profile_name", "rev_profile_is_flops",
    "rev_profile_get", "rev_last_error",
)


class RevCfg(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("d_mlp", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("batch", ctypes.c_int32),
                ("mode", ctypes.c_int32), ("ln_eps", ctypes.c_float)]


class RevMergeCfg(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32),
                ("window", ctypes.c_int32), ("d_in", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("ln_eps", ctypes.c_float), ("fusion", ctypes.c_int32)]


class RevError(RuntimeError):
    pass


_lib = None


def lib():
    """Loads the C-ABI library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RevError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_09342_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        cp = ctypes.POINTER(RevCfg)
        L.rev_stack_check_cfg.argtypes = [cp]
        L.rev_stack_check_cfg.restype = ctypes.c_int
        L.rev_stack_param_count.argtypes = [cp]
        L.rev_stack_param_count.restype = i64
        L.rev_stack_param_offset.argtypes = [cp, i32, i32, ctypes.POINTER(i64)]
        L.rev_stack_param_offset.restype = i64
        for n in ("rev_stack_workspace_bytes", "rev_stack_workspace_bytes_reprop", "rev_stack_slot_bytes"):
            getattr(L, n).argtypes = [cp]
            getattr(L, n).restype = i64
        L.rev_stack_forward.argtypes = [cp, vp, vp, vp, vp, vp, vp, i64, vp]
        L.rev_stack_forward.restype = ctypes.c_int
        bw = [cp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64]
        L.rev_stack_backward_reprop.argtypes = bw + [vp]
        L.rev_stack_backward_reprop.restype = ctypes.c_int
        L.rev_stack_backward_reprop_static.argtypes = bw[:-2] + [vp]
        L.rev_stack_backward_reprop_static.restype = ctypes.c_int
        L.rev_stack_backward_pareprop.argtypes = bw + [vp, vp]
        L.rev_stack_backward_pareprop.restype = ctypes.c_int
        L.rev_stack_backward_chain.argtypes = bw + [vp, i32]
        L.rev_stack_backward_chain.restype = ctypes.c_int
        L.rev_stack_forward_masked.argtypes = [cp, vp, vp, vp, vp, vp, vp, vp, i64, vp]
        L.rev_stack_forward_masked.restype = ctypes.c_int
        bwm = [cp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64]
        L.rev_stack_backward_reprop_masked.argtypes = bwm + [vp]
        L.rev_stack_backward_reprop_masked.restype = ctypes.c_int
        L.rev_stack_backward_pareprop_masked.argtypes = bwm + [vp, vp]
        L.rev_stack_backward_pareprop_masked.restype = ctypes.c_int
        f32 = ctypes.c_float
        L.rev_adamw_step.argtypes = [i64, vp, vp, vp, vp, vp, i32, f32, f32, f32, f32, f32, vp]
        L.rev_adamw_step.restype = ctypes.c_int
        L.rev_sgd_step.argtypes = [i64, vp, vp, vp, f32, vp]
        L.rev_sgd_step.restype = ctypes.c_int
        mp = ctypes.POINTER(RevMergeCfg)
        L.rev_merge_check_cfg.argtypes = [mp]
        L.rev_merge_check_cfg.restype = ctypes.c_int
        for n in ("rev_merge_param_count", "rev_merge_workspace_bytes"):
            getattr(L, n).argtypes = [mp]
            getattr(L, n).restype = i64
        L.rev_merge_forward.argtypes = [mp, vp, vp, vp, vp, vp, i64, vp]
        L.rev_merge_forward.restype = ctypes.c_int
        L.rev_merge_backward.argtypes = [mp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp]
        L.rev_merge_backward.restype = ctypes.c_int
        for n in ("rev_profile_begin", "rev_profile_end", "rev_profile_kinds"):
            getattr(L, n).argtypes = []
            getattr(L, n).restype = ctypes.c_int
        L.rev_profile_name.argtypes = [ctypes.c_int]
        L.rev_profile_name.restype = ctypes.c_char_p
        L.rev_profile_is_flops.argtypes = [ctypes.c_int]
        L.rev_profile_is_flops.restype = ctypes.c_int
        L.rev_profile_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64),
                                      ctypes.POINTER(ctypes.c_double)]
        L.rev_profile_get.restype = ctypes.c_int
        L.rev_last_error.argtypes = []
        L.rev_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def make_cfg(n_blocks, d_model, n_heads, d_mlp, seq_len, batch, mode="bf16", ln_eps=1e-6, **_ignored) -> RevCfg:
    m = MODES[mode] if isinstance(mode, str) else int(mode)
    return RevCfg(n_blocks, d_model, n_heads, d_mlp, seq_len, batch, m, ln_eps)


def rev_last_error() -> str:
    return lib().rev_last_error().decode()


def _check(rc):
    if rc < 0:
        raise RevError(f"librevstack error {rc}: {rev_last_error()}")
    return rc


def rev_stack_check_cfg(cfg: RevCfg) -> int:
    return lib().rev_stack_check_cfg(ctypes.byref(cfg))


def rev_stack_param_count(cfg: RevCfg) -> int:
    return _check(lib().rev_stack_param_count(ctypes.byref(cfg)))


def rev_stack_param_offset(cfg: RevCfg, block: int, tensor: int):
    cnt = ctypes.c_int64(0)
    off = _check(lib().rev_stack_param_offset(ctypes.byref(cfg), block, tensor, ctypes.byref(cnt)))
    return off, cnt.value


def rev_stack_workspace_bytes(cfg: RevCfg) -> int:
    return _check(lib().rev_stack_workspace_bytes(ctypes.byref(cfg)))


def rev_stack_workspace_bytes_reprop(cfg: RevCfg) -> int:
    return _check(lib().rev_stack_workspace_bytes_reprop(ctypes.byref(cfg)))


def rev_stack_slot_bytes(cfg: RevCfg) -> int:
    return _check(lib().rev_stack_slot_bytes(ctypes.byref(cfg)))


def param_dtype(cfg: RevCfg):
    return torch.bfloat16 if cfg.mode == REV_MODE_BF16 else torch.float32


def alloc_workspace(cfg: RevCfg, device="cuda", reprop_only: bool = False) -> torch.Tensor:
    n = rev_stack_workspace_bytes_reprop(cfg) if reprop_only else rev_stack_workspace_bytes(cfg)
    return torch.empty(n, dtype=torch.uint8, device=device)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(s):
    if s is None:
        s = torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _want(t, dtype, shape=None):
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, "expected a contiguous CUDA tensor of " + str(dtype)
    if shape is not None:
        assert tuple(t.shape) == tuple(shape), f"shape {tuple(t.shape)} != {tuple(shape)}"


def rev_stack_forward(cfg, params, X1, X2, workspace=None, stream=None, Y1=None, Y2=None):
    shape = (cfg.batch, cfg.seq_len, cfg.d_model)
    _want(params, param_dtype(cfg), (rev_stack_param_count(cfg),))
    _want(X1, torch.float32, shape)
    _want(X2, torch.float32, shape)
    Y1 = torch.empty_like(X1) if Y1 is None else Y1
    Y2 = torch.empty_like(X2) if Y2 is None else Y2
    ws = alloc_workspace(cfg, X1.device) if workspace is None else workspace
    _check(lib().rev_stack_forward(ctypes.byref(cfg), _ptr(params), _ptr(X1), _ptr(X2), _ptr(Y1), _ptr(Y2),
                                   _ptr(ws), ws.numel(), _stream_handle(stream)))
    return Y1, Y2


def _backward_args(cfg, params, Y1, Y2, dY1, dY2, workspace, want_inputs, out):
    shape = (cfg.batch, cfg.seq_len, cfg.d_model)
    _want(params, param_dtype(cfg), (rev_stack_param_count(cfg),))
    for t in (Y1, Y2, dY1, dY2):
        _want(t, torch.float32, shape)
    if out is None:
        out = {}
    dX1 = out.get("dX1", None)
    dX1 = torch.empty_like(Y1) if dX1 is None else dX1
    dX2 = out.get("dX2", None)
    dX2 = torch.empty_like(Y1) if dX2 is None else dX2
    dparams = out.get("dparams", None)
    dparams = torch.empty(params.numel(), dtype=torch.float32, device=Y1.device) if dparams is None else dparams
    X1o = X2o = None
    if want_inputs:
        X1o = out.get("X1", None)
        X1o = torch.empty_like(Y1) if X1o is None else X1o
        X2o = out.get("X2", None)
        X2o = torch.empty_like(Y1) if X2o is None else X2o
    ws = alloc_workspace(cfg, Y1.device) if workspace is None else workspace
    res = {"dX1": dX1, "dX2": dX2, "dparams": dparams, "X1": X1o, "X2": X2o}
    args = [ctypes.byref(cfg), _ptr(params), _ptr(Y1), _ptr(Y2), _ptr(dY1), _ptr(dY2), _ptr(dX1), _ptr(dX2),
            _ptr(X1o), _ptr(X2o), _ptr(dparams), _ptr(ws), ws.numel()]
    return args, res


def rev_stack_backward_reprop(cfg, params, Y1, Y2, dY1, dY2, workspace=None, stream=None, want_inputs=False, out=None):
    args, res = _backward_args(cfg, params, Y1, Y2, dY1, dY2, workspace, want_inputs, out)
    _check(lib().rev_stack_backward_reprop(*args, _stream_handle(stream)))
    return res


STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024      # REV_STATIC_WORKSPACE_BYTES of the header


def rev_stack_backward_reprop_static(cfg, params, Y1, Y2, dY1, dY2, out, stream=None):
    """The sequential schedule in the library's built-in workspace: nothing is allocated, here or in the
    library, so `out` must hold dX1, dX2 and dparams (and X1, X2 if the reconstructed inputs are wanted)."""
    shape = (cfg.batch, cfg.seq_len, cfg.d_model)
    _want(params, param_dtype(cfg), (rev_stack_param_count(cfg),))
    for t in (Y1, Y2, dY1, dY2, out["dX1"], out["dX2"]):
        _want(t, torch.float32, shape)
    _want(out["dparams"], torch.float32, (params.numel(),))
    _check(lib().rev_stack_backward_reprop_static(
        ctypes.byref(cfg), _ptr(params), _ptr(Y1), _ptr(Y2), _ptr(dY1), _ptr(dY2), _ptr(out["dX1"]), _ptr(out["dX2"]),
        _ptr(out.get("X1")), _ptr(out.get("X2")), _ptr(out["dparams"]), _stream_handle(stream)))
    return out


def rev_stack_backward_pareprop(cfg, params, Y1, Y2, dY1, dY2, stream_recompute, workspace=None, stream_grad=None,
                                want_inputs=False, out=None):
    args, res = _backward_args(cfg, params, Y1, Y2, dY1, dY2, workspace, want_inputs, out)
    _check(lib().rev_stack_backward_pareprop(*args, _stream_handle(stream_grad), _stream_handle(stream_recompute)))
    return res


def _want_key_len(cfg, key_len):
    _want(key_len, torch.int32, (cfg.batch,))


def rev_stack_forward_masked(cfg, params, X1, X2, key_len, workspace=None, stream=None, Y1=None, Y2=None):
    """rev_stack_forward with a key-padding mask: key_len is an int32 CUDA tensor [batch] of valid lengths."""
    shape = (cfg.batch, cfg.seq_len, cfg.d_model)
    _want(params, param_dtype(cfg), (rev_stack_param_count(cfg),))
    _want(X1, torch.float32, shape)
    _want(X2, torch.float32, shape)
    _want_key_len(cfg, key_len)
    Y1 = torch.empty_like(X1) if Y1 is None else Y1
    Y2 = torch.empty_like(X2) if Y2 is None else Y2
    ws = alloc_workspace(cfg, X1.device) if workspace is None else workspace
    _check(lib().rev_stack_forward_masked(ctypes.byref(cfg), _ptr(params), _ptr(X1), _ptr(X2), _ptr(key_len), _ptr(Y1),
                                          _ptr(Y2), _ptr(ws), ws.numel(), _stream_handle(stream)))
    return Y1, Y2


def _masked(args, key_len):
    return args[:4] + [_ptr(key_len)] + args[4:]


def rev_stack_backward_reprop_masked(cfg, params, Y1, Y2, key_len, dY1, dY2, workspace=None, stream=None,
                                     want_inputs=False, out=None):
    _want_key_len(cfg, key_len)
    args, res = _backward_args(cfg, params, Y1, Y2, dY1, dY2, workspace, want_inputs, out)
    _check(lib().rev_stack_backward_reprop_masked(*_masked(args, key_len), _stream_handle(stream)))
    return res


def rev_stack_backward_pareprop_masked(cfg, params, Y1, Y2, key_len, dY1, dY2, stream_recompute, workspace=None,
                                       stream_grad=None, want_inputs=False, out=None):
    _want_key_len(cfg, key_len)
    args, res = _backward_args(cfg, params, Y1, Y2, dY1, dY2, workspace, want_inputs, out)
    _check(lib().rev_stack_backward_pareprop_masked(*_masked(args, key_len), _stream_handle(stream_grad),
                                                    _stream_handle(stream_recompute)))
    return res


def rev_stack_backward_chain(cfg, params, Y1, Y2, dY1, dY2, chain, workspace=None, stream=None, want_inputs=False,
                             out=None):
    args, res = _backward_args(cfg, params, Y1, Y2, dY1, dY2, workspace, want_inputs, out)
    _check(lib().rev_stack_backward_chain(*args, _stream_handle(stream), int(chain)))
    return res


def rev_adamw_step(master, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01,
                   params_bf16=None, stream=None):
    """In-place AdamW update of the float32 `master` weights and moments `m`, `v` from the float32
    gradient; `params_bf16` (optional) receives the bf16 copy of the new weights."""
    for t in (master, grad, m, v):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == master.numel()
    if params_bf16 is not None:
        assert params_bf16.is_cuda and params_bf16.dtype == torch.bfloat16 and params_bf16.is_contiguous()
        assert params_bf16.numel() == master.numel()
    _check(lib().rev_adamw_step(master.numel(), _ptr(master), _ptr(params_bf16), _ptr(grad), _ptr(m), _ptr(v),
                                int(step), lr, beta1, beta2, eps, weight_decay, _stream_handle(stream)))


def rev_sgd_step(master, grad, lr, params_bf16=None, stream=None):
    """In-place plain SGD update of the float32 `master` weights; `params_bf16` (optional) receives the bf16 copy."""
    for t in (master, grad):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == master.numel()
    if params_bf16 is not None:
        assert params_bf16.is_cuda and params_bf16.dtype == torch.bfloat16 and params_bf16.is_contiguous()
        assert params_bf16.numel() == master.numel()
    _check(lib().rev_sgd_step(master.numel(), _ptr(master), _ptr(params_bf16), _ptr(grad), lr, _stream_handle(stream)))


FUSIONS = {"average": 0, "mlp": 1}


def make_merge_cfg(batch, grid_h, grid_w, window, d_in, mode="bf16", ln_eps=1e-5, fusion="average") -> RevMergeCfg:
    m = MODES[mode] if isinstance(mode, str) else int(mode)
    f = FUSIONS[fusion] if isinstance(fusion, str) else int(fusion)
    return RevMergeCfg(batch, grid_h, grid_w, window, d_in, m, ln_eps, f)


def rev_merge_check_cfg(cfg: RevMergeCfg) -> int:
    return lib().rev_merge_check_cfg(ctypes.byref(cfg))


def rev_merge_param_count(cfg: RevMergeCfg) -> int:
    return _check(lib().rev_merge_param_count(ctypes.byref(cfg)))


def rev_merge_workspace_bytes(cfg: RevMergeCfg) -> int:
    return _check(lib().rev_merge_workspace_bytes(ctypes.byref(cfg)))


def _merge_shapes(cfg):
    m_in = cfg.batch * cfg.grid_h * cfg.grid_w
    return (m_in, cfg.d_in), (m_in // 4, 2 * cfg.d_in)


def rev_merge_forward(cfg, params, X1, X2, workspace=None, stream=None, out=None):
    """Stage transition: average of the two streams, 2x2 patch merging, LayerNorm, linear map 4C -> 2C."""
    s_in, s_out = _merge_shapes(cfg)
    _want(params, param_dtype(cfg), (rev_merge_param_count(cfg),))
    _want(X1, torch.float32, s_in)
    _want(X2, torch.float32, s_in)
    out = torch.empty(s_out, dtype=torch.float32, device=X1.device) if out is None else out
    _want(out, torch.float32, s_out)
    ws = torch.empty(rev_merge_workspace_bytes(cfg), dtype=torch.uint8, device=X1.device) if workspace is None else workspace
    _check(lib().rev_merge_forward(ctypes.byref(cfg), _ptr(params), _ptr(X1), _ptr(X2), _ptr(out), _ptr(ws), ws.numel(),
                                   _stream_handle(stream)))
    return out


def rev_merge_backward(cfg, params, X1, X2, dOutA, dOutB, workspace=None, stream=None, out=None):
    """Backward of the stage transition; dOutA and dOutB are the cotangents of the two copies of its output."""
    s_in, s_out = _merge_shapes(cfg)
    _want(params, param_dtype(cfg), (rev_merge_param_count(cfg),))
    for t in (X1, X2):
        _want(t, torch.float32, s_in)
    for t in (dOutA, dOutB):
        _want(t, torch.float32, s_out)
    out = {} if out is None else out
    dX1 = out.get("dX1")
    dX1 = torch.empty_like(X1) if dX1 is None else dX1
    dX2 = out.get("dX2")
    dX2 = torch.empty_like(X1) if dX2 is None else dX2
    dparams = out.get("dparams")
    dparams = torch.empty(params.numel(), dtype=torch.float32, device=X1.device) if dparams is None else dparams
    for t, shp in ((dX1, s_in), (dX2, s_in), (dparams, (params.numel(),))):
        _want(t, torch.float32, shp)
    ws = torch.empty(rev_merge_workspace_bytes(cfg), dtype=torch.uint8, device=X1.device) if workspace is None else workspace
    _check(lib().rev_merge_backward(ctypes.byref(cfg), _ptr(params), _ptr(X1), _ptr(X2), _ptr(dOutA), _ptr(dOutB),
                                    _ptr(dX1), _ptr(dX2), _ptr(dparams), _ptr(ws), ws.numel(), _stream_handle(stream)))
    return {"dX1": dX1, "dX2": dX2, "dparams": dparams}


def rev_profile_begin():
    _check(lib().rev_profile_begin())


def rev_profile_end():
    """Stops recording and returns {family: (total_ms, launches, work, is_flops)}."""
    L = lib()
    _check(L.rev_profile_end())
    out = {}
    for k in range(L.rev_profile_kinds()):
        ms, n, w = ctypes.c_double(0), ctypes.c_int64(0), ctypes.c_double(0)
        _check(L.rev_profile_get(k, ctypes.byref(ms), ctypes.byref(n), ctypes.byref(w)))
        out[L.rev_profile_name(k).decode()] = (ms.value, n.value, w.value, bool(L.rev_profile_is_flops(k)))
    return out
