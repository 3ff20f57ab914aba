"""GPU parity: the HIP path, called through the C-ABI binding, against the fp64
CPU oracle on the same seeded inputs.  Tolerances and the error measure are in
parity_util (1e-4 float32 mode, 3e-2 bf16 mode, max-abs error over max-abs
reference, per tensor).  PaReprop must equal Reprop bit for bit."""
import numpy as np
import pytest
import torch

from oracle import rev_oracle as O
from paper_2306_09342_amd import binding as B
from paper_2306_09342_amd import synth

from parity_util import TOL, compare_backward, gpu_cfg, make_case, oracle_forward, rel_err, to_dev

pytestmark = pytest.mark.gpu

# small shapes that still span several tiles and ragged tails: M = B*T is not a
# multiple of 64, T is odd, head_dim 64 / 80 / 32 / 128
SHAPES = {
    "tiny": dict(synth.CONFIGS["tiny"]),
    "ragged_dh64": dict(n_blocks=2, d_model=128, n_heads=2, d_mlp=512, seq_len=77, batch=3),
    "ragged_dh80": dict(n_blocks=2, d_model=160, n_heads=2, d_mlp=328, seq_len=51, batch=2),
    "dh128_T1": dict(n_blocks=2, d_model=256, n_heads=2, d_mlp=264, seq_len=1, batch=5),
    "vit_s_slice": dict(n_blocks=3, d_model=384, n_heads=6, d_mlp=1536, seq_len=197, batch=3),
    "one_sample_T300": dict(n_blocks=1, d_model=64, n_heads=2, d_mlp=64, seq_len=300, batch=1),
    # window-attention shaped stages (49 tokens, head_dim 32): narrow first stage, many-headed last stage
    "window_stage1": dict(n_blocks=2, d_model=96, n_heads=3, d_mlp=384, seq_len=49, batch=7),
    "window_stage4": dict(n_blocks=1, d_model=768, n_heads=24, d_mlp=3072, seq_len=49, batch=2),
    # the largest head the one-workgroup attention backward takes (256 tokens, 8 wavefronts, 133 KB of LDS), a ragged
    # length just below it, and the first length beyond it (two-kernel path again)
    "dh64_T256": dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=128, seq_len=256, batch=2),
    "dh64_T231": dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=128, seq_len=231, batch=1),
    "dh64_T257": dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=128, seq_len=257, batch=1),
    # 32-wide heads beyond one window: 7 wavefronts with a ragged tail, a single partial row tile, and the 256-token limit
    "dh32_T200": dict(n_blocks=1, d_model=64, n_heads=2, d_mlp=128, seq_len=200, batch=2),
    "dh32_T20": dict(n_blocks=2, d_model=64, n_heads=2, d_mlp=128, seq_len=20, batch=3),
    "dh32_T256": dict(n_blocks=1, d_model=64, n_heads=2, d_mlp=128, seq_len=256, batch=1),
    # 1024 tokens: keys and values no longer fit the on-chip tile pair, the streamed attention path runs
    "T1024_dh64": dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=128, seq_len=1024, batch=1),
}


def _run_case(name, mode, seed=0):
    cfg = dict(SHAPES[name])
    cfg["mode"] = mode
    print(f"[case] {name} mode={mode} seed={seed} cfg={cfg}", flush=True)
    flat, blocks, x, dy1, dy2 = make_case(cfg, seed=seed)
    x2 = x[:, ::-1].copy()                      # distinct streams so a swap shows
    H = cfg["n_heads"]
    y1, y2 = oracle_forward(cfg, blocks, x, x2)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)
    ref = O.stack_backward_reversible_chunked(y1f, y2f, blocks, H, dy1, dy2)

    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    ws = B.alloc_workspace(c)
    # forward parity
    gy1, gy2 = B.rev_stack_forward(c, params, to_dev(x), to_dev(x2), workspace=ws)
    torch.cuda.synchronize()
    tol = TOL[mode]
    assert rel_err(gy1.cpu().numpy(), y1) <= tol and rel_err(gy2.cpu().numpy(), y2) <= tol
    # backward parity, both schedules
    dY1, dY2, Y1, Y2 = to_dev(dy1), to_dev(dy2), to_dev(y1f), to_dev(y2f)
    rep = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    worst = compare_backward(cfg, rep, ref, tol, what=f"{name}/{mode}/reprop")
    side = torch.cuda.Stream()
    par = B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws, want_inputs=True)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams", "X1", "X2"):
        assert torch.equal(rep[k], par[k]), f"PaReprop differs from Reprop in {k}"
    # the reconstructed inputs are the true inputs
    assert rel_err(rep["X1"].cpu().numpy(), x) <= tol and rel_err(rep["X2"].cpu().numpy(), x2) <= tol
    print(f"[ok] {name}/{mode}: worst {max(worst.values()):.3e} at {max(worst, key=worst.get)}", flush=True)


@pytest.mark.parametrize("name", list(SHAPES))
def test_fp32_mode_matches_oracle(name):
    _run_case(name, "fp32")


@pytest.mark.parametrize("name", list(SHAPES))
def test_bf16_mode_matches_oracle(name):
    _run_case(name, "bf16")


# Shapes whose forward-form GEMMs the sequential schedule and the forward map run with 160-row tiles
# (128-row tiles would leave a short second round of workgroups) while PaReprop keeps 128-row tiles:
# oracle parity of the tall-tile kernel with the bias+GELU epilogue (first shape: the wide fc1) and with
# the residual epilogue (second shape: proj and fc2 of a narrow layer over 81 920 tokens), and
# bit-identity of the two schedules across the two tile shapes.
TALL_SHAPES = {
    "tall_fc1": dict(n_blocks=1, d_model=256, n_heads=4, d_mlp=8192, seq_len=64, batch=20),
    "tall_narrow": dict(n_blocks=1, d_model=128, n_heads=2, d_mlp=512, seq_len=64, batch=1280),
}
SHAPES.update(TALL_SHAPES)


@pytest.mark.parametrize("name", list(TALL_SHAPES))
def test_tall_tile_shapes_match_oracle_bf16(name):
    _run_case(name, "bf16")


def test_paper_recipe_inputs_tiny_fp32():
    """The tiny config exactly as specified: X duplicated to both streams, unit
    gains, zero biases, seed 0."""
    cfg = dict(synth.CONFIGS["tiny"])
    flat = synth.make_params(cfg, seed=0)
    x, dy1, dy2 = synth.make_inputs(cfg, seed=0)
    blocks = O.unpack_params(flat, cfg["n_blocks"], cfg["d_model"], cfg["d_mlp"])
    y1, y2 = oracle_forward(cfg, blocks, x, x)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)
    ref = O.stack_backward_reversible_chunked(y1f, y2f, blocks, cfg["n_heads"], dy1, dy2)
    c = gpu_cfg(cfg)
    res = B.rev_stack_backward_reprop(c, to_dev(flat), to_dev(y1f), to_dev(y2f), to_dev(dy1), to_dev(dy2),
                                      want_inputs=True)
    torch.cuda.synchronize()
    compare_backward(cfg, res, ref, TOL["fp32"], what="tiny recipe")


def test_outputs_do_not_depend_on_stale_workspace_or_repeat():
    """Two calls in a row on a workspace filled with NaN bytes give identical bits."""
    cfg = dict(SHAPES["ragged_dh64"], mode="bf16")
    flat, blocks, x, dy1, dy2 = make_case(cfg, seed=3)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    ws = B.alloc_workspace(c)
    Y1, Y2 = B.rev_stack_forward(c, params, to_dev(x), to_dev(x), workspace=ws)
    ws.fill_(0xFF)
    a = B.rev_stack_backward_reprop(c, params, Y1, Y2, to_dev(dy1), to_dev(dy2), workspace=ws)
    torch.cuda.synchronize()
    ws.fill_(0x7F)
    side = torch.cuda.Stream()
    b = B.rev_stack_backward_pareprop(c, params, Y1, Y2, to_dev(dy1), to_dev(dy2), side, workspace=ws)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams"):
        assert torch.isfinite(a[k]).all()
        assert torch.equal(a[k], b[k]), k


def test_short_workspace_is_an_error_on_the_gpu_too():
    cfg = dict(SHAPES["tiny"])
    c = gpu_cfg(cfg)
    flat, _, x, _, _ = make_case(cfg)
    ws = torch.empty(B.rev_stack_workspace_bytes_reprop(c) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.RevError, match="workspace too small"):
        B.rev_stack_forward(c, to_dev(flat), to_dev(x), to_dev(x), workspace=ws)


@pytest.mark.parametrize("name,mode", [("tiny", "fp32"), ("ragged_dh64", "bf16"), ("vit_s_slice", "bf16")])
def test_reprop_in_its_smaller_workspace_gives_the_same_bits(name, mode):
    """The sequential schedule and the forward map run in the one-slot workspace
    (guard bytes behind it stay untouched) and return exactly what they return in
    the large one; the parallel schedule refuses the small one."""
    cfg = dict(SHAPES[name], mode=mode)
    print(f"[case] small workspace {name} mode={mode}", flush=True)
    flat, blocks, x, dy1, dy2 = make_case(cfg, seed=5)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    small = B.rev_stack_workspace_bytes_reprop(c)
    assert small < B.rev_stack_workspace_bytes(c)
    guard = 4096
    buf = torch.empty(small + guard, dtype=torch.uint8, device="cuda")
    buf.fill_(0xA5)
    ws_small, ws_full = buf[:small], B.alloc_workspace(c)
    X, dY1, dY2 = to_dev(x), to_dev(dy1), to_dev(dy2)
    Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws_full)
    y1s, y2s = B.rev_stack_forward(c, params, X, X, workspace=ws_small)
    torch.cuda.synchronize()
    assert torch.equal(Y1, y1s) and torch.equal(Y2, y2s)
    a = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws_full, want_inputs=True)
    b = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2, workspace=ws_small, want_inputs=True)
    side = torch.cuda.Stream()
    p = B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws_full, want_inputs=True)
    torch.cuda.synchronize()
    for k in ("dX1", "dX2", "dparams", "X1", "X2"):
        assert torch.equal(a[k], b[k]) and torch.equal(a[k], p[k]), k
    assert bool((buf[small:] == 0xA5).all()), "wrote past the small workspace"
    with pytest.raises(B.RevError, match="workspace too small"):
        B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws_small)


def test_pareprop_call_can_be_captured_into_a_graph_and_replayed():
    """The two-stream call enqueues only kernels and event waits, so a caller may capture it into a
    HIP graph (both streams join the capture through the call's own fork / join events).  Replays,
    with eager work and a scrambled workspace in between, reproduce the eager bits."""
    cfg = dict(SHAPES["ragged_dh64"], mode="bf16")
    flat, blocks, x, dy1, dy2 = make_case(cfg, seed=7)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    ws = B.alloc_workspace(c)
    X, dY1, dY2 = to_dev(x), to_dev(dy1), to_dev(dy2)
    Y1, Y2 = B.rev_stack_forward(c, params, X, X, workspace=ws)
    side = torch.cuda.Stream()
    out = {}
    out.update(B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws, want_inputs=True))
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in out.items()}
    cap = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, side, workspace=ws, want_inputs=True, out=out)
    torch.cuda.synchronize()
    for rep in range(3):
        for v in out.values():
            v.zero_()
        ws.fill_(0x7F)
        eager = B.rev_stack_backward_reprop(c, params, Y1, Y2, dY1, dY2)      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(out[k], ref[k]), (rep, k)
            assert torch.equal(eager[k], ref[k]) if eager.get(k) is not None else True


def test_gelu_tails_bf16_large_preactivations():
    """fc1 weights and biases scaled so that the MLP pre-activations reach |h| of 10 and more: the bf16 GELU
    and GELU' epilogues (a polynomial for the normal CDF inside |h| <= 3.8, exactly 0 / 1 beyond) against the
    oracle's erf form, through the forward map, the inversion and the gradient step."""
    cfg = dict(n_blocks=2, d_model=128, n_heads=2, d_mlp=512, seq_len=77, batch=3, mode="bf16")
    flat, _, x, dy1, dy2 = make_case(cfg, seed=11)
    D, Dm = cfg["d_model"], cfg["d_mlp"]
    per = synth.params_per_block(D, Dm)
    rng = np.random.default_rng(5)
    for blk in range(cfg["n_blocks"]):
        off = blk * per
        for tname, shape in synth.block_tensors(D, Dm):
            n = int(np.prod(shape))
            if tname == "w_fc1":
                flat[off:off + n] *= 20.0
            if tname == "b_fc1":
                flat[off:off + n] = 2.0 * rng.standard_normal(n)
            off += n
    flat = synth.to_bf16_grid(flat)
    blocks = O.unpack_params(flat, cfg["n_blocks"], D, Dm)
    H = cfg["n_heads"]
    # how far the pre-activations of the first block's MLP reach (oracle)
    y1_0 = x.astype(np.float64) + O.F_forward(x.astype(np.float64), blocks[0], H, 1e-6)[0]
    h = O.layer_norm(y1_0, blocks[0]["ln2_g"], blocks[0]["ln2_b"], 1e-6)[0] @ blocks[0]["w_fc1"].T + blocks[0]["b_fc1"]
    frac_tail = float((np.abs(h) > 3.8).mean())
    print(f"[case] gelu tails: max|h| {np.abs(h).max():.1f}, {100 * frac_tail:.1f} % beyond 3.8", flush=True)
    assert np.abs(h).max() > 10 and frac_tail > 0.2 and float((h < -3.8).mean()) > 0.1
    y1, y2 = oracle_forward(cfg, blocks, x, x)
    y1f, y2f = y1.astype(np.float32), y2.astype(np.float32)
    ref = O.stack_backward_reversible_chunked(y1f, y2f, blocks, H, dy1, dy2)
    c = gpu_cfg(cfg)
    params = to_dev(flat, B.param_dtype(c))
    gy1, gy2 = B.rev_stack_forward(c, params, to_dev(x), to_dev(x))
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    assert rel_err(gy1.cpu().numpy(), y1) <= tol and rel_err(gy2.cpu().numpy(), y2) <= tol
    rep = B.rev_stack_backward_reprop(c, params, to_dev(y1f), to_dev(y2f), to_dev(dy1), to_dev(dy2), want_inputs=True)
    torch.cuda.synchronize()
    worst = compare_backward(cfg, rep, ref, tol, what="gelu tails")
    print(f"[ok] gelu tails: worst {max(worst.values()):.3e} at {max(worst, key=worst.get)}", flush=True)


def test_two_host_threads_issue_pareprop_calls_concurrently():
    """Two host threads, each with its own workspace, stream pair, inputs and outputs, enqueue two-stream calls
    at the same time (each call leases its own events): every result equals, bit for bit, what the same call
    returns when it is the only one in flight."""
    import threading
    cfgs = [dict(SHAPES["ragged_dh64"], mode="bf16"), dict(SHAPES["vit_s_slice"], mode="bf16")]
    jobs = []
    for i, cfg in enumerate(cfgs):
        flat, _, x, dy1, dy2 = make_case(cfg, seed=20 + i)
        c = gpu_cfg(cfg)
        params = to_dev(flat, B.param_dtype(c))
        X, dY1, dY2 = to_dev(x), to_dev(dy1), to_dev(dy2)
        Y1, Y2 = B.rev_stack_forward(c, params, X, X)
        torch.cuda.synchronize()
        ws = B.alloc_workspace(c)
        sg, sr = torch.cuda.Stream(), torch.cuda.Stream()
        alone = B.rev_stack_backward_pareprop(c, params, Y1, Y2, dY1, dY2, sr, workspace=ws, stream_grad=sg)
        torch.cuda.synchronize()
        jobs.append(dict(c=c, params=params, Y1=Y1, Y2=Y2, dY1=dY1, dY2=dY2, ws=ws, sg=sg, sr=sr,
                         alone={k: v.clone() for k, v in alone.items() if v is not None}, results=[], err=None))
    start = threading.Barrier(len(jobs))

    def worker(j):
        try:
            torch.cuda.set_device(0)
            start.wait()
            for _ in range(6):
                out = B.rev_stack_backward_pareprop(j["c"], j["params"], j["Y1"], j["Y2"], j["dY1"], j["dY2"], j["sr"],
                                                    workspace=j["ws"], stream_grad=j["sg"])
                j["sg"].synchronize()
                j["results"].append({k: v.clone() for k, v in out.items() if v is not None})
        except Exception as e:          # surfaces in the main thread
            j["err"] = e

    threads = [threading.Thread(target=worker, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for j in jobs:
        assert j["err"] is None, j["err"]
        assert len(j["results"]) == 6
        for r in j["results"]:
            for k, v in j["alone"].items():
                assert torch.equal(r[k], v), k
