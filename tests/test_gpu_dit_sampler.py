"""GPU parity of dit_forward and sampler_run against the CPU oracle, through the C ABI.

fp32 (tiny network): 1e-4 relative on eps, on every per-step sample and on the per-step
relative MAEs.  bf16 (CogVideoX-2b width): rel-MAE <= 2e-2 against the float64 oracle run
on the same bf16-rounded weights and inputs.
"""
import numpy as np
import pytest
import torch

from oracle import parastep_oracle as O
from paper_2505_14741_amd import binding as B
from paper_2505_14741_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a, dtype=torch.float32):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(DEV)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def close_fp32(got, ref, tol=1e-4):
    scale = max(np.abs(ref).max(), 1e-30)
    err = np.abs(got - ref).max()
    assert err <= tol * scale, (err, scale)
    assert O.rel_mae(ref, got)[2] <= tol


def worst_token(ref, got, patch):
    """Largest per-token relative MAE of a predicted latent [B, C, F, H, W] (tokens = patches)."""
    worst = 0.0
    for b in range(ref.shape[0]):
        r, g = O.patchify(ref[b], patch), O.patchify(got[b], patch)
        per = np.abs(r - g).sum(axis=1) / np.maximum(np.abs(r).sum(axis=1), 1e-30)
        worst = max(worst, float(per.max()))
    return worst


# bf16 whole-forward bound per token: the global bar is 2e-2 rel-MAE; a single token (64 output values at
# the CogVideoX-2b shape) may lie above the average, a wrong tile of rows lies far above it (rel-MAE ~ 1)
WORST_TOKEN_BF16 = 6e-2

_CACHE = {}


def setup(name, init="std002", cfg=None):
    """Weights (host copy for the oracle, device copy behind a dit handle), cached per case."""
    cfg = cfg or I.CONFIGS[name]
    key = (name, init, cfg.layers)
    if key not in _CACHE:
        weights = I.make_weights(cfg, I.WEIGHT_SEED.get(name, 1000), init)
        _CACHE[key] = (cfg, dict(weights), B.dit_create(cfg, B.weights_to_device(cfg, weights)))
    return _CACHE[key]


# ----------------------------------------------------------------------------- dit_forward
@pytest.mark.parametrize("name", ["tiny", "tiny_text"])
@pytest.mark.parametrize("init", ["std002", "unit"])
def test_tiny_forward_fp32(name, init):
    print(f"dit_forward {name} {init}", flush=True)
    cfg, W, d = setup(name, init)
    x, ctx = I.make_latent(cfg, 2), I.make_context(cfg, 2)
    t = [875, 125]
    eps = host(B.dit_forward(d, dev(x), dev(ctx), t))
    ref = O.dit_forward(cfg, W, x, ctx, t)
    close_fp32(eps, ref)


def test_tiny_forward_batch_invariance_bitwise():
    cfg, W, d = setup("tiny_text", "unit")
    x, ctx = dev(I.make_latent(cfg, 4)), dev(I.make_context(cfg, 4))
    t = [875, 625, 375, 0]
    full = B.dit_forward(d, x, ctx, t).clone()
    for b in range(4):
        one = B.dit_forward(d, x[b:b + 1].contiguous(), ctx[b:b + 1].contiguous(), t[b:b + 1])
        assert torch.equal(one[0], full[b]), b


@pytest.mark.parametrize("init", ["std002", "unit"])
def test_reduced_30_layer_forward_bf16(init):
    """All 30 layers at width 1920 on 112 tokens: whole-model parity the oracle can afford."""
    print(f"dit_forward reduced {init}", flush=True)
    cfg, W, d = setup("reduced", init)
    x, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    eps = host(B.dit_forward(d, dev(x), dev(ctx, torch.bfloat16), [500]))
    ref = O.dit_forward(cfg, W, x, ctx, [500])
    r = O.rel_mae(ref, eps)[2]
    worst = worst_token(ref, eps, cfg.patch)
    print(f"  rel-MAE {r:.3e}, worst token {worst:.3e}", flush=True)
    assert r <= 2e-2 and np.isfinite(eps).all()
    assert worst <= WORST_TOKEN_BF16


def test_reduced_forward_generic_and_mfma_paths_agree():
    cfg, W, d = setup("reduced", "unit", cfg=I.CONFIGS["reduced"].with_(layers=2))
    x, ctx = dev(I.make_latent(cfg, 1)), dev(I.make_context(cfg, 1), torch.bfloat16)
    fast = host(B.dit_forward(d, x, ctx, [300]))
    B.dit_set_kernel_path(d, 1)
    try:
        slow = host(B.dit_forward(d, x, ctx, [300]))
    finally:
        B.dit_set_kernel_path(d, 0)
    assert O.rel_mae(slow, fast)[2] < 1e-2


def test_reduced_forward_bf16_batch_of_three():
    """Batch 3 with different timesteps on the MFMA kernels: 3 x 112 token rows, fewer than one tile of
    rows per sample (every workgroup works on one sample; partial tiles in every projection).  Every sample
    against the oracle, and against the same sample run alone (bitwise: rows do not interact)."""
    cfg, W, d = setup("reduced", "unit", cfg=I.CONFIGS["reduced"].with_(layers=2))
    x, ctx = I.make_latent(cfg, 3), I.make_context(cfg, 3)
    t = [900, 500, 20]
    xd, cd = dev(x), dev(ctx, torch.bfloat16)
    eps = B.dit_forward(d, xd, cd, t)
    ref = O.dit_forward(cfg, W, x, ctx, t)
    for b in range(3):
        r = O.rel_mae(ref[b], host(eps[b]))[2]
        print(f"  sample {b} rel-MAE {r:.3e}", flush=True)
        assert r <= 2e-2
        one = B.dit_forward(d, xd[b:b + 1].contiguous(), cd[b:b + 1].contiguous(), t[b:b + 1])
        assert torch.equal(one[0], eps[b]), b


@pytest.mark.parametrize("init", ["std002", "unit"])
def test_block_forward_bf16_whole(init):
    """One block at CogVideoX-2b width, 4290 video + 226 text tokens, whole output vs oracle."""
    print(f"dit_forward block {init}", flush=True)
    cfg, W, d = setup("block", init)
    x, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    eps = host(B.dit_forward(d, dev(x), dev(ctx, torch.bfloat16), [500]))
    ref = O.dit_forward(cfg, W, x, ctx, [500])
    r = O.rel_mae(ref, eps)[2]
    worst = worst_token(ref, eps, cfg.patch)
    print(f"  rel-MAE {r:.3e}, worst token {worst:.3e}", flush=True)
    assert r <= 2e-2
    assert worst <= WORST_TOKEN_BF16


@pytest.mark.parametrize("name", ["full", "long"])
def test_single_layer_forward_at_the_full_token_count_sampled_patches(name):
    """One layer on the 13x60x90 latent (17550 video + 226 text tokens: the launch shapes the benchmark times)
    and on the 25x60x90 latent (33750 + 226).

    The oracle evaluates attention for the listed tokens only (all keys and values take part); their patches
    are compared.  The list holds the first and last token, neighbours across a patch row, a frame and the last
    full 256-row tile of the projections, and seeded random tokens.
    """
    cfg = I.CONFIGS[name].with_(layers=1)
    print(f"dit_forward single layer, {cfg.tokens} tokens", flush=True)
    _, W, d = setup(name, "std002", cfg)
    x, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    eps = host(B.dit_forward(d, dev(x), dev(ctx, torch.bfloat16), [500]))
    assert np.isfinite(eps).all()
    Wp, per_frame = cfg.grid[2], cfg.grid[1] * cfg.grid[2]
    edge = cfg.tokens // 256 * 256 - cfg.text_tokens          # first video token of the projections' last row tile
    video = np.array([0, 1, Wp - 1, Wp, per_frame - 1, per_frame, edge - 1, edge, cfg.video_tokens - 1])
    video = np.unique(np.concatenate([video, np.random.default_rng(77).integers(0, cfg.video_tokens, 40)]))
    ref = O.dit_forward(cfg, W, x, ctx, [500], query_rows=cfg.text_tokens + video)
    got = O.patchify(eps[0], cfg.patch)[video]
    want = O.patchify(ref[0], cfg.patch)[video]
    assert np.isfinite(want).all()
    r = O.rel_mae(want, got)[2]
    worst = max(O.rel_mae(want[i], got[i])[2] for i in range(len(video)))
    print(f"  rel-MAE {r:.3e}, worst token {worst:.3e}", flush=True)
    assert r <= 2e-2 and worst <= 4e-2


# ----------------------------------------------------------------------------- sampler_run
def oracle_run(cfg, W, x_T, ctx, S, m, cyc, mode="reuse_then_predict"):
    tau, a, b = O.ddim_coefficients(steps=S)
    f = lambda x, t: O.dit_forward(cfg, W, x[None], ctx, [t])[0]
    return O.run_sampler(f, x_T[0], tau, a, b, warmup=m, cycle_len=cyc, mode=mode)


def gpu_run(d, x_T, ctx, S, m, cyc, batched=False, mode=0):
    ts, a, b = B.ddim_coefficients(S)
    sched = B.Schedule(ts, a, b, m, cyc, batched=batched, mode=mode)
    x0, sums, calls = B.sampler_run(d, sched, x_T, ctx)
    torch.cuda.synchronize()
    return x0, sums, calls


@pytest.mark.parametrize("name,init,S,m,cyc", [
    ("tiny", "std002", 8, 2, [2, 2, 2]),
    ("tiny", "unit", 8, 2, [2, 2, 2]),
    ("tiny_text", "unit", 7, 1, [3, 3]),
    ("tiny", "unit", 6, 2, [3, 3]),            # run ends mid-cycle
    ("tiny_text", "unit", 10, 1, [1, 2, 4, 2]),  # changing cycle lengths
])
def test_tiny_run_matches_oracle(name, init, S, m, cyc):
    print(f"sampler_run {name} {init} S={S} m={m} cyc={cyc}", flush=True)
    cfg, W, d = setup(name, init)
    x_T, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    ref = oracle_run(cfg, W, x_T, ctx, S, m, cyc)
    x0, sums, calls = gpu_run(d, dev(x_T), dev(ctx), S, m, cyc)
    assert calls == S == ref["calls"]
    close_fp32(host(x0)[0], ref["x0"])
    s = host(sums)
    rx = s[:, 0] / s[:, 1]
    re = s[1:, 2] / s[1:, 3]
    np.testing.assert_allclose(rx, ref["rx"], rtol=1e-4)
    np.testing.assert_allclose(re, ref["re"][1:], rtol=1e-4, atol=1e-7)
    assert s[0, 2] == 0.0


@pytest.mark.parametrize("S,m,cyc", [(8, 2, [2, 2, 2]), (9, 1, [4, 4]), (7, 1, [3, 3]), (10, 1, [1, 2, 4, 2])])
def test_batched_run_equals_unbatched_bitwise(S, m, cyc):
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = dev(I.make_latent(cfg, 1)), dev(I.make_context(cfg, 1))
    x0a, sa, ca = gpu_run(d, x_T, ctx, S, m, cyc, batched=False)
    x0b, sb, cb = gpu_run(d, x_T, ctx, S, m, cyc, batched=True)
    assert torch.equal(x0a, x0b) and torch.equal(sa, sb)
    assert ca == S and cb == m + len(O.expand_cycles(S, m, cyc))


def test_window_one_is_the_plain_loop_bitwise():
    cfg, W, d = setup("tiny", "unit")
    x_T = dev(I.make_latent(cfg, 1))
    S = 8
    ts, a, b = B.ddim_coefficients(S)
    x = x_T.clone()
    for i in range(S):
        eps = B.dit_forward(d, x, None, [int(ts[i])])
        x, _ = B.sampler_step(x, eps, None, float(a[i]), float(b[i]), want_sums=False)
    for m, cyc in [(0, [1] * S), (S, []), (3, [1] * S)]:
        x0, _, calls = gpu_run(d, x_T, None, S, m, cyc)
        assert torch.equal(x0, x) and calls == S


def test_direct_reuse_matches_oracle():
    cfg, W, d = setup("tiny", "unit")
    x_T = I.make_latent(cfg, 1)
    ref = oracle_run(cfg, W, x_T, None, 7, 1, [2, 2, 2], mode="direct_reuse")
    x0, sums, calls = gpu_run(d, dev(x_T), None, 7, 1, [2, 2, 2], mode=1)
    assert calls == 4 == ref["calls"]
    close_fp32(host(x0)[0], ref["x0"])
    s = host(sums)
    np.testing.assert_allclose(s[:, 0] / s[:, 1], ref["rx"], rtol=1e-4)


@pytest.mark.parametrize("S,m,cyc", [(7, 1, [3, 3]), (10, 1, [1, 2, 4, 2]), (12, 2, [2, 4, 8])])
def test_latest_eps_variant_matches_oracle_and_batched_is_bitwise(S, m, cyc):
    """mode 2: the caches of all ranks are refreshed with the last applied eps at the end of a cycle."""
    print(f"sampler_run latest-eps S={S} m={m} cyc={cyc}", flush=True)
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    ref = oracle_run(cfg, W, x_T, ctx, S, m, cyc, mode="latest_eps")
    own = oracle_run(cfg, W, x_T, ctx, S, m, cyc)
    assert np.abs(ref["x0"] - own["x0"]).max() > 1e-6 * np.abs(own["x0"]).max()   # the variants really differ
    x0, sums, calls = gpu_run(d, dev(x_T), dev(ctx), S, m, cyc, mode=2)
    assert calls == S
    close_fp32(host(x0)[0], ref["x0"])
    s = host(sums)
    np.testing.assert_allclose(s[:, 0] / s[:, 1], ref["rx"], rtol=1e-4)
    np.testing.assert_allclose(s[1:, 2] / s[1:, 3], ref["re"][1:], rtol=1e-4, atol=1e-7)
    x0b, sb, cb = gpu_run(d, dev(x_T), dev(ctx), S, m, cyc, batched=True, mode=2)
    assert torch.equal(x0b, x0) and torch.equal(sb, sums)
    assert cb == m + len(O.expand_cycles(S, m, cyc))


def test_latest_eps_equals_mode_0_for_cycles_of_two_bitwise():
    cfg, W, d = setup("tiny", "unit")
    x_T = dev(I.make_latent(cfg, 1))
    x0a, sa, _ = gpu_run(d, x_T, None, 9, 1, [2] * 4, mode=0)
    x0b, sb, _ = gpu_run(d, x_T, None, 9, 1, [2] * 4, mode=2)
    assert torch.equal(x0a, x0b) and torch.equal(sa, sb)


def test_cycle_of_eight_batched_matches_oracle():
    """One predictor call over a batch of eight per cycle (the widest BatchStep setting of Section 4.3)."""
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    S, m, cyc = 19, 2, [8, 8, 8]                  # the last cycle is cut to one step
    ref = oracle_run(cfg, W, x_T, ctx, S, m, cyc)
    x0, sums, calls = gpu_run(d, dev(x_T), dev(ctx), S, m, cyc, batched=True)
    assert calls == 2 + 3
    close_fp32(host(x0)[0], ref["x0"])
    s = host(sums)
    np.testing.assert_allclose(s[:, 0] / s[:, 1], ref["rx"], rtol=1e-4)
    x0u, su, cu = gpu_run(d, dev(x_T), dev(ctx), S, m, cyc, batched=False)
    assert torch.equal(x0u, x0) and torch.equal(su, sums) and cu == S


def test_reduced_30_layer_reuse_run_bf16():
    """Six DDIM steps, window 2, 30 layers at width 1920 on 112 tokens, vs the oracle."""
    print("sampler_run reduced", flush=True)
    cfg, W, d = setup("reduced", "unit")
    x_T, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    ref = oracle_run(cfg, W, x_T, ctx, 6, 2, [2, 2])
    x0, sums, calls = gpu_run(d, dev(x_T), dev(ctx, torch.bfloat16), 6, 2, [2, 2])
    r = O.rel_mae(ref["x0"], host(x0)[0])[2]
    worst = worst_token(ref["x0"][None], host(x0), cfg.patch)
    print(f"  x0 rel-MAE {r:.3e}, worst token {worst:.3e}", flush=True)
    assert calls == 6 and r <= 2e-2
    assert worst <= WORST_TOKEN_BF16
    # reuse changes the result but stays finite and reproducible; window 1 is the no-reuse run
    x0p, _, _ = gpu_run(d, dev(x_T), dev(ctx, torch.bfloat16), 6, 2, [1, 1, 1, 1])
    dev_r = host(B.rel_mae(x0p, x0))[2]
    assert np.isfinite(dev_r) and dev_r > 0
    x0again, _, _ = gpu_run(d, dev(x_T), dev(ctx, torch.bfloat16), 6, 2, [2, 2])
    assert torch.equal(x0again, x0)


def test_step_batched_round_at_full_shape_equals_one_call_per_step_bitwise():
    """30 layers at 17776 tokens: one warm-up step and one cycle of four, as four calls and as one call of batch 4.

    Every sample of a batch is tiled, split and summed as if it were alone (the attention's key split of its last
    partial round and the projections' K split are planned per sample), so the batched round reproduces the
    per-step process bit for bit, as Section 3.3 requires of BatchStep.
    """
    print("sampler_run full shape, cycle of four, batched against unbatched", flush=True)
    cfg = I.CONFIGS["full"]
    _, W, d = setup("full", "std002")
    x_T = dev(I.make_latent(cfg, 1))
    ctx = dev(I.make_context(cfg, 1), torch.bfloat16)
    x0a, sa, ca = gpu_run(d, x_T, ctx, 5, 1, [4], batched=False)
    x0b, sb, cb = gpu_run(d, x_T, ctx, 5, 1, [4], batched=True)
    assert ca == 5 and cb == 2
    assert bool(torch.isfinite(x0a).all()) and bool(torch.isfinite(x0b).all())
    assert torch.equal(x0a, x0b)
    assert torch.equal(sa, sb)


def test_forward_batch_invariance_at_the_block_shape_bitwise():
    """One block at 4516 tokens (attention splits its last 28 work items, fc2 its last tiles along K), batch 3 with
    different timesteps against three single calls."""
    cfg, W, d = setup("block", "unit")
    x, ctx = dev(I.make_latent(cfg, 3)), dev(I.make_context(cfg, 3), torch.bfloat16)
    t = [900, 500, 20]
    full = B.dit_forward(d, x, ctx, t).clone()
    for b in range(3):
        one = B.dit_forward(d, x[b:b + 1].contiguous(), ctx[b:b + 1].contiguous(), t[b:b + 1])
        assert torch.equal(one[0], full[b]), b


def test_two_handles_with_different_kernel_paths_side_by_side():
    """The kernel path belongs to the handle: a handle on the generic kernels and one on the MFMA kernels, used
    in turn, each reproduce what they give alone; tile variants do not change a single bit."""
    cfg = I.CONFIGS["reduced"].with_(layers=2)
    weights = I.make_weights(cfg, 1000, "unit")
    wd = B.weights_to_device(cfg, weights)
    fast, slow, tiled = B.dit_create(cfg, wd), B.dit_create(cfg, wd), B.dit_create(cfg, wd)
    B.dit_set_kernel_path(slow, 1)
    B.dit_set_kernel_path(tiled, 0x300)
    x, ctx = dev(I.make_latent(cfg, 2)), dev(I.make_context(cfg, 2), torch.bfloat16)
    t = [300, 700]
    alone_fast = B.dit_forward(fast, x, ctx, t).clone()
    alone_slow = B.dit_forward(slow, x, ctx, t).clone()
    for _ in range(2):
        assert torch.equal(B.dit_forward(slow, x, ctx, t), alone_slow)
        assert torch.equal(B.dit_forward(fast, x, ctx, t), alone_fast)
        assert torch.equal(B.dit_forward(tiled, x, ctx, t), alone_fast)
    assert not torch.equal(alone_fast, alone_slow)                  # different kernels, different rounding
    assert O.rel_mae(host(alone_slow), host(alone_fast))[2] < 1e-2


def test_forward_captured_in_a_hip_graph_replays_bit_identically():
    """The forward only enqueues kernels on the caller's stream (no memsets, no synchronisation, workspace owned by
    the caller), so it can be captured in a HIP graph: 30 layers at width 1920 on 112 tokens (about 330 launches, a
    launch-bound shape).  Three replays, with eager work and synchronisations of the program in between, against
    the eager result."""
    cfg, W, d = setup("reduced", "unit")
    x = dev(I.make_latent(cfg, 2))
    ctx = dev(I.make_context(cfg, 2), torch.bfloat16)
    t = [500, 120]
    eps = torch.empty_like(x)
    eager = B.dit_forward(d, x, ctx, t).clone()         # also sizes and allocates the workspace
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.dit_forward(d, x, ctx, t, eps_out=eps)        # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        B.dit_forward(d, x, ctx, t, eps_out=eps)
    for rep in range(3):
        eps.fill_(float("nan"))
        other = B.dit_forward(d, x.flip(0).contiguous(), ctx.flip(0).contiguous(), t[::-1])   # eager work in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(eps, eager), rep
        assert torch.equal(other.flip(0), eager)         # (batch invariance once more)


# ----------------------------------------------------------------------- a run in pieces
@pytest.mark.parametrize("batched,mode,S,m,cyc,stops", [
    (False, 0, 10, 1, [1, 2, 4, 2], [1, 4, 6, 9]),
    (False, 2, 9, 2, [3, 4], [3, 4, 8]),
    (False, 1, 7, 1, [2, 2, 2], [2, 5]),
    (True, 0, 10, 1, [1, 2, 4, 2], [1, 2, 4, 8]),
])
def test_a_run_in_pieces_equals_the_whole_run_bitwise(batched, mode, S, m, cyc, stops):
    """sampler_run_steps stopped at `stops` and continued -- the last piece from a COPY of the state in a new
    workspace, as a restarted process would -- against sampler_run: final sample, per-step sums and trajectory."""
    print(f"sampler_run_steps batched={batched} mode={mode} S={S} stops={stops}", flush=True)
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = dev(I.make_latent(cfg, 1)), dev(I.make_context(cfg, 1))
    ts, a, b = B.ddim_coefficients(S)
    sched = B.Schedule(ts, a, b, m, cyc, batched=batched, mode=mode)
    x0, sums, calls, traj = B.sampler_run(d, sched, x_T, ctx, want_trajectory=True)
    torch.cuda.synchronize()
    ws = B.sampler_workspace(d, sched, DEV)
    state = B.SamplerState()
    sums2 = torch.zeros_like(sums)
    traj2 = torch.zeros_like(traj)
    out = torch.empty_like(x_T)
    for k in stops:
        B.sampler_run_steps(d, sched, state, k, x_T, ctx, ws, x_out=out, step_sums=sums2, trajectory=traj2)
        torch.cuda.synchronize()
        assert state.step == k and torch.equal(out, traj[k - 1])
    # "another process": the struct and the state bytes copied into a fresh, poisoned workspace
    nstate = B.sampler_state_bytes(d, sched)
    assert 0 < nstate < ws.numel()
    ws2 = torch.full_like(ws, 0xFF)
    ws2[:nstate] = ws[:nstate]
    state2 = B.SamplerState.from_buffer_copy(bytes(state))
    del ws
    B.sampler_run_steps(d, sched, state2, S, None, ctx, ws2, x_out=out, step_sums=sums2, trajectory=traj2)
    torch.cuda.synchronize()
    assert state2.step == S and state2.calls == calls
    assert torch.equal(out, x0) and torch.equal(sums2, sums) and torch.equal(traj2, traj)


def test_a_run_in_pieces_at_the_full_shape_is_bitwise_the_whole_run():
    """The benchmark times its steps one sampler_run_steps call per step: at its shape (30 layers, 17776 tokens, one
    warm-up step, cycles of two) a run taken step by step -- the last step from a copy of the state in another
    workspace -- gives the whole run's sample and per-step sums bit for bit."""
    print("sampler_run_steps full shape, step by step", flush=True)
    cfg = I.CONFIGS["full"]
    _, W, d = setup("full", "std002")
    x_T = dev(I.make_latent(cfg, 1))
    ctx = dev(I.make_context(cfg, 1), torch.bfloat16)
    S = 5
    ts, a, b = B.ddim_coefficients(S)
    sched = B.Schedule(ts, a, b, 1, [2, 2])
    x0, sums, calls = B.sampler_run(d, sched, x_T, ctx)
    torch.cuda.synchronize()
    ws = B.sampler_workspace(d, sched, DEV)
    state, sums2, out = B.SamplerState(), torch.zeros_like(sums), torch.empty_like(x_T)
    for k in range(1, S):
        B.sampler_run_steps(d, sched, state, k, x_T, ctx, ws, x_out=out, step_sums=sums2)
    torch.cuda.synchronize()
    nstate = B.sampler_state_bytes(d, sched)
    ws2 = torch.full_like(ws, 0xFF)
    ws2[:nstate] = ws[:nstate]
    del ws
    state2 = B.SamplerState.from_buffer_copy(bytes(state))
    B.sampler_run_steps(d, sched, state2, S, None, ctx, ws2, x_out=out, step_sums=sums2)
    torch.cuda.synchronize()
    assert state2.step == S and state2.calls == calls
    assert bool(torch.isfinite(x0).all())
    assert torch.equal(out, x0) and torch.equal(sums2, sums)


def test_run_in_pieces_rejects_states_and_stops_that_do_not_fit():
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = dev(I.make_latent(cfg, 1)), dev(I.make_context(cfg, 1))
    ts, a, b = B.ddim_coefficients(8)
    sched = B.Schedule(ts, a, b, 2, [3, 3])
    ws = B.sampler_workspace(d, sched, DEV)
    st = B.SamplerState()
    with pytest.raises(B.PsError) as e:
        B.sampler_run_steps(d, sched, st, 0, x_T, ctx, ws)           # nothing to do
    assert e.value.status == -5
    with pytest.raises(B.PsError) as e:
        B.sampler_run_steps(d, sched, st, 9, x_T, ctx, ws)           # past the end
    assert e.value.status == -5
    with pytest.raises(B.PsError) as e:
        B.sampler_run_steps(d, sched, st, 3, None, ctx, ws)          # a fresh run needs x_T
    assert e.value.status == -1
    B.sampler_run_steps(d, sched, st, 4, x_T, ctx, ws)
    assert (st.step, st.cycle, st.round) == (4, 0, 2)
    bad = B.SamplerState.from_buffer_copy(bytes(st)); bad.round = 1
    with pytest.raises(B.PsError) as e:
        B.sampler_run_steps(d, sched, bad, 8, None, ctx, ws)         # round does not belong to step 4
    assert e.value.status == -5
    with pytest.raises(B.PsError) as e:
        B.sampler_run_steps(d, sched, st, 3, None, ctx, ws)          # backwards
    assert e.value.status == -5
    batched = B.Schedule(ts, a, b, 2, [3, 3], batched=True)
    wsb = B.sampler_workspace(d, batched, DEV)
    with pytest.raises(B.PsError) as e:
        B.sampler_run_steps(d, batched, B.SamplerState(), 4, x_T, ctx, wsb)   # inside a cycle
    assert e.value.status == -5
    B.sampler_run_steps(d, batched, B.SamplerState(), 5, x_T, ctx, wsb)
    torch.cuda.synchronize()


# ------------------------------------------------- trajectories, deviation curves, other schedulers
@pytest.mark.parametrize("batched", [False, True])
def test_trajectory_output_matches_oracle_step_by_step(batched):
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    S, m, cyc = 9, 1, [2, 4, 2]
    ref = oracle_run(cfg, W, x_T, ctx, S, m, cyc)
    ts, a, b = B.ddim_coefficients(S)
    sched = B.Schedule(ts, a, b, m, cyc, batched=batched)
    x0, sums, calls, traj = B.sampler_run(d, sched, dev(x_T), dev(ctx), want_trajectory=True)
    torch.cuda.synchronize()
    assert traj.shape[0] == S and torch.equal(traj[-1], x0)
    for i in range(S):
        close_fp32(host(traj[i])[0], ref["xs"][i])


def test_deviation_curves_direct_reuse_vs_reuse_then_predict():
    """Per-step relative MAE against the original process (Section 3.1's comparison), for direct reuse with
    stride 2 and reuse-then-predict with degree 2; GPU curves against the oracle's.  With random weights the
    sizes are informational; the mechanism (same trajectories, same metric) is what is checked."""
    cfg, W, d = setup("tiny", "unit")
    x_T = I.make_latent(cfg, 1)
    S, m = 9, 1
    ts, a, b = B.ddim_coefficients(S)
    runs = {}
    for key, cyc, mode in [("orig", [1] * S, 0), ("direct", [2] * 4, 1), ("rtp", [2] * 4, 0)]:
        sched = B.Schedule(ts, a, b, m, cyc, mode=mode)
        runs[key] = B.sampler_run(d, sched, dev(x_T), None, want_trajectory=True)[3]
    torch.cuda.synchronize()
    refs = {"orig": oracle_run(cfg, W, x_T, None, S, m, [1] * S),
            "direct": oracle_run(cfg, W, x_T, None, S, m, [2] * 4, mode="direct_reuse"),
            "rtp": oracle_run(cfg, W, x_T, None, S, m, [2] * 4)}
    for key in ("direct", "rtp"):
        gpu_curve = np.array([host(B.rel_mae(runs["orig"][i], runs[key][i]))[2] for i in range(S)])
        ora_curve = np.array([O.rel_mae(refs["orig"]["xs"][i], refs[key]["xs"][i])[2] for i in range(S)])
        assert gpu_curve[0] == 0.0 == ora_curve[0]            # the warm-up step is shared
        np.testing.assert_allclose(gpu_curve[1:], ora_curve[1:], rtol=2e-2, atol=1e-6)
        assert gpu_curve[-1] > 0


@pytest.mark.parametrize("kind", ["euler_discrete", "flow_euler"])
def test_other_schedulers_run_matches_oracle(kind):
    """The same loop and fused update under the sigma-space Euler table and the flow-matching table."""
    cfg, W, d = setup("tiny_text", "unit")
    x_T, ctx = I.make_latent(cfg, 1), I.make_context(cfg, 1)
    S, m, cyc = 8, 2, [3, 3]
    if kind == "euler_discrete":
        ts, a, b = B.euler_discrete_coefficients(S)
        tau, ao, bo = O.euler_discrete_coefficients(steps=S)
    else:
        ts, a, b = B.flow_euler_coefficients(S)
        tau, ao, bo = O.flow_euler_coefficients(steps=S)
    f = lambda x, t: O.dit_forward(cfg, W, x[None], ctx, [t])[0]
    ref = O.run_sampler(f, x_T[0], tau, ao, bo, warmup=m, cycle_len=cyc)
    sched = B.Schedule(ts, a, b, m, cyc)
    x0, sums, calls = B.sampler_run(d, sched, dev(x_T), dev(ctx))
    torch.cuda.synchronize()
    assert calls == S
    close_fp32(host(x0)[0], ref["x0"])
    s = host(sums)
    np.testing.assert_allclose(s[:, 0] / s[:, 1], ref["rx"], rtol=1e-4)


def test_bench_prints_one_json_line_with_the_agreed_fields():
    """bench.py (one step, no CPU leg, the two cheap extra workloads) as a child process: one JSON line, the
    contract's keys, sane values."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    print("bench.py --steps 1 --warmup 1 --no-cpu-baseline --workloads block,fallback_attention", flush=True)
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "1", "--warmup", "1",
                        "--no-cpu-baseline", "--workloads", "block,fallback_attention"],
                       capture_output=True, text=True, timeout=170)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "step_ms", "gemm", "ln_modulate",
                "sampler_step_stress", "rel_mae_stress", "mfma_only_probe", "clocks", "workloads"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 1 and out["unit"] == "ms" and out["higher_is_better"] is False
    assert out["vs_baseline"] is None and out["dtype"] == "bf16" and out["data"] == "synthetic"
    assert "workload" in out["config"] and "model" not in out["config"]
    roof = out["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert roof["launches"] == 30 and 0.2 < roof["frac"] < 1.0
    assert 30.0 < out["value"] < 1000.0
    assert out["step_ms"]["n"] == 1 and abs(out["step_ms"]["mean"] - out["value"]) < 0.05 * out["value"]
    for key in ("sampler_step_stress", "rel_mae_stress", "ln_modulate"):
        assert out[key]["bound"] == "hbm" and 0.2 < out[key]["frac"] < 1.0, key
    assert 0.4 < out["mfma_only_probe"]["frac_of_nominal_peak"] <= 1.0
    assert set(out["workloads"]) == {"block", "fallback_attention"}
    assert 0.2 < out["workloads"]["fallback_attention"]["reference_tracking_kernel"]["frac_of_bf16_peak"] < 1.0
    assert out["workloads"]["block"]["attn3d_ms"]["n"] == 10
