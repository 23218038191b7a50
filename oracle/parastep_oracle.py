"""CPU oracle for the reuse-then-predict denoising hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 NumPy statement of what the HIP library computes: the relative
MAE metric (paper Eq. 1), a deterministic DDIM scheduler standing in for the paper's
generic Scheduler(x_t, t, eps_t) (Preliminaries, "Denoising computation"), full
(unmasked) softmax attention over all text+video tokens, a DiT noise predictor with
adaLN-style modulation and 3D RoPE, and the round-based reuse-then-predict loop
(Appendix A, Algorithm 1) with every rank simulated, plus its single-device batched
form (Section 3.3, BatchStep) and the direct-reuse process (Section 3.1).

Nothing here is tiled, fused or reordered; matrix products use numpy.matmul as a
library step.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
import this module; the product path never does, and this module imports nothing
from the product's kernels or bindings.

Pin status (see tests/test_oracle_*.py):
  rel_mae, ddim_*, sampler_step : closed forms and brute force            -> pinned
  attn3d, layer_norm, gelu_tanh, silu, rope3d : library routines of a different
      package (torch CPU float64), complex-number rotation, invariants     -> pinned
  run_sampler (Algorithm 1 wiring) : hand trace, straight-line scalar script,
      constant / point-mass predictors, p = 1 == plain loop                -> pinned
  dit_forward : the paper fixes none of the network's internals; its wiring is pinned
      by invariants (zero gates, zero keys, permutation, batch independence) and by a
      second loop-level implementation, not by any printed value.  Its `query_rows`
      option is pinned against the whole evaluation.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- metric
def rel_mae(a, b):
    """Relative MAE of paper Eq. (1): sum|a_i - b_i| / sum|a_i| (the 1/n cancel).

    The denominator is the FIRST argument.  Returns (numerator, denominator, ratio);
    a zero denominator follows IEEE division (inf or nan), it is not an error.
    """
    a = np.asarray(a, dtype=F64).ravel()
    b = np.asarray(b, dtype=F64).ravel()
    num = float(np.sum(np.abs(a - b)))
    den = float(np.sum(np.abs(a)))
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = float(np.float64(num) / np.float64(den))
    return num, den, ratio


# ------------------------------------------------------------------------ scheduler
def ddim_alphas_cumprod(train_steps=1000, beta_start=1e-4, beta_end=2e-2):
    """abar_k = prod_{j<=k} (1 - beta_j) for a linear beta schedule (paper Section 2:
    abar_t is derived from the predefined schedule {beta_t})."""
    k = np.arange(train_steps, dtype=F64)
    beta = beta_start + k * (beta_end - beta_start) / (train_steps - 1)
    return np.cumprod(1.0 - beta)


def ddim_timesteps(train_steps: int, steps: int):
    """Descending integer grid tau_i = (S-1-i) * floor(train_steps / S)."""
    stride = train_steps // steps
    return np.array([(steps - 1 - i) * stride for i in range(steps)], dtype=np.int64)


def ddim_coefficients(train_steps=1000, beta_start=1e-4, beta_end=2e-2, steps=50):
    """Per-step (tau_i, a_i, b_i) of the deterministic (eta = 0) DDIM update
        x0_hat = (x - sqrt(1-abar_tau) eps) / sqrt(abar_tau)
        x'     = sqrt(abar_prev) x0_hat + sqrt(1-abar_prev) eps  =  a x + b eps,
    with abar_prev = abar at the next grid point, and 1 after the last step."""
    abar = ddim_alphas_cumprod(train_steps, beta_start, beta_end)
    tau = ddim_timesteps(train_steps, steps)
    a = np.empty(steps, dtype=F64)
    b = np.empty(steps, dtype=F64)
    for i in range(steps):
        ab_t = abar[tau[i]]
        ab_p = abar[tau[i + 1]] if i + 1 < steps else 1.0
        a[i] = math.sqrt(ab_p / ab_t)
        b[i] = math.sqrt(1.0 - ab_p) - a[i] * math.sqrt(1.0 - ab_t)
    return tau, a, b


def euler_discrete_coefficients(train_steps=1000, beta_start=1e-4, beta_end=2e-2, steps=50):
    """Deterministic Euler step in sigma space, the scheduler Section 4.2 names for SVD.  Samples are held
    as x = x0 + sigma*eps with sigma_t = sqrt((1-abar_t)/abar_t); along the DDIM grid, with sigma = 0
    after the last step:  x' = x + (sigma_next - sigma_t) * eps,  i.e. a = 1, b = sigma_next - sigma_t."""
    abar = ddim_alphas_cumprod(train_steps, beta_start, beta_end)
    tau = ddim_timesteps(train_steps, steps)
    sigma = np.sqrt((1.0 - abar) / abar)
    a = np.ones(steps, dtype=F64)
    b = np.empty(steps, dtype=F64)
    for i in range(steps):
        s_next = sigma[tau[i + 1]] if i + 1 < steps else 0.0
        b[i] = s_next - sigma[tau[i]]
    return tau, a, b


def flow_euler_coefficients(train_steps=1000, steps=50):
    """Flow Matching (Preliminaries): z_{t+dt} = z_t + dt * v(z_t, t), integrated from t = 0 (reference
    sample) to t = 1 on a uniform grid: dt = 1/steps, a = 1, b = dt.  The predictor is given the integer
    time index floor(t_i * train_steps) with t_i = i/steps."""
    tau = np.array([(i * train_steps) // steps for i in range(steps)], dtype=np.int64)
    return tau, np.ones(steps, dtype=F64), np.full(steps, 1.0 / steps, dtype=F64)


def sampler_step(x, eps, a, b):
    """x_{t-1} = Scheduler(x_t, t, eps_t) for DDIM: a*x + b*eps, element-wise."""
    return F64(a) * np.asarray(x, dtype=F64) + F64(b) * np.asarray(eps, dtype=F64)


# ------------------------------------------------------------------------ attention
def softmax_rows(s):
    """Row softmax with the max subtracted; asserts every row sums to 1."""
    s = np.asarray(s, dtype=F64)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    p = e / e.sum(axis=-1, keepdims=True)
    assert np.all(np.abs(p.sum(axis=-1) - 1.0) < 1e-12)
    return p


def attn3d(q, k, v, scale):
    """Full attention over the flattened (text, frame, row, col) token axis.

    q [B,Nq,H,d], k,v [B,N,H,d] -> o [B,Nq,H,d].  For every batch and head:
    S = scale * Q K^T (the whole Nq x N matrix), P = softmax over keys, O = P V.
    No mask, no dropout.  Nq may be a subset of query rows (each output row depends
    only on its own query row and on all keys and values).
    """
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    B, Nq, H, d = q.shape
    o = np.empty((B, Nq, H, d), dtype=F64)
    for b in range(B):
        for h in range(H):
            s = scale * (q[b, :, h, :] @ k[b, :, h, :].T)
            p = softmax_rows(s)
            o[b, :, h, :] = p @ v[b, :, h, :]
    return o


# ------------------------------------------------------------------- DiT components
def layer_norm(x, eps):
    """LayerNorm over the last axis, no affine, biased variance."""
    x = np.asarray(x, dtype=F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def gelu_tanh(x):
    x = np.asarray(x, dtype=F64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    x = np.asarray(x, dtype=F64)
    return x / (1.0 + np.exp(-x))


def timestep_sinusoid(t, width):
    """s(t) = [cos(t w_j) | sin(t w_j)], w_j = 10000^(-j/(width/2)), j < width/2."""
    half = width // 2
    w = np.power(10000.0, -np.arange(half, dtype=F64) / half)
    ang = F64(t) * w
    return np.concatenate([np.cos(ang), np.sin(ang)])


def rope_axis_widths(head_dim):
    """Head dim split over (frame, row, col) axes: d/4, 3d/8, 3d/8."""
    return (head_dim // 4, 3 * head_dim // 8, 3 * head_dim // 8)


def rope3d_angles(grid, head_dim, theta_base=10000.0):
    """Rotation angle of every (video token, pair): [N_v, d/2].

    Token order is (f, i, j) with j fastest.  Axis A of width d_A at integer position
    pos_A contributes pairs m < d_A/2 with angle pos_A * theta_base^(-2m/d_A).
    """
    F, Hp, Wp = grid
    widths = rope_axis_widths(head_dim)
    f, i, j = np.meshgrid(np.arange(F), np.arange(Hp), np.arange(Wp), indexing="ij")
    pos = [f.ravel().astype(F64), i.ravel().astype(F64), j.ravel().astype(F64)]
    cols = []
    for axis in range(3):
        dA = widths[axis]
        for m in range(dA // 2):
            cols.append(pos[axis] * theta_base ** (-2.0 * m / dA))
    return np.stack(cols, axis=1)


def rope3d_apply(u, angles):
    """Rotate interleaved pairs (u_{2m}, u_{2m+1}) of u [N_v, H, d] by angles [N_v, d/2]."""
    u = np.asarray(u, dtype=F64)
    c = np.cos(angles)[:, None, :]
    s = np.sin(angles)[:, None, :]
    ue, uo = u[..., 0::2], u[..., 1::2]
    out = np.empty_like(u)
    out[..., 0::2] = ue * c - uo * s
    out[..., 1::2] = ue * s + uo * c
    return out


def patchify(x, patch):
    """[C,F,H,W] -> [N_v, C*ps*ps]; token (f,i,j), vector order (c, dy, dx), c slowest."""
    C, F, H, W = x.shape
    Hp, Wp = H // patch, W // patch
    x = x.reshape(C, F, Hp, patch, Wp, patch)
    x = x.transpose(1, 2, 4, 0, 3, 5)          # f, i, j, c, dy, dx
    return x.reshape(F * Hp * Wp, C * patch * patch)


def unpatchify(tok, shape, patch):
    """Inverse of patchify: [N_v, C*ps*ps] -> [C,F,H,W]."""
    C, F, H, W = shape
    Hp, Wp = H // patch, W // patch
    t = tok.reshape(F, Hp, Wp, C, patch, patch).transpose(3, 0, 1, 4, 2, 5)
    return t.reshape(C, F, H, W)


MOD_CHUNKS = ("v.shift_a", "v.scale_a", "v.gate_a", "v.shift_m", "v.scale_m", "v.gate_m",
              "t.shift_a", "t.scale_a", "t.gate_a", "t.shift_m", "t.scale_m", "t.gate_m")


def _per_token(mod, D, Lt, N, name):
    """Broadcast the text / video variant of a modulation chunk over the token axis."""
    iv = MOD_CHUNKS.index("v." + name)
    it = MOD_CHUNKS.index("t." + name)
    out = np.empty((N, D), dtype=F64)
    out[:Lt] = mod[it * D:(it + 1) * D]
    out[Lt:] = mod[iv * D:(iv + 1) * D]
    return out


def dit_forward(cfg, W: Dict[str, np.ndarray], x, ctx, t, taps: Optional[list] = None,
                query_rows: Optional[Sequence[int]] = None):
    """Noise predictor eps_theta(x_t, t, c): a DiT with full 3D attention.

    x [B,C,F,H,W]; ctx [B,L_txt,D] or None; t [B] integer timesteps -> eps [B,C,F,H,W].
    Tokens: text first, then video patches.  Each block: adaLN-modulated LayerNorm,
    QKV projection, 3D RoPE on video q/k, full attention, gated residual; then
    modulated LayerNorm, GELU MLP, gated residual.  Text and video tokens use
    separate modulation chunks.  If `taps` is a list, the token matrix after the
    embedding and after every block is appended to it (per batch sample).

    `query_rows` (single-layer networks only) makes long sequences affordable: attention
    is evaluated for these token rows alone (all keys and values still take part) and
    NaN stands in for every other row of its output.  In a single layer a token's output
    depends on the other tokens through keys and values only, so the patches of the
    listed video tokens come out as in the whole evaluation and all others as NaN.
    """
    assert query_rows is None or cfg.layers == 1
    x = np.asarray(x, dtype=F64)
    B = x.shape[0]
    D, H, d, Lt = cfg.hidden, cfg.heads, cfg.head_dim, cfg.text_tokens
    Nv, N = cfg.video_tokens, cfg.tokens

    class _Widen(dict):
        # weights are widened to float64 where they are used, one tensor at a time
        def __getitem__(self, key):
            return np.asarray(W[key], dtype=F64)

    Wd = _Widen()
    angles = rope3d_angles(cfg.grid, d, cfg.rope_theta)
    out = np.empty_like(x)
    for b in range(B):
        # time conditioning
        s = timestep_sinusoid(int(t[b]), D)
        temb = Wd["W_t2"] @ silu(Wd["W_t1"] @ s + Wd["b_t1"]) + Wd["b_t2"]
        c = silu(temb)
        # tokens
        X = np.empty((N, D), dtype=F64)
        if Lt:
            X[:Lt] = np.asarray(ctx[b], dtype=F64)
        X[Lt:] = patchify(x[b], cfg.patch) @ Wd["W_pe"].T + Wd["b_pe"]
        if taps is not None:
            taps.append(X.copy())
        for l in range(cfg.layers):
            mod = Wd[f"W_mod.{l}"] @ c + Wd[f"b_mod.{l}"]
            ch = lambda name: _per_token(mod, D, Lt, N, name)
            h = layer_norm(X, cfg.ln_eps) * (1.0 + ch("scale_a")) + ch("shift_a")
            qkv = h @ Wd[f"W_qkv.{l}"].T + Wd[f"b_qkv.{l}"]
            q = qkv[:, 0 * D:1 * D].reshape(N, H, d).copy()
            k = qkv[:, 1 * D:2 * D].reshape(N, H, d).copy()
            v = qkv[:, 2 * D:3 * D].reshape(N, H, d)
            q[Lt:] = rope3d_apply(q[Lt:], angles)
            k[Lt:] = rope3d_apply(k[Lt:], angles)
            if query_rows is None:
                o = attn3d(q[None], k[None], v[None], 1.0 / math.sqrt(d))[0].reshape(N, D)
            else:
                rows = np.asarray(query_rows, dtype=np.int64)
                o = np.full((N, D), np.nan, dtype=F64)
                o[rows] = attn3d(q[None, rows], k[None], v[None], 1.0 / math.sqrt(d))[0].reshape(len(rows), D)
            X = X + ch("gate_a") * (o @ Wd[f"W_o.{l}"].T + Wd[f"b_o.{l}"])
            h2 = layer_norm(X, cfg.ln_eps) * (1.0 + ch("scale_m")) + ch("shift_m")
            u = gelu_tanh(h2 @ Wd[f"W_1.{l}"].T + Wd[f"b_1.{l}"])
            X = X + ch("gate_m") * (u @ Wd[f"W_2.{l}"].T + Wd[f"b_2.{l}"])
            if taps is not None:
                taps.append(X.copy())
        modf = Wd["W_fm"] @ c + Wd["b_fm"]
        y = layer_norm(X[Lt:], cfg.ln_eps) * (1.0 + modf[D:2 * D]) + modf[0:D]
        tok = y @ Wd["W_out"].T + Wd["b_out"]
        out[b] = unpatchify(tok, cfg.latent_shape, cfg.patch)
    return out


# -------------------------------------------------------------- reuse-then-predict
def expand_cycles(steps: int, warmup: int, cycle_len: Sequence[int]) -> List[int]:
    """Cycle lengths covering the steps after warm-up; the last one may be cut short
    by the end of the run (the loop of Algorithm 1 simply stops)."""
    out, left = [], steps - warmup
    for p in cycle_len:
        if left <= 0:
            break
        out.append(int(p))
        left -= int(p)
    if left > 0:
        raise ValueError("cycle lengths do not cover the steps after warm-up")
    return out


def run_sampler(predict: Callable, x_T, tau, a, b, warmup: int, cycle_len: Sequence[int],
                mode: str = "reuse_then_predict", trace: Optional[list] = None,
                reuse_trace: Optional[list] = None, state: Optional[dict] = None,
                stop: Optional[int] = None):
    """Denoising loop of Algorithm 1 with every rank simulated on one host.

    predict(x, tau) -> eps is the noise predictor for one sample.  Every rank r keeps
    its own sample x[r] and its own eps_cache[r].  Warm-up steps run the original
    process on all ranks.  Afterwards, in round `rnd` of a cycle of length p, the rank
    with r == rnd evaluates the predictor on ITS sample and caches the result; rank 0
    applies that result (it receives it), every other rank applies its own cache; all
    ranks take the scheduler step; after the last round rank 0's sample is copied to
    all ranks.  A rank's cache is written only when that rank evaluates the predictor.

    mode="direct_reuse" is the direct reuse process: the predictor is evaluated only
    in round 0 of a cycle and the same eps is applied in the remaining rounds.

    mode="latest_eps" is a variant of Algorithm 1 in which, whenever rank 0's sample is
    copied to all ranks at the end of a cycle, the eps rank 0 applied in that last step
    is copied to every rank's cache as well (Algorithm 1 itself never sends eps to a
    non-root rank), so the reuse updates of the next cycle use an eps that is 1..r
    steps old instead of the rank's own older prediction.  With cycles of length 2 the
    two coincide.

    Returns dict(x0, xs=[x after each step on rank 0], eps=[eps applied by rank 0],
    rx=[rel_mae(x_{i+1}, x_i)], re=[rel_mae(eps_i, eps_{i-1}), nan for i=0], calls).
    `trace`, if a list, receives (step, evaluating rank or -1, rank whose eps rank 0
    applies) tuples; `reuse_trace`, if a list, receives (step, rank, step at which the
    eps that rank reuses was predicted) for every reuse update of a non-root rank.

    A run in pieces: `stop` ends the loop after step stop-1, and the returned dict's
    "state" holds what Algorithm 1 carries from one step to the next -- the step count,
    cycle and round, every rank's sample and eps_cache, and the last applied eps (for the
    adjacent-step relative MAE); passing it back as `state` continues from there.  The
    lists then cover the steps of that piece only.
    """
    S = len(tau)
    if mode not in ("reuse_then_predict", "direct_reuse", "latest_eps"):
        raise ValueError(mode)
    cycles = expand_cycles(S, warmup, cycle_len) if warmup < S else []
    if warmup < 1 and any(p > 1 for p in cycles):
        raise ValueError("eps_cache is undefined without a warm-up step")
    pmax = max(cycles) if cycles else 1
    x = [np.asarray(x_T, dtype=F64).copy() for _ in range(pmax)]
    cache = [None] * pmax
    born = [None] * pmax                 # step at which cache[r] was predicted
    xs, eps_used, rx, re = [], [], [], []
    calls = 0
    cyc, rnd = 0, 0
    first, eps_last = 0, None
    if state is not None:
        first, cyc, rnd, calls = state["step"], state["cycle"], state["round"], state["calls"]
        x = [v.copy() for v in state["x"]]
        cache = [None if v is None else v.copy() for v in state["cache"]]
        born = list(state["born"])
        eps_last = state["eps_last"]
    last = S if stop is None else stop
    for i in range(first, last):
        x_before = x[0]
        if i < warmup:
            e = predict(x[0], int(tau[i]))
            calls += 1
            for r in range(pmax):
                cache[r] = e
                born[r] = i
                x[r] = sampler_step(x[r], e, a[i], b[i])
            applied = e
            if trace is not None:
                trace.append((i, 0, 0))
        else:
            p = cycles[cyc]
            if mode != "direct_reuse":
                master = rnd
                e_m = predict(x[master], int(tau[i]))
                calls += 1
                cache[master] = e_m
                born[master] = i
                applied = e_m
                for r in range(p):
                    e_r = e_m if (r == master or r == 0) else cache[r]
                    if reuse_trace is not None and r > master:
                        reuse_trace.append((i, r, born[r]))
                    x[r] = sampler_step(x[r], e_r, a[i], b[i])
                if trace is not None:
                    trace.append((i, master, master))
            else:
                if rnd == 0:
                    cache[0] = predict(x[0], int(tau[i]))
                    calls += 1
                applied = cache[0]
                x[0] = sampler_step(x[0], applied, a[i], b[i])
                if trace is not None:
                    trace.append((i, 0 if rnd == 0 else -1, 0))
            if rnd == p - 1:
                for r in range(1, pmax):
                    x[r] = x[0].copy()
                    if mode == "latest_eps":
                        cache[r] = applied
                        born[r] = i
                cyc += 1
                rnd = 0
            else:
                rnd += 1
        xs.append(x[0].copy())
        rx.append(rel_mae(x[0], x_before)[2])
        re.append(rel_mae(applied, eps_last)[2] if eps_last is not None else float("nan"))
        eps_last = np.asarray(applied, dtype=F64).copy()
        eps_used.append(eps_last)
    out_state = dict(step=last, cycle=cyc, round=rnd, calls=calls, x=[v.copy() for v in x],
                     cache=[None if v is None else np.asarray(v, dtype=F64).copy() for v in cache],
                     born=list(born), eps_last=eps_last)
    return dict(x0=x[0], xs=xs, eps=eps_used, rx=rx, re=re, calls=calls, state=out_state)


def run_sampler_batched(predict_batch: Callable, x_T, tau, a, b, warmup: int,
                        cycle_len: Sequence[int], mode: str = "reuse_then_predict"):
    """Single-device batched form (BatchStep): at the start of a cycle of length p the
    inputs of all p predictor evaluations are known -- rank r's input is the current
    sample advanced r times with that rank's cached eps -- so they are evaluated as one
    batch with per-sample timesteps, after which the p scheduler steps are taken on the
    true trajectory in order.

    predict_batch(xb [B,...], taus [B]) -> eps [B,...].  Returns the same dict as
    run_sampler; its results must equal run_sampler's for the same schedule and mode
    ("reuse_then_predict" or "latest_eps").
    """
    S = len(tau)
    if mode not in ("reuse_then_predict", "latest_eps"):
        raise ValueError(mode)
    cycles = expand_cycles(S, warmup, cycle_len) if warmup < S else []
    if warmup < 1 and any(p > 1 for p in cycles):
        raise ValueError("eps_cache is undefined without a warm-up step")
    pmax = max(cycles) if cycles else 1
    x0 = np.asarray(x_T, dtype=F64).copy()
    cache = [None] * pmax
    xs, eps_used, rx, re = [], [], [], []
    calls = 0

    def record(x_new, x_old, e):
        xs.append(x_new.copy())
        rx.append(rel_mae(x_new, x_old)[2])
        re.append(rel_mae(e, eps_used[-1])[2] if eps_used else float("nan"))
        eps_used.append(np.asarray(e, dtype=F64).copy())

    i = 0
    while i < min(warmup, S):
        e = predict_batch(x0[None], np.array([tau[i]]))[0]
        calls += 1
        for r in range(pmax):
            cache[r] = e
        x_new = sampler_step(x0, e, a[i], b[i])
        record(x_new, x0, e)
        x0 = x_new
        i += 1
    for p in cycles:
        n = min(p, S - i)                       # last cycle may be cut short
        inputs = []
        for r in range(n):
            xr = x0
            for jj in range(r):
                xr = sampler_step(xr, cache[r], a[i + jj], b[i + jj])
            inputs.append(xr)
        eb = predict_batch(np.stack(inputs), np.asarray(tau[i:i + n]))
        calls += 1
        for r in range(n):
            cache[r] = eb[r]
            x_new = sampler_step(x0, eb[r], a[i + r], b[i + r])
            record(x_new, x0, eb[r])
            x0 = x_new
        if mode == "latest_eps":
            for r in range(pmax):
                cache[r] = eb[n - 1]
        i += n
    return dict(x0=x0, xs=xs, eps=eps_used, rx=rx, re=re, calls=calls)


def critical_path_calls(steps: int, warmup: int, p: int) -> int:
    """Predictor evaluations on one device's critical path: every warm-up step plus one
    per cycle (Section 3.1: each device runs one forward per cycle)."""
    m = min(warmup, steps)
    return m + -(-(steps - m) // p)


def amdahl_bound(warmup_ratio: float, p: int) -> float:
    """Speedup bound 1 / (m + (1-m)/p) of Section 4.4 ("Impact of warm-up steps")."""
    return 1.0 / (warmup_ratio + (1.0 - warmup_ratio) / p)
