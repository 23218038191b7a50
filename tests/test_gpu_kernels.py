"""GPU parity of the stand-alone entry points (sampler_step, rel_mae, attn3d, dit_linear)
against the CPU oracle, element by element, through the C ABI.

Tolerances: fp32 paths must agree with the float64 oracle to 1e-4 relative
(rel-MAE <= 1e-4 and max |err| <= 1e-4 * max |ref|); bf16 paths to 2e-2 rel-MAE against
the oracle run on the same bf16-rounded inputs.
"""
import math

import numpy as np
import pytest
import torch

from oracle import parastep_oracle as O
from paper_2505_14741_amd import binding as B
from paper_2505_14741_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(DEV)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_close_fp32(got, ref, tol=1e-4):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    scale = max(np.abs(ref).max(), 1e-30)
    assert np.abs(got - ref).max() <= tol * scale, (np.abs(got - ref).max(), scale)
    assert O.rel_mae(ref, got)[2] <= tol


def assert_close_bf16(got, ref, tol=2e-2, max_tol=None):
    r = O.rel_mae(ref, got)[2]
    assert r <= tol, r
    if max_tol is not None:
        assert np.abs(np.asarray(got) - np.asarray(ref)).max() <= max_tol * max(np.abs(ref).max(), 1e-30)
    return r


# ------------------------------------------------------------------- sampler_step / rel_mae
@pytest.mark.parametrize("n", [4, 5, 7, 1000, 4099, 2048 * 16 + 3, 1123200])
def test_sampler_step_matches_oracle(n):
    print(f"sampler_step n={n}", flush=True)
    rng = np.random.default_rng(n)
    x, e, p = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    a, b = np.float32(1.0372), np.float32(-0.2114)
    xo, sums = B.sampler_step(dev(x), dev(e), dev(p), a, b)
    torch.cuda.synchronize()
    ref = O.sampler_step(x, e, a, b)
    assert_close_fp32(host(xo), ref, 1e-6)
    want = [np.abs(ref - x).sum(), np.abs(ref).sum(), np.abs(e.astype(np.float64) - p).sum(), np.abs(e).sum()]
    np.testing.assert_allclose(host(sums), want, rtol=2e-5)
    # without eps_prev, and in place
    xd = dev(x)
    xo2, sums2 = B.sampler_step(xd, dev(e), None, a, b, x_out=xd)
    torch.cuda.synchronize()
    assert torch.equal(xo2, xo)
    got = host(sums2)
    np.testing.assert_allclose(got[[0, 1, 3]], np.array(want)[[0, 1, 3]], rtol=2e-5)
    assert got[2] == 0.0
    # no sums requested
    xo3, none = B.sampler_step(dev(x), dev(e), None, a, b, want_sums=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(xo3, xo)


def test_sampler_step_is_deterministic_and_exact_in_fp32():
    n = 1123200
    rng = np.random.default_rng(1)
    x, e, p = (dev(rng.standard_normal(n).astype(np.float32)) for _ in range(3))
    r1 = B.sampler_step(x, e, p, 0.99, 0.05)
    r2 = B.sampler_step(x, e, p, 0.99, 0.05)
    torch.cuda.synchronize()
    assert torch.equal(r1[0], r2[0]) and torch.equal(r1[1], r2[1])
    # element-wise result is the fp32 expression a*x + b*e up to one rounding of each product/sum
    ref = np.float32(0.99) * x.cpu().numpy() + np.float32(0.05) * e.cpu().numpy()
    assert np.abs(r1[0].cpu().numpy() - ref).max() <= 2.5e-7 * np.abs(ref).max()


def test_sampler_step_and_rel_mae_above_the_grid_cap():
    """More 16 KB chunks than the 32768 workgroups of the grid: workgroups walk several chunks, the last one is
    partial and 5 elements do not fill a vector.  Sampled outputs and all sums against the oracle."""
    n = 3 * (1 << 26) + 5
    print(f"sampler_step n={n}", flush=True)
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    x, e, p = (torch.randn(n, generator=g, device="cuda") for _ in range(3))
    a, b = np.float32(0.9931), np.float32(0.0517)
    xo, sums = B.sampler_step(x, e, p, a, b)
    torch.cuda.synchronize()
    xh, eh, ph = host(x), host(e), host(p)
    idx = np.unique(np.concatenate([[0, 1, 4095, 4096, n - 6, n - 5, n - 1],
                                    np.random.default_rng(3).integers(0, n, 4096)]))
    ref = O.sampler_step(xh[idx], eh[idx], a, b)
    assert_close_fp32(host(xo[torch.from_numpy(idx).to(DEV)]), ref, 1e-6)
    step = 1 << 24                                   # sums in pieces: fp64 copies of 2e8 values are large
    want = np.zeros(4)
    for i in range(0, n, step):
        xs, es, ps = (v[i:i + step].astype(np.float64) for v in (xh, eh, ph))
        r = O.sampler_step(xs, es, a, b)
        want += [np.abs(r - xs).sum(), np.abs(r).sum(), np.abs(es - ps).sum(), np.abs(es).sum()]
    np.testing.assert_allclose(host(sums), want, rtol=2e-5)
    out = host(B.rel_mae(x, e))
    num = sum(np.abs(xh[i:i + step].astype(np.float64) - eh[i:i + step]).sum() for i in range(0, n, step))
    den = sum(np.abs(xh[i:i + step].astype(np.float64)).sum() for i in range(0, n, step))
    np.testing.assert_allclose(out, [num, den, num / den], rtol=2e-5)


@pytest.mark.parametrize("n", [1, 4, 6, 1023, 65537, 1123200])
def test_rel_mae_matches_oracle(n):
    print(f"rel_mae n={n}", flush=True)
    rng = np.random.default_rng(n + 1)
    a, b = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
    out = host(B.rel_mae(dev(a), dev(b)))
    num, den, ratio = O.rel_mae(a, b)
    np.testing.assert_allclose(out, [num, den, ratio], rtol=2e-5)


def test_rel_mae_closed_forms_and_zero_denominator():
    a = dev(np.random.default_rng(0).standard_normal(5000).astype(np.float32))
    assert host(B.rel_mae(a, a))[2] == 0.0
    assert host(B.rel_mae(a, torch.zeros_like(a)))[2] == pytest.approx(1.0, rel=1e-6)
    assert host(B.rel_mae(a, -a))[2] == pytest.approx(2.0, rel=1e-6)
    assert host(B.rel_mae(a, 1.25 * a))[2] == pytest.approx(0.25, rel=1e-5)
    z = torch.zeros(64, device=DEV)
    assert math.isnan(host(B.rel_mae(z, z))[2])
    assert math.isinf(host(B.rel_mae(z, torch.ones_like(z)))[2])


def test_sampler_step_and_rel_mae_on_empty_inputs():
    """n = 0: nothing is read or written, the sums are zero, the ratio is the oracle's 0/0."""
    print("sampler_step / rel_mae n=0", flush=True)
    buf = torch.full((8,), 3.0, device=DEV)
    x, e, p = buf[:0], buf[4:4], buf[4:4]
    out = torch.full((8,), 7.0, device=DEV)
    _, sums = B.sampler_step(x, e, p, 0.9, 0.1, x_out=out[:0])
    torch.cuda.synchronize()
    assert host(sums).tolist() == [0.0, 0.0, 0.0, 0.0]
    assert bool((out == 7.0).all()) and bool((buf == 3.0).all())
    got = host(B.rel_mae(x, e))
    num, den, ratio = O.rel_mae(np.zeros(0), np.zeros(0))
    assert got[0] == num == 0.0 and got[1] == den == 0.0 and math.isnan(got[2]) and math.isnan(ratio)


# ---------------------------------------------------------------------------------- attn3d
@pytest.mark.parametrize("d", [16, 32, 64])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 127, 129, 300])
def test_attention_fp32_matches_oracle(N, d):
    print(f"attn3d fp32 N={N} d={d}", flush=True)
    q, k, v = I.make_qkv(2, N, 3, d, dtype="f32")
    scale = 1.0 / math.sqrt(d)
    o = B.attn3d(dev(q), dev(k), dev(v), scale)
    torch.cuda.synchronize()
    assert_close_fp32(host(o), O.attn3d(q, k, v, scale))


@pytest.mark.parametrize("N", [1, 31, 63, 64, 65, 127, 129, 255, 257, 1000])
def test_attention_bf16_mfma_matches_oracle(N):
    print(f"attn3d bf16 N={N}", flush=True)
    q, k, v = I.make_qkv(2, N, 3, 64, dtype="bf16")
    o = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125)
    torch.cuda.synchronize()
    ref = O.attn3d(q, k, v, 0.125)
    r = assert_close_bf16(host(o), ref, 2e-2, max_tol=3e-2)
    assert r < 8e-3      # bf16 rounding of P and of the output only


def test_attention_bf16_large_logits_and_poisoned_workspace():
    """Logit std ~ 4 (sharp softmax), NaN-filled scratch and output must not leak."""
    N = 333
    q, k, v = I.make_qkv(1, N, 2, 64, dtype="bf16", scale=2.0)
    qd, kd, vd = (dev(a, torch.bfloat16) for a in (q, k, v))
    out = torch.full_like(qd, float("nan"))
    junk = torch.full((1 << 22,), float("nan"), device=DEV)      # poison recently freed memory
    del junk
    o = B.attn3d(qd, kd, vd, 0.125, out=out)
    torch.cuda.synchronize()
    assert torch.isfinite(o).all()
    assert_close_bf16(host(o), O.attn3d(q, k, v, 0.125), 2e-2)


@pytest.mark.parametrize("case", ["huge_everywhere", "small_first_tile_then_huge", "all_far_below_zero",
                                  "moderate_above_window", "common_offset_plus_70", "common_offset_minus_30"])
def test_attention_bf16_reference_shifts(case):
    """The kernel without a softmax reference checks its own sums and hands heads it cannot do to the kernel that
    tracks a reference, which keeps that reference at 0 while it safely can; these inputs overflow 2^(c s)
    everywhere, only from a later tile on, or underflow it (all handed over, the reference moves on the first tile,
    on a later tile, downwards), or stay inside the range the first kernel accepts although every exponent is
    far from zero (+70, -30: no hand-over, sums of 2^80 and 2^-20)."""
    N = 700
    print(f"attn3d bf16 reference case {case}", flush=True)
    q, k, v = I.make_qkv(1, N, 2, 64, dtype="bf16")
    scale = 0.125
    if case == "huge_everywhere":
        scale = 8.0                                   # exponents ~ N(0, 92^2)
    elif case == "small_first_tile_then_huge":
        scale = 8.0
        k[:, :64] = I.round_to_bf16((k[:, :64] * 0.01).astype(np.float32))
    elif case == "all_far_below_zero":
        scale = 1.0
        q, k = q * 0.125, k * 0.125
        q[..., 0], k[..., 0] = 8.0, -8.0              # every score ~ -64: exponent ~ -92
        q, k = I.round_to_bf16(q.astype(np.float32)), I.round_to_bf16(k.astype(np.float32))
    elif case.startswith("common_offset"):
        scale = 1.0
        q, k = q * 0.125, k * 0.125
        a = 7.0 if case.endswith("plus_70") else 4.56     # s = +-a^2 + small: exponents ~ +70.7 / -30.0
        q[..., 0], k[..., 0] = a, (a if case.endswith("plus_70") else -a)
        q, k = I.round_to_bf16(q.astype(np.float32)), I.round_to_bf16(k.astype(np.float32))
    else:
        scale = 1.0                                   # exponents ~ N(0, 11.5^2): some rows peak above 32
    o = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), scale)
    torch.cuda.synchronize()
    assert torch.isfinite(o).all()
    assert_close_bf16(host(o), O.attn3d(q, k, v, scale), 2e-2, max_tol=3e-2)


@pytest.mark.parametrize("N", [64, 300, 1000])
def test_attention_bf16_reference_tracking_kernel_on_ordinary_inputs(N):
    """Kernel path 3 sends every head through the kernel that keeps a softmax reference (the fallback for
    unbounded scores); on ordinary inputs it must agree with the oracle like the default path does."""
    print(f"attn3d bf16 path 3 N={N}", flush=True)
    q, k, v = I.make_qkv(2, N, 3, 64, dtype="bf16")
    o = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125, kernel_path=3)
    torch.cuda.synchronize()
    assert_close_bf16(host(o), O.attn3d(q, k, v, 0.125), 2e-2, max_tol=3e-2)


@pytest.mark.parametrize("moved_heads", [(), (0, 13, 28, 29)])
def test_attention_bf16_reference_tracking_kernel_split_items_and_merge(moved_heads):
    """Kernel path 3 at a shape whose work items exceed the chip's workgroup slots (4516 tokens x 30 heads = 540
    items of 256 queries on 512 slots): the last 28 items -- head 28 from query 2048 on, all of head 29 -- are each
    computed as 8 key ranges that carry their own softmax reference, and merged with weights
    2^(c (r_i - max r)).  Once with ordinary inputs (all references 0) and once with q and k of some heads,
    split ones included, scaled so that the references move and differ between key ranges.  Sampled query rows
    of every head against the oracle, most of them inside the split items."""
    cfg = I.CONFIGS["block"]
    N, H = cfg.tokens, cfg.heads
    print(f"attn3d bf16 path 3 N={N} H={H} moved heads {moved_heads}", flush=True)
    q, k, v = I.make_qkv(1, N, H, 64, dtype="bf16")
    for h in moved_heads:
        q[:, :, h, :] *= 6.0
        k[:, :, h, :] *= 6.0                          # exponents ~ N(0, 52^2): far outside the +-32 window
    # keys of one key range much larger than the others: the ranges' references differ by construction
    if moved_heads:
        k[:, 3 * (N // 8):4 * (N // 8), 29, :] *= 2.0
    q, k = I.round_to_bf16(q.astype(np.float32)), I.round_to_bf16(k.astype(np.float32))
    o = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125, kernel_path=3)
    torch.cuda.synchronize()
    assert torch.isfinite(o).all()
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, 255, 2047, 2048, 2049, 2303, 2304, N - 257, N - 2, N - 1],
                                     rng.integers(2048, N, 30), rng.integers(0, 2048, 8)]))
    ref = O.attn3d(q[:, rows], k, v, 0.125)
    got = host(o[:, torch.from_numpy(rows).to(DEV)])
    for h in range(H):
        assert_close_bf16(got[:, :, h], ref[:, :, h], 2e-2, max_tol=4e-2)
    # the same call without the split (path 2 keeps the bounded kernel; both must agree with the oracle alike)
    o2 = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125, kernel_path=0)
    got2 = host(o2[:, torch.from_numpy(rows).to(DEV)])
    for h in range(H):
        assert_close_bf16(got2[:, :, h], ref[:, :, h], 2e-2, max_tol=4e-2)


def test_attention_bf16_batch_invariance_at_a_shape_that_splits():
    """4516 tokens x 30 heads splits its last 28 work items per sample; a sample's output must not depend on
    the batch it is computed in (bitwise), on the default path and on the reference-tracking path."""
    cfg = I.CONFIGS["block"]
    q, k, v = I.make_qkv(3, cfg.tokens, cfg.heads, 64, dtype="bf16")
    qd, kd, vd = (dev(a, torch.bfloat16) for a in (q, k, v))
    for path in (0, 3):
        print(f"attn3d bf16 batch of 3 against single calls, kernel path {path}", flush=True)
        full = B.attn3d(qd, kd, vd, 0.125, kernel_path=path)
        for b in range(3):
            one = B.attn3d(qd[b:b + 1].contiguous(), kd[b:b + 1].contiguous(), vd[b:b + 1].contiguous(), 0.125,
                           kernel_path=path)
            assert torch.equal(one[0], full[b]), (path, b)


def test_attention_bf16_marked_head_in_one_sample_of_a_batch():
    """A head whose scores overflow in sample 1 only: that (sample, head) alone is handed to the reference-tracking
    kernel, every sample still equals its single call bit for bit, and all agree with the oracle."""
    N, H = 700, 3
    q, k, v = I.make_qkv(3, N, H, 64, dtype="bf16")
    q[1, :, 2, :] *= 16.0
    k[1, :, 2, :] *= 16.0                            # exponents ~ N(0, 370^2) for sample 1, head 2
    q, k = I.round_to_bf16(q), I.round_to_bf16(k)
    qd, kd, vd = (dev(a, torch.bfloat16) for a in (q, k, v))
    full = B.attn3d(qd, kd, vd, 0.125)
    torch.cuda.synchronize()
    assert torch.isfinite(full).all()
    ref = O.attn3d(q, k, v, 0.125)
    for b in range(3):
        one = B.attn3d(qd[b:b + 1].contiguous(), kd[b:b + 1].contiguous(), vd[b:b + 1].contiguous(), 0.125)
        assert torch.equal(one[0], full[b]), b
        for h in range(H):
            assert_close_bf16(host(full)[b, :, h], ref[b, :, h], 2e-2, max_tol=3e-2)
    # the overflowing head really needs the other kernel: forced through it, the result is the same
    forced = B.attn3d(qd[1:2].contiguous(), kd[1:2].contiguous(), vd[1:2].contiguous(), 0.125, kernel_path=3)
    assert torch.equal(forced[0, :, 2], full[1, :, 2])


def test_attention_bf16_mixed_heads_take_different_kernels():
    """One head with huge scores (its key sums overflow without a softmax reference) next to ordinary heads: the
    first kernel marks that head, the reference-tracking kernel redoes it, and all agree with the oracle."""
    N = 700
    q, k, v = I.make_qkv(1, N, 3, 64, dtype="bf16")
    q[:, :, 1, :] *= 16.0
    k[:, :, 1, :] *= 16.0                             # head 1: exponents ~ N(0, 370^2) at scale 0.125
    q, k = I.round_to_bf16(q), I.round_to_bf16(k)
    o = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125)
    torch.cuda.synchronize()
    assert torch.isfinite(o).all()
    ref = O.attn3d(q, k, v, 0.125)
    for h in range(3):
        assert_close_bf16(host(o)[:, :, h], ref[:, :, h], 2e-2, max_tol=3e-2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_invariants(dtype):
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    N, H, d = 200, 2, 64
    q, k, v = I.make_qkv(1, N, H, d, dtype=dtype)
    # identical keys -> mean of V for every query
    k1 = k.copy(); k1[:] = k[:, :1]
    o = host(B.attn3d(dev(q, td), dev(k1, td), dev(v, td), 0.125))
    ref = np.broadcast_to(v.astype(np.float64).mean(axis=1, keepdims=True), o.shape)
    assert np.abs(o - ref).max() < (1e-5 if dtype == "f32" else 6e-3)
    # one dominant key -> its value
    k2 = np.zeros_like(k)
    qn = q[0, 5, 0] / np.linalg.norm(q[0, 5, 0])
    k2[0, 77, 0] = I.round_to_bf16((60.0 * qn).astype(np.float32)) if dtype == "bf16" else 60.0 * qn
    o2 = host(B.attn3d(dev(q, td), dev(k2, td), dev(v, td), 1.0))
    assert np.abs(o2[0, 5, 0] - v[0, 77, 0]).max() < (1e-5 if dtype == "f32" else 1e-2)
    # permuting keys together with values changes nothing but the summation order
    perm = np.random.default_rng(0).permutation(N)
    oa = host(B.attn3d(dev(q, td), dev(k, td), dev(v, td), 0.125))
    ob = host(B.attn3d(dev(q, td), dev(k[:, perm], td), dev(v[:, perm], td), 0.125))
    assert np.abs(oa - ob).max() < (1e-5 if dtype == "f32" else 8e-3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_rotary_position_offset_and_token_permutation(dtype):
    """Video tokens only, q and k rotated on the host with the 3D rotary angles (the oracle's routine): moving every
    token by the same (frame, row, column) offset leaves the attention output unchanged, and permuting the tokens
    together with their angles permutes the output -- here through the GPU attention (the tiny network's head
    width for fp32, the MFMA kernel's for bf16)."""
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    grid, H, d = (2, 8, 8), 4, (16 if dtype == "f32" else 64)
    N = grid[0] * grid[1] * grid[2]
    rng = np.random.default_rng(8)
    q, k, v = (rng.standard_normal((N, H, d)) for _ in range(3))
    prep = (lambda a: a.astype(np.float32)) if dtype == "f32" else (lambda a: I.round_to_bf16(a.astype(np.float32)))
    v = prep(v)

    def shifted(offset):
        big = tuple(g + o for g, o in zip(grid, offset))
        ang = O.rope3d_angles(big, d).reshape(big + (d // 2,))
        return ang[offset[0]:, offset[1]:, offset[2]:].reshape(N, d // 2)

    scale = 1.0 / math.sqrt(d)
    run = lambda qq, kk, vv: host(B.attn3d(dev(qq[None], td), dev(kk[None], td), dev(vv[None], td), scale))[0]
    a0 = shifted((0, 0, 0))
    q0, k0 = prep(O.rope3d_apply(q, a0)), prep(O.rope3d_apply(k, a0))
    base = run(q0, k0, v)
    ref = O.attn3d(q0[None], k0[None], v[None], scale)[0]
    tol = 1e-4 if dtype == "f32" else 2e-2
    assert O.rel_mae(ref, base)[2] <= tol
    a1 = shifted((3, 1, 2))
    q1, k1 = prep(O.rope3d_apply(q, a1)), prep(O.rope3d_apply(k, a1))
    assert np.abs(q1 - q0).max() > 0.1
    moved = run(q1, k1, v)
    assert O.rel_mae(base, moved)[2] <= (2e-6 if dtype == "f32" else 1.5e-2)   # bf16: q1, k1 are rounded again
    perm = rng.permutation(N)
    permuted = run(q0[perm], k0[perm], v[perm])
    assert O.rel_mae(base[perm], permuted)[2] <= (2e-6 if dtype == "f32" else 8e-3)


def test_attention_bf16_generic_and_mfma_paths_agree():
    q, k, v = I.make_qkv(1, 190, 2, 64, dtype="bf16")
    args = (dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125)
    fast = host(B.attn3d(*args))
    slow = host(B.attn3d(*args, kernel_path=1))
    ref = O.attn3d(q, k, v, 0.125)
    assert O.rel_mae(ref, slow)[2] < 4e-3 and O.rel_mae(ref, fast)[2] < 8e-3


def test_attention_block_shape_whole():
    """One block's attention at CogVideoX-2b width: 4516 tokens, 30 heads of 64, logit std ~1."""
    cfg = I.CONFIGS["block"]
    print("attn3d bf16 N=4516 H=30 whole", flush=True)
    q, k, v = I.make_qkv(1, cfg.tokens, cfg.heads, 64, dtype="bf16")
    o = host(B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125))
    ref = O.attn3d(q, k, v, 0.125)
    assert_close_bf16(o, ref, 2e-2)


@pytest.mark.parametrize("name,batch", [("full", 1), ("long", 1), ("full", 4)])
def test_attention_full_shape_sampled_rows(name, batch):
    """Launch configuration of the benchmark; the oracle evaluates 48 sampled query rows of
    every head (each output row needs only its query row and all keys/values)."""
    cfg = I.CONFIGS[name]
    N = cfg.tokens
    print(f"attn3d bf16 N={N} B={batch} sampled rows", flush=True)
    q, k, v = I.make_qkv(batch, N, cfg.heads, 64, dtype="bf16")
    o = B.attn3d(dev(q, torch.bfloat16), dev(k, torch.bfloat16), dev(v, torch.bfloat16), 0.125)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 63, 64, 255, 256, N - 257, N - 2, N - 1], rng.integers(0, N, 40)]))
    for b in sorted({0, batch - 1}):
        ref = O.attn3d(q[b:b + 1, rows], k[b:b + 1], v[b:b + 1], 0.125)
        got = host(o[b:b + 1, torch.from_numpy(rows).to(DEV)])
        assert_close_bf16(got, ref, 2e-2)
    assert torch.isfinite(o).all()


# ------------------------------------------------------------------------------ dit_linear
@pytest.mark.parametrize("M,Nn,K", [(777, 320, 256), (4516, 1920, 1920), (200, 64, 128)])
def test_linear_tile_variants_give_identical_results(M, Nn, K):
    """The tile variant decides which workgroup computes an output, never its value: every variant sums the k
    products of an output in the same order."""
    print(f"dit_linear tile variants M={M} N={Nn} K={K}", flush=True)
    rng = np.random.default_rng(M)
    a = dev(I.make_tokens(M, K, 5, "bf16"), torch.bfloat16)
    w = dev(I.round_to_bf16((rng.standard_normal((Nn, K)) / math.sqrt(K)).astype(np.float32)), torch.bfloat16)
    bias = dev(rng.standard_normal(Nn).astype(np.float32))
    for act in (0, 1):
        outs = [B.dit_linear(a, w, bias, act, kernel_path=v << 8) for v in (0, 1, 2, 3, 4)]
        torch.cuda.synchronize()
        for v in (1, 2, 3, 4):
            assert torch.equal(outs[v], outs[0]), (v, act)
    ref = host(a) @ host(w).T + host(bias)
    assert_close_bf16(host(B.dit_linear(a, w, bias, 0, kernel_path=0x300)), ref, 5e-3, max_tol=1e-2)


@pytest.mark.parametrize("M,Nn,K", [(1, 64, 64), (5, 66, 64), (130, 192, 128), (257, 130, 192), (300, 384, 64)])
@pytest.mark.parametrize("act", [0, 1])
def test_linear_small_shapes_both_dtypes(M, Nn, K, act):
    print(f"dit_linear M={M} N={Nn} K={K} act={act}", flush=True)
    rng = np.random.default_rng(M + Nn)
    for dtype, td in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        a = I.make_tokens(M, K, 3, dtype)
        w = (rng.standard_normal((Nn, K)) / math.sqrt(K)).astype(np.float32)
        w = I.round_to_bf16(w) if dtype == "bf16" else w
        bias = rng.standard_normal(Nn).astype(np.float32)
        out = host(B.dit_linear(dev(a, td), dev(w, td), dev(bias), act))
        ref = a.astype(np.float64) @ w.astype(np.float64).T + bias
        if act:
            ref = O.gelu_tanh(ref)
        if dtype == "f32":
            assert_close_fp32(out, ref)
        else:
            assert_close_bf16(out, ref, 5e-3, max_tol=1e-2)


@pytest.mark.parametrize("variant", [0, 3, 4])
@pytest.mark.parametrize("Nn,K,act", [(5760, 1920, 0), (1920, 1920, 0), (7680, 1920, 1), (1920, 7680, 0)])
def test_linear_full_shapes_sampled_rows(Nn, K, act, variant):
    """The four projections of a block at 17776 tokens; the oracle checks 64 sampled rows.  Variant 0 is the
    tile the library picks, 3 and 4 force the 192-row tiles (17776 = 92 * 192 + 112: a ragged last tile row)."""
    M = I.CONFIGS["full"].tokens
    print(f"dit_linear M={M} N={Nn} K={K} variant={variant}", flush=True)
    a = I.make_tokens(M, K, 21, "bf16")
    rng = np.random.default_rng(22)
    w = I.round_to_bf16((rng.standard_normal((Nn, K)) / math.sqrt(K)).astype(np.float32))
    bias = rng.standard_normal(Nn).astype(np.float32)
    out = B.dit_linear(dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), act, kernel_path=variant << 8)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 127, 128, 191, 192, 255, 256, M - 129, M - 113, M - 112, M - 1],
                                     rng.integers(0, M, 57)]))
    ref = a[rows].astype(np.float64) @ w.astype(np.float64).T + bias
    if act:
        ref = O.gelu_tanh(ref)
    assert_close_bf16(host(out[torch.from_numpy(rows).to(DEV)]), ref, 5e-3, max_tol=1e-2)
    assert torch.isfinite(out).all()
    # the long-K shape splits its last partial round of tiles along K when given scratch (the sampled rows M-129
    # and M-1 lie in those tiles); without scratch the same product is computed unsplit
    nb = B.lib().dit_linear_workspace_bytes(M, Nn, K, 1, variant << 8)
    if nb:
        out2 = B.dit_linear(dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), act, use_workspace=False,
                            kernel_path=variant << 8)
        torch.cuda.synchronize()
        assert_close_bf16(host(out2[torch.from_numpy(rows).to(DEV)]), ref, 5e-3, max_tol=1e-2)
        d = (out2.float() - out.float()).abs()
        assert float(d.max()) <= 2.0 ** -6 * float(out.float().abs().max())      # a bf16 rounding step at most
        assert float((d > 0).float().mean()) < 0.02                              # and only in the split tiles
