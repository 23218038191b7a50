"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, its
host-only DDIM table matches the oracle, and every error path answers before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import parastep_oracle as O
from paper_2505_14741_amd import binding as B
from paper_2505_14741_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "parastep.h")).read()
    return re.findall(r"^PS_API\s+[\w\s\*]+?\b(\w+)\(", text, flags=re.M)


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(B.EXPORTED)


def test_strerror_is_total():
    L = B.lib()
    seen = {L.ps_strerror(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and L.ps_strerror(-99) == b"unknown status"


@pytest.mark.parametrize("S", [5, 8, 50])
def test_ddim_table_matches_oracle(S):
    ts, a, b = B.ddim_coefficients(S)
    tau, ao, bo = O.ddim_coefficients(steps=S)
    np.testing.assert_array_equal(ts, tau)
    np.testing.assert_allclose(a, ao, rtol=1e-14)
    np.testing.assert_allclose(b, bo, rtol=1e-12)


@pytest.mark.parametrize("S", [5, 8, 50])
def test_euler_and_flow_tables_match_oracle(S):
    ts, a, b = B.euler_discrete_coefficients(S)
    tau, ao, bo = O.euler_discrete_coefficients(steps=S)
    np.testing.assert_array_equal(ts, tau)
    np.testing.assert_array_equal(a, ao)
    np.testing.assert_allclose(b, bo, rtol=1e-12)
    ts, a, b = B.flow_euler_coefficients(S)
    tau, ao, bo = O.flow_euler_coefficients(steps=S)
    np.testing.assert_array_equal(ts, tau)
    np.testing.assert_array_equal(a, ao)
    np.testing.assert_array_equal(b, bo)
    L = B.lib()
    t4 = (C.c_int32 * 4)(); a4 = (C.c_double * 4)(); b4 = (C.c_double * 4)()
    assert L.euler_discrete_coefficients(1000, 1e-4, 2e-2, 4, t4, None, b4) == -1
    assert L.euler_discrete_coefficients(1000, 1e-4, 2e-2, 0, t4, a4, b4) == -5
    assert L.flow_euler_coefficients(1000, 4, None, a4, b4) == -1
    assert L.flow_euler_coefficients(3, 4, t4, a4, b4) == -5


def test_ddim_table_rejects_bad_arguments():
    L = B.lib()
    ts = (C.c_int32 * 4)(); a = (C.c_double * 4)(); b = (C.c_double * 4)()
    assert L.ddim_coefficients(1000, 1e-4, 2e-2, 4, None, a, b) == -1
    assert L.ddim_coefficients(1000, 1e-4, 2e-2, 0, ts, a, b) == -5
    assert L.ddim_coefficients(3, 1e-4, 2e-2, 4, ts, a, b) == -5
    assert L.ddim_coefficients(1000, 2e-2, 1e-4, 4, ts, a, b) == -5


def _cfg_struct(cfg, **over):
    vals = dict(layers=cfg.layers, hidden=cfg.hidden, heads=cfg.heads, head_dim=cfg.head_dim,
                mlp_ratio=cfg.mlp_ratio, in_channels=cfg.in_channels, patch=cfg.patch, frames=cfg.frames,
                height=cfg.height, width=cfg.width, text_tokens=cfg.text_tokens,
                time_embed_dim=cfg.time_embed_dim, dtype=0, ln_eps=cfg.ln_eps, rope_theta=cfg.rope_theta)
    vals.update(over)
    return B._DitConfig(**vals)


def _fake_weights(n):
    # never dereferenced: creation only records the addresses
    return (C.c_void_p * n)(*[0x1000 * (i + 1) for i in range(n)])


def _create(cfg_struct, nw=None, weights=None):
    L = B.lib()
    n = L.dit_num_weights(cfg_struct.layers) if nw is None else nw
    h = C.c_void_p()
    w = _fake_weights(max(n, 1)) if weights is None else weights
    rc = L.dit_create(C.byref(cfg_struct), w, n, C.byref(h))
    return rc, h


def test_dit_create_validation():
    L = B.lib()
    cfg = I.CONFIGS["tiny"]
    assert L.dit_num_weights(2) == 30 and L.dit_num_weights(30) == 310
    rc, h = _create(_cfg_struct(cfg))
    assert rc == 0 and h.value
    assert L.dit_workspace_bytes(h, 1) > 0 and L.dit_workspace_bytes(h, 0) == 0 and L.dit_workspace_bytes(h, 17) == 0
    assert L.dit_workspace_bytes(h, 4) > 3 * L.dit_workspace_bytes(h, 1) // 2
    assert L.dit_destroy(h) == 0
    assert L.dit_destroy(None) == -1
    assert _create(_cfg_struct(cfg, dtype=7))[0] == -3
    assert _create(_cfg_struct(cfg, hidden=60))[0] == -2            # != heads*head_dim
    assert _create(_cfg_struct(cfg, head_dim=24, hidden=96))[0] == -2
    assert _create(_cfg_struct(cfg, height=15))[0] == -2            # not divisible by patch
    assert _create(_cfg_struct(cfg, layers=0))[0] == -2
    assert _create(_cfg_struct(cfg, text_tokens=-1))[0] == -2
    assert _create(_cfg_struct(cfg), nw=29)[0] == -2                # wrong weight count
    w = _fake_weights(30); w[7] = None
    assert _create(_cfg_struct(cfg), weights=w)[0] == -1            # NULL weight
    w = _fake_weights(30); w[3] = 0x1004
    assert _create(_cfg_struct(cfg), weights=w)[0] == -2            # misaligned weight
    assert L.dit_create(None, _fake_weights(30), 30, C.byref(C.c_void_p())) == -1


def test_kernel_path_is_a_property_of_the_handle():
    """Two handles hold different kernel paths side by side; nothing process-wide is involved."""
    L = B.lib()
    cfg = I.CONFIGS["tiny"]
    (rc1, h1), (rc2, h2) = _create(_cfg_struct(cfg)), _create(_cfg_struct(cfg))
    assert rc1 == 0 and rc2 == 0
    assert L.dit_get_kernel_path(h1) == 0 and L.dit_get_kernel_path(h2) == 0
    assert L.dit_set_kernel_path(h1, 1) == 0 and L.dit_set_kernel_path(h2, 0x203) == 0
    assert L.dit_get_kernel_path(h1) == 1 and L.dit_get_kernel_path(h2) == 0x203
    ws = L.dit_workspace_bytes(h2, 2)
    for bad in (-1, 5, 0x500, 0x1000, 1 << 20):
        assert L.dit_set_kernel_path(h2, bad) == -2
    assert L.dit_get_kernel_path(h2) == 0x203 and L.dit_workspace_bytes(h2, 2) == ws
    assert L.dit_set_kernel_path(h2, 0) == 0 and L.dit_workspace_bytes(h2, 2) == ws   # size independent of the path
    assert L.dit_set_kernel_path(None, 0) == -1 and L.dit_get_kernel_path(None) == -1
    assert not hasattr(L, "ps_set_kernel_path")
    L.dit_destroy(h1); L.dit_destroy(h2)


def test_dit_create_rejects_shapes_no_kernel_serves():
    cfg = I.CONFIGS["tiny"]
    assert _create(_cfg_struct(cfg, in_channels=300))[0] == -2                    # 1200 patch values: LDS staging
    assert _create(_cfg_struct(cfg, in_channels=256))[0] == 0
    # bf16: a sample's widest activation must stay below 2^31 elements (32-bit offsets in the MFMA projections)
    big = dict(hidden=2048, heads=32, head_dim=64, mlp_ratio=8, frames=33, height=128, width=128, patch=2)
    assert _create(_cfg_struct(cfg, dtype=1, **big))[0] == -2
    assert _create(_cfg_struct(cfg, dtype=0, **big))[0] == 0


def test_dit_forward_validation_has_no_side_effects():
    L = B.lib()
    cfg = I.CONFIGS["tiny_text"]
    rc, h = _create(_cfg_struct(cfg))
    assert rc == 0
    need = L.dit_workspace_bytes(h, 1)
    t = (C.c_int32 * 1)(500)
    X, E, CTX, WS = 0x10000, 0x20000, 0x30000, 0x40000
    f = lambda **k: L.dit_forward(k.get("h", h), k.get("x", X), k.get("ctx", CTX), k.get("t", t), k.get("e", E),
                                  k.get("batch", 1), k.get("ws", WS), k.get("wsb", need), None)
    assert f(x=None) == -1 and f(e=None) == -1 and f(t=None) == -1 and f(h=None) == -1
    assert f(ctx=None) == -1                                        # text tokens need a context
    assert f(batch=0) == -2 and f(batch=17) == -2
    assert f(e=X) == -2                                             # aliasing
    assert f(x=X + 4) == -2                                         # misaligned
    assert f(t=(C.c_int32 * 1)(-3)) == -2
    assert f(ws=None) == -4 and f(wsb=need - 1) == -4 and f(ws=WS + 16) == -4
    L.dit_destroy(h)


def test_attn3d_validation():
    L = B.lib()
    Q, K, V, Oo, WS = 0x1000, 0x2000, 0x3000, 0x4000, 0x10000
    f = lambda **k: L.attn3d(k.get("q", Q), K, V, k.get("o", Oo), k.get("b", 1), k.get("n", 10), 2, k.get("d", 16),
                             k.get("scale", 0.25), k.get("dt", 0), k.get("path", 0), k.get("ws", None), k.get("wsb", 0),
                             None)
    assert f(q=None) == -1 and f(o=None) == -1
    assert f(path=5) == -2 and f(path=-1) == -2 and f(path=0x500) == -2 and f(path=0x1000) == -2
    assert f(dt=5) == -3
    assert f(n=0) == -2 and f(b=0) == -2 and f(d=48) == -2 and f(d=128) == -2
    assert f(scale=0.0) == -2 and f(scale=float("nan")) == -2 and f(scale=-1.0) == -2
    assert f(o=Q) == -2 and f(q=Q + 2) == -2
    # the bf16 head-dim-64 kernels keep one flag per (batch, head) in the workspace (one 256-byte
    # block here); a short sequence has no key-split pieces.  The other kernels need no scratch.
    assert L.attn3d_workspace_bytes(1, 100, 2, 64, 1) == 256
    assert f(dt=1, d=64, ws=None, wsb=0) == -4
    assert L.attn3d_workspace_bytes(1, 100, 2, 16, 0) == 0
    assert L.attn3d_workspace_bytes(0, 100, 2, 16, 0) == 0


def test_dit_linear_validation_and_workspace_size():
    L = B.lib()
    A, W, BI, OUT, WS = 0x1000, 0x2000, 0x3000, 0x4000, 0x10000
    f = lambda **k: L.dit_linear(k.get("a", A), W, k.get("bias", BI), k.get("out", OUT), k.get("m", 8), k.get("n", 64),
                                 k.get("k", 64), k.get("act", 0), k.get("dt", 1), k.get("path", 0), k.get("ws", None),
                                 k.get("wsb", 0), None)
    assert f(a=None) == -1 and f(bias=None) == -1 and f(out=None) == -1
    assert f(path=7) == -2 and f(path=0x900) == -2
    assert f(dt=7) == -3
    assert f(m=0) == -2 and f(n=63) == -2 and f(k=60) == -2 and f(act=2) == -2
    assert f(out=A) == -2 and f(a=A + 2) == -2 and f(bias=BI + 4) == -2
    assert f(ws=WS + 16, wsb=1 << 20) == -4
    assert f(m=1 << 20, n=4096) == -2                                  # 2^32 bf16 outputs: beyond the MFMA kernel's offsets
    # scratch is only asked for where the K-split of the last partial round of tiles pays: 17776 x 1920 x 7680
    # leaves 37 of 2085 tiles of 128 x 128 for a 5th round on 512 workgroup slots; they are split 8 ways
    assert L.dit_linear_workspace_bytes(17776, 1920, 7680, 1, 0x200) == 37 * 8 * 128 * 128 * 4
    assert L.dit_linear_workspace_bytes(17776, 1920, 7680, 1, 0x204) == 0   # mode 4: no K-split
    assert L.dit_linear_workspace_bytes(17776, 1920, 1920, 1, 0x200) == 0   # short K
    assert L.dit_linear_workspace_bytes(17776, 7680, 1920, 1, 0x100) == 0   # 256 x 256 tiles
    assert L.dit_linear_workspace_bytes(17776, 1920, 7680, 0, 0) == 0       # fp32 runs on the generic kernel
    assert L.dit_linear_workspace_bytes(100, 64, 64, 1, 0) == 0
    assert L.dit_linear_workspace_bytes(100, 64, 64, 1, 0x700) == 0         # unknown tile variant


def test_sampler_step_and_rel_mae_validation():
    L = B.lib()
    X, E, P, WS = 0x1000, 0x2000, 0x3000, 0x10000
    need = L.sampler_step_workspace_bytes(1000)
    assert need > 0 and need % 256 == 0
    f = lambda **k: L.sampler_step(k.get("x", X), k.get("e", E), k.get("p", P), k.get("xo", X), 1.0, 0.5, 1000,
                                   k.get("s", 0x5000), k.get("ws", WS), k.get("wsb", need), None)
    assert f(x=None) == -1 and f(e=None) == -1 and f(xo=None) == -1
    assert f(xo=E) == -2 and f(xo=P) == -2 and f(x=X + 8) == -2
    assert f(ws=None) == -4 and f(wsb=need - 1) == -4 and f(ws=WS + 64) == -4
    # the entry point without a workspace: same checks, and a size limit (the scratch array is fixed)
    h = lambda **k: L.sampler_step_noalloc(k.get("x", X), k.get("e", E), k.get("p", P), k.get("xo", X), 1.0, 0.5,
                                           k.get("n", 1000), None, None)
    assert h(x=None) == -1 and h(e=None) == -1 and h(xo=None) == -1
    assert h(xo=E) == -2 and h(xo=P) == -2 and h(x=X + 8) == -2
    assert h(n=(1 << 31) + 1) == -2
    g = lambda **k: L.rel_mae(k.get("a", X), k.get("b", E), 1000, k.get("o", 0x5000), k.get("ws", WS),
                              k.get("wsb", need), None)
    assert g(a=None) == -1 and g(o=None) == -1 and g(ws=None) == -4 and g(a=X + 4) == -2


def _sched(steps=8, warmup=2, cyc=(2, 2, 2), batched=0, mode=0, ts=None):
    tau, a, b = O.ddim_coefficients(steps=steps)
    return B.Schedule(tau if ts is None else ts, a, b, warmup, list(cyc), batched=batched, mode=mode)


def test_schedule_validation():
    L = B.lib()
    cfg = I.CONFIGS["tiny"]
    rc, h = _create(_cfg_struct(cfg))
    ok = _sched()
    # event timing modes: off, every class, attention only
    assert [L.dit_profile_enable(h, m) for m in (1, 2, 0, 3, -1)] == [0, 0, 0, -2, -2]
    assert L.dit_profile_enable(None, 1) == -1
    assert L.sampler_workspace_bytes(h, C.byref(ok.c)) > 0
    assert L.sampler_workspace_bytes(h, C.byref(_sched(batched=1).c)) > L.sampler_workspace_bytes(h, C.byref(ok.c))
    assert L.sampler_workspace_bytes(h, C.byref(_sched(mode=2).c)) == L.sampler_workspace_bytes(h, C.byref(ok.c))
    assert L.sampler_workspace_bytes(h, C.byref(_sched(mode=2, batched=1).c)) > 0
    bad = [
        _sched(warmup=0),                         # eps_cache undefined: no warm-up, window 2
        _sched(cyc=(2, 2)),                       # cycles do not cover steps - warmup
        _sched(cyc=(2, 0, 4)),                    # zero-length cycle
        _sched(cyc=(17,)),                        # beyond the batch limit
        _sched(mode=3), _sched(mode=-1), _sched(batched=1, mode=1), _sched(warmup=-1),
        _sched(ts=[875, 750, 625, 625, 375, 250, 125, 0]),     # not strictly monotonic
        _sched(ts=[875, 750, 625, 700, 375, 250, 125, 0]),     # changes direction
    ]
    for s in bad:
        assert L.sampler_workspace_bytes(h, C.byref(s.c)) == 0
        assert L.sampler_run(h, C.byref(s.c), 0x1000, None, 0x2000, None, None, None, 0x10000, 1 << 40, None) == -5
    # an ascending time index (flow matching integrates t from 0 to 1) is as valid as a descending one
    assert L.sampler_workspace_bytes(h, C.byref(_sched(ts=[0, 125, 250, 375, 500, 625, 750, 875]).c)) > 0
    # window 1 needs no warm-up; all-warm-up needs no cycles
    assert L.sampler_workspace_bytes(h, C.byref(_sched(warmup=0, cyc=[1] * 8).c)) > 0
    assert L.sampler_workspace_bytes(h, C.byref(_sched(warmup=8, cyc=[]).c)) > 0
    # pointer and workspace checks
    need = L.sampler_workspace_bytes(h, C.byref(ok.c))
    assert L.sampler_run(h, C.byref(ok.c), None, None, 0x2000, None, None, None, 0x10000, need, None) == -1
    assert L.sampler_run(h, C.byref(ok.c), 0x1000, None, 0x2000, None, None, None, 0x10000, need - 1, None) == -4
    assert L.sampler_run(h, C.byref(ok.c), 0x1000, None, 0x2000, None, None, None, None, need, None) == -4
    assert L.sampler_run(h, C.byref(ok.c), 0x1000, None, 0x2000, None, 0x1000, None, 0x10000, need, None) == -2   # trajectory aliases x_T
    L.dit_destroy(h)


def test_inputs_are_reproducible_and_bf16_exact():
    cfg = I.CONFIGS["reduced"]
    w1 = I.make_weights(cfg.with_(layers=1), 5)
    w2 = I.make_weights(cfg.with_(layers=1), 5)
    for (n1, a1), (n2, a2) in zip(w1, w2):
        assert n1 == n2 and np.array_equal(a1, a2)
    m = dict(w1)["W_qkv.0"]
    assert np.array_equal(m, I.round_to_bf16(m))                    # already representable
    assert (m.view(np.uint32) & 0xFFFF).max() == 0
    r = I.round_to_bf16(np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -1.0 - 2 ** -9], dtype=np.float32))
    np.testing.assert_array_equal(r, np.array([1.0, 1.0 + 2 ** -6, -1.0], dtype=np.float32))   # ties to even
    assert [n for n, _ in I.weight_shapes(cfg)][:8] == ["W_pe", "b_pe", "W_t1", "b_t1", "W_t2", "b_t2",
                                                         "W_mod.0", "b_mod.0"]
    assert cfg.tokens == 16 + 2 * 6 * 8 and I.CONFIGS["full"].tokens == 17776 and I.CONFIGS["long"].tokens == 33976
    assert I.CONFIGS["block"].tokens == 4516 and I.CONFIGS["full"].latent_elems == 1123200


def test_binding_fails_loudly_without_the_built_library(monkeypatch):
    """No fallback: with the shared library missing the binding raises instead of computing anything."""
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_PATH", os.path.join(ROOT, "paper_2505_14741_amd", "no_such_library.so"))
    with pytest.raises(RuntimeError, match="missing"):
        B.lib()
    with pytest.raises(RuntimeError, match="missing"):
        B.ddim_coefficients(4)


def test_the_product_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing under the package imports or includes it."""
    pkg = os.path.join(ROOT, "paper_2505_14741_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|import_module\(.oracle|#include.*oracle", text, flags=re.M), \
                    os.path.join(dirpath, f)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
