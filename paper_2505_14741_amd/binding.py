"""ctypes binding of the HIP C-ABI library: argument marshalling only.

Every function has the name of the C entry point it calls.  PyTorch supplies device
memory (tensors) and the stream; all arithmetic runs in the library's kernels.  The
library must have been built (`python -m paper_2505_14741_amd.build` or
`__graft_entry__.build()`); if it is missing this module raises at import of the
library handle -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

from .inputs import DiTConfig

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libparastep_hip.so")
_lib = None

PS_F32, PS_BF16 = 0, 1
KERNEL_CLASSES = ("attention", "gemm_qkv", "gemm_oproj", "gemm_fc1", "gemm_fc2", "ln_modulate", "other")


class PsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().ps_strerror(status).decode()} (status {status})")


class _DitConfig(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("layers", "hidden", "heads", "head_dim", "mlp_ratio", "in_channels",
                                       "patch", "frames", "height", "width", "text_tokens",
                                       "time_embed_dim", "dtype")] + [("ln_eps", C.c_float), ("rope_theta", C.c_float)]


class _Schedule(C.Structure):
    _fields_ = [("steps", C.c_int), ("timesteps", C.POINTER(C.c_int32)), ("coef_a", C.POINTER(C.c_double)),
                ("coef_b", C.POINTER(C.c_double)), ("warmup", C.c_int), ("n_cycles", C.c_int),
                ("cycle_len", C.POINTER(C.c_int32)), ("batched", C.c_int), ("mode", C.c_int)]


class SamplerState(C.Structure):
    """Host part of a run's state between two steps (`sampler_state`); plain data, may be stored."""
    _fields_ = [("step", C.c_int32), ("cycle", C.c_int32), ("round", C.c_int32), ("toggle", C.c_int32),
                ("eps_prev", C.c_int32), ("calls", C.c_int32), ("src", C.c_int32 * 16)]


def lib():
    """Load the shared library once; fail loudly if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it first (python -m paper_2505_14741_amd.build)")
    L = C.CDLL(_LIB_PATH)
    vp, sz, i32, f32 = C.c_void_p, C.c_size_t, C.c_int, C.c_float
    sig = {
        "ps_strerror": (C.c_char_p, [i32]),
        "dit_set_kernel_path": (i32, [vp, i32]),
        "dit_get_kernel_path": (i32, [vp]),
        "dit_num_weights": (i32, [i32]),
        "dit_create": (i32, [C.POINTER(_DitConfig), C.POINTER(vp), i32, C.POINTER(vp)]),
        "dit_destroy": (i32, [vp]),
        "dit_workspace_bytes": (sz, [vp, i32]),
        "dit_forward": (i32, [vp, vp, vp, C.POINTER(C.c_int32), vp, i32, vp, sz, vp]),
        "dit_profile_enable": (i32, [vp, i32]),
        "dit_profile_read": (i32, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "ps_mfma_probe": (i32, [i32, vp, C.POINTER(C.c_double), vp]),
        "attn3d_workspace_bytes": (sz, [i32, i32, i32, i32, i32]),
        "attn3d": (i32, [vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, i32, vp, sz, vp]),
        "dit_linear_workspace_bytes": (C.c_size_t, [i32, i32, i32, i32, i32]),
        "dit_linear": (i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, C.c_size_t, vp]),
        "sampler_step_workspace_bytes": (sz, [sz]),
        "sampler_step": (i32, [vp, vp, vp, vp, C.c_double, C.c_double, sz, vp, vp, sz, vp]),
        "sampler_step_noalloc": (i32, [vp, vp, vp, vp, C.c_double, C.c_double, sz, vp, vp]),
        "rel_mae_workspace_bytes": (sz, [sz]),
        "rel_mae": (i32, [vp, vp, sz, vp, vp, sz, vp]),
        "ddim_coefficients": (i32, [i32, C.c_double, C.c_double, i32, C.POINTER(C.c_int32),
                                    C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "euler_discrete_coefficients": (i32, [i32, C.c_double, C.c_double, i32, C.POINTER(C.c_int32),
                                              C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "flow_euler_coefficients": (i32, [i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                          C.POINTER(C.c_double)]),
        "sampler_workspace_bytes": (sz, [vp, C.POINTER(_Schedule)]),
        "sampler_state_bytes": (sz, [vp, C.POINTER(_Schedule)]),
        "sampler_run_steps": (i32, [vp, C.POINTER(_Schedule), C.POINTER(SamplerState), i32, vp, vp, vp, vp, vp, vp, sz,
                                    vp]),
        "sampler_run": (i32, [vp, C.POINTER(_Schedule), vp, vp, vp, vp, vp, C.POINTER(i32), vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


EXPORTED = ("ps_strerror", "ps_mfma_probe", "dit_set_kernel_path", "dit_get_kernel_path", "sampler_step_noalloc", "dit_num_weights", "dit_create", "dit_destroy",
            "dit_workspace_bytes", "dit_forward", "dit_profile_enable", "dit_profile_read",
            "attn3d_workspace_bytes", "attn3d", "dit_linear_workspace_bytes", "dit_linear", "sampler_step_workspace_bytes", "sampler_step",
            "rel_mae_workspace_bytes", "rel_mae", "ddim_coefficients", "euler_discrete_coefficients",
            "flow_euler_coefficients", "sampler_workspace_bytes", "sampler_run", "sampler_state_bytes",
            "sampler_run_steps")


def _check(status: int, where: str):
    if status != 0:
        raise PsError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(name: str) -> int:
    return {"f32": PS_F32, "bf16": PS_BF16}[name]


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


# ---------------------------------------------------------------------------- predictor
class Dit:
    """Owner of a `dit*` handle and of the weight tensors it borrows."""

    def __init__(self, cfg: DiTConfig, weights: Sequence[torch.Tensor]):
        L = lib()
        self.cfg = cfg
        self.weights = list(weights)            # keep alive
        c = _DitConfig(cfg.layers, cfg.hidden, cfg.heads, cfg.head_dim, cfg.mlp_ratio, cfg.in_channels,
                       cfg.patch, cfg.frames, cfg.height, cfg.width, cfg.text_tokens, cfg.time_embed_dim,
                       _dt(cfg.dtype), cfg.ln_eps, cfg.rope_theta)
        arr = (C.c_void_p * len(self.weights))(*[w.data_ptr() for w in self.weights])
        h = C.c_void_p()
        _check(L.dit_create(C.byref(c), arr, len(self.weights), C.byref(h)), "dit_create")
        self.handle = h
        self._ws = {}

    def close(self):
        if getattr(self, "handle", None):
            lib().dit_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, batch: int) -> torch.Tensor:
        if batch not in self._ws:
            n = lib().dit_workspace_bytes(self.handle, batch)
            if n == 0:
                raise PsError(-2, "dit_workspace_bytes")
            self._ws[batch] = _workspace(n, self.weights[0].device)
        return self._ws[batch]


def dit_create(cfg: DiTConfig, weights: Sequence[torch.Tensor]) -> Dit:
    return Dit(cfg, weights)


def dit_set_kernel_path(d: Dit, path: int):
    _check(lib().dit_set_kernel_path(d.handle, int(path)), "dit_set_kernel_path")


def dit_forward(d: Dit, x: torch.Tensor, ctx: Optional[torch.Tensor], t: Sequence[int],
                eps_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    B = x.shape[0]
    if eps_out is None:
        eps_out = torch.empty_like(x)
    ws = d.workspace(B)
    tt = (C.c_int32 * B)(*[int(v) for v in t])
    _check(lib().dit_forward(d.handle, _ptr(x), _ptr(ctx), tt, _ptr(eps_out), B, _ptr(ws), ws.numel(), _stream()),
           "dit_forward")
    return eps_out


def dit_profile_enable(d: Dit, on):
    """on: False/0 off, True/1 every kernel class, 2 the attention class only."""
    _check(lib().dit_profile_enable(d.handle, int(on)), "dit_profile_enable")


def dit_profile_read(d: Dit):
    ms = (C.c_double * 7)()
    cnt = (C.c_int64 * 7)()
    _check(lib().dit_profile_read(d.handle, ms, cnt), "dit_profile_read")
    return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}


def ps_mfma_probe(iters: int, sink: torch.Tensor) -> float:
    """Enqueue the MFMA-only launch; returns the operations it performs (time it with events)."""
    flops = C.c_double(0.0)
    _check(lib().ps_mfma_probe(int(iters), _ptr(sink), C.byref(flops), _stream()), "ps_mfma_probe")
    return flops.value


# ---------------------------------------------------------------------------- attention
def attn3d(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scale: float,
           out: Optional[torch.Tensor] = None, kernel_path: int = 0) -> torch.Tensor:
    B, N, H, d = q.shape
    dt = PS_BF16 if q.dtype == torch.bfloat16 else PS_F32
    if out is None:
        out = torch.empty_like(q)
    n = lib().attn3d_workspace_bytes(B, N, H, d, dt)
    ws = _workspace(n, q.device)
    _check(lib().attn3d(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, N, H, d, float(scale), dt, int(kernel_path),
                        _ptr(ws), n, _stream()), "attn3d")
    return out


def dit_linear(a: torch.Tensor, w: torch.Tensor, bias: torch.Tensor, act: int = 0,
               out: Optional[torch.Tensor] = None, use_workspace: bool = True, kernel_path: int = 0) -> torch.Tensor:
    M, K = a.shape
    Nn = w.shape[0]
    dt = PS_BF16 if a.dtype == torch.bfloat16 else PS_F32
    if out is None:
        out = torch.empty(M, Nn, dtype=a.dtype, device=a.device)
    nb = lib().dit_linear_workspace_bytes(M, Nn, K, dt, int(kernel_path)) if use_workspace else 0
    ws = _workspace(nb, a.device)
    _check(lib().dit_linear(_ptr(a), _ptr(w), _ptr(bias), _ptr(out), M, Nn, K, int(act), dt, int(kernel_path),
                            _ptr(ws), nb, _stream()), "dit_linear")
    return out


# ---------------------------------------------------------------- scheduler and metric
def sampler_step(x: torch.Tensor, eps: torch.Tensor, eps_prev: Optional[torch.Tensor], a: float, b: float,
                 x_out: Optional[torch.Tensor] = None, want_sums: bool = True):
    n = x.numel()
    if x_out is None:
        x_out = torch.empty_like(x)
    sums = torch.empty(4, dtype=torch.float32, device=x.device) if want_sums else None
    nb = lib().sampler_step_workspace_bytes(n) if want_sums else 0
    ws = _workspace(nb, x.device)
    _check(lib().sampler_step(_ptr(x), _ptr(eps), _ptr(eps_prev), _ptr(x_out), float(a), float(b), n, _ptr(sums),
                              _ptr(ws), nb, _stream()), "sampler_step")
    return x_out, sums


def sampler_step_noalloc(x: torch.Tensor, eps: torch.Tensor, eps_prev: Optional[torch.Tensor], a: float, b: float,
                         x_out: torch.Tensor, sums: Optional[torch.Tensor]):
    """The caller supplies every buffer; neither this wrapper nor the library allocates."""
    _check(lib().sampler_step_noalloc(_ptr(x), _ptr(eps), _ptr(eps_prev), _ptr(x_out), float(a), float(b), x.numel(),
                                      _ptr(sums), _stream()), "sampler_step_noalloc")
    return x_out, sums


def rel_mae(a: torch.Tensor, b: torch.Tensor) -> torch.Tensor:
    n = a.numel()
    out = torch.empty(3, dtype=torch.float32, device=a.device)
    nb = lib().rel_mae_workspace_bytes(n)
    ws = _workspace(nb, a.device)
    _check(lib().rel_mae(_ptr(a), _ptr(b), n, _ptr(out), _ptr(ws), nb, _stream()), "rel_mae")
    return out


def ddim_coefficients(steps: int, train_steps: int = 1000, beta_start: float = 1e-4, beta_end: float = 2e-2):
    ts = (C.c_int32 * steps)()
    a = (C.c_double * steps)()
    b = (C.c_double * steps)()
    _check(lib().ddim_coefficients(train_steps, beta_start, beta_end, steps, ts, a, b), "ddim_coefficients")
    return (np.array(ts[:], dtype=np.int32), np.array(a[:], dtype=np.float64), np.array(b[:], dtype=np.float64))


def euler_discrete_coefficients(steps: int, train_steps: int = 1000, beta_start: float = 1e-4, beta_end: float = 2e-2):
    ts = (C.c_int32 * steps)()
    a = (C.c_double * steps)()
    b = (C.c_double * steps)()
    _check(lib().euler_discrete_coefficients(train_steps, beta_start, beta_end, steps, ts, a, b),
           "euler_discrete_coefficients")
    return (np.array(ts[:], dtype=np.int32), np.array(a[:], dtype=np.float64), np.array(b[:], dtype=np.float64))


def flow_euler_coefficients(steps: int, train_steps: int = 1000):
    ts = (C.c_int32 * steps)()
    a = (C.c_double * steps)()
    b = (C.c_double * steps)()
    _check(lib().flow_euler_coefficients(train_steps, steps, ts, a, b), "flow_euler_coefficients")
    return (np.array(ts[:], dtype=np.int32), np.array(a[:], dtype=np.float64), np.array(b[:], dtype=np.float64))


# ------------------------------------------------------------------ reuse-then-predict
class Schedule:
    """Host arrays behind a `sampler_schedule` (kept alive while the struct is in use)."""

    def __init__(self, timesteps, coef_a, coef_b, warmup: int, cycle_len: Sequence[int], batched: bool = False,
                 mode: int = 0):
        self.ts = np.ascontiguousarray(timesteps, dtype=np.int32)
        self.a = np.ascontiguousarray(coef_a, dtype=np.float64)
        self.b = np.ascontiguousarray(coef_b, dtype=np.float64)
        self.cyc = np.ascontiguousarray(cycle_len, dtype=np.int32)
        self.c = _Schedule(len(self.ts), self.ts.ctypes.data_as(C.POINTER(C.c_int32)),
                           self.a.ctypes.data_as(C.POINTER(C.c_double)), self.b.ctypes.data_as(C.POINTER(C.c_double)),
                           int(warmup), len(self.cyc), self.cyc.ctypes.data_as(C.POINTER(C.c_int32)),
                           int(batched), int(mode))


def sampler_run(d: Dit, sched: Schedule, x_T: torch.Tensor, ctx: Optional[torch.Tensor],
                want_trajectory: bool = False):
    """Returns (x0, step_sums [steps,4], predictor launches), plus the per-step samples [steps, ...] if asked."""
    L = lib()
    nb = L.sampler_workspace_bytes(d.handle, C.byref(sched.c))
    if nb == 0:
        raise PsError(-5, "sampler_workspace_bytes")
    ws = _workspace(nb, x_T.device)
    x0 = torch.empty_like(x_T)
    sums = torch.zeros(len(sched.ts), 4, dtype=torch.float32, device=x_T.device)
    traj = (torch.empty((len(sched.ts),) + tuple(x_T.shape), dtype=torch.float32, device=x_T.device)
            if want_trajectory else None)
    calls = C.c_int(0)
    _check(L.sampler_run(d.handle, C.byref(sched.c), _ptr(x_T), _ptr(ctx), _ptr(x0), _ptr(sums), _ptr(traj),
                         C.byref(calls), _ptr(ws), nb, _stream()), "sampler_run")
    if want_trajectory:
        return x0, sums, calls.value, traj
    return x0, sums, calls.value


def sampler_workspace(d: Dit, sched: Schedule, device) -> torch.Tensor:
    nb = lib().sampler_workspace_bytes(d.handle, C.byref(sched.c))
    if nb == 0:
        raise PsError(-5, "sampler_workspace_bytes")
    return _workspace(nb, device)


def sampler_state_bytes(d: Dit, sched: Schedule) -> int:
    return lib().sampler_state_bytes(d.handle, C.byref(sched.c))


def sampler_run_steps(d: Dit, sched: Schedule, state: SamplerState, stop_step: int, x_T: Optional[torch.Tensor],
                      ctx: Optional[torch.Tensor], ws: torch.Tensor, x_out: Optional[torch.Tensor] = None,
                      step_sums: Optional[torch.Tensor] = None, trajectory: Optional[torch.Tensor] = None):
    """Advance a run from state.step to stop_step; `ws` (from sampler_workspace) carries the tensors of the state."""
    _check(lib().sampler_run_steps(d.handle, C.byref(sched.c), C.byref(state), int(stop_step), _ptr(x_T), _ptr(ctx),
                                   _ptr(x_out), _ptr(step_sums), _ptr(trajectory), _ptr(ws), ws.numel(), _stream()),
           "sampler_run_steps")
    return x_out


def weights_to_device(cfg: DiTConfig, weights, device="cuda") -> List[torch.Tensor]:
    """Upload a weight list (name, fp32 ndarray): matrices in cfg.dtype, biases fp32."""
    out = []
    for _, w in weights:
        t = torch.from_numpy(np.ascontiguousarray(w))
        if w.ndim == 2:
            t = t.to(torch_dtype(cfg.dtype))
        out.append(t.to(device).contiguous())
    return out
