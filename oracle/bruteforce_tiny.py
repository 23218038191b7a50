"""Loop-level DiT forward for tiny shapes.  TEST INFRASTRUCTURE ONLY.

A second statement of the noise predictor, written token by token and head by head
with Python loops, Python complex numbers for the rotary embedding and explicit
exp/sum softmax.  The only library step is the inner product of two vectors.  It
exists so the vectorised oracle's wiring (token order, chunk order of the modulation
vector, head slicing, pair interleaving, patch order) is checked against code with a
different shape; it shares nothing with the HIP path and is usable only at sizes of
a few hundred tokens.
"""
from __future__ import annotations

import cmath
import math

import numpy as np


def _dot(u, v):
    return float(np.dot(np.asarray(u, dtype=np.float64), np.asarray(v, dtype=np.float64)))


def _linear(Wm, bias, vec):
    return [_dot(Wm[o], vec) + float(bias[o]) for o in range(Wm.shape[0])]


def _silu(z):
    return z / (1.0 + math.exp(-z))


def _gelu(z):
    return 0.5 * z * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z * z * z)))


def _ln(vec, eps):
    n = len(vec)
    mu = sum(vec) / n
    var = sum((z - mu) * (z - mu) for z in vec) / n
    r = 1.0 / math.sqrt(var + eps)
    return [(z - mu) * r for z in vec]


def dit_forward_loops(cfg, W, x, ctx, t):
    """eps for ONE sample: x [C,F,H,W], ctx [L_txt,D] or None, integer t."""
    D, H, d, Lt = cfg.hidden, cfg.heads, cfg.head_dim, cfg.text_tokens
    C, Fr, Hh, Ww = cfg.latent_shape
    ps = cfg.patch
    Hp, Wp = Hh // ps, Ww // ps
    x = np.asarray(x, dtype=np.float64)

    # timestep features: cosines first, then sines
    half = D // 2
    feat = [math.cos(t * 10000.0 ** (-j / half)) for j in range(half)]
    feat += [math.sin(t * 10000.0 ** (-j / half)) for j in range(half)]
    hid = [_silu(z) for z in _linear(W["W_t1"], W["b_t1"], feat)]
    cvec = [_silu(z) for z in _linear(W["W_t2"], W["b_t2"], hid)]

    # tokens: text rows, then one row per (frame, patch row, patch col)
    toks, pos = [], []
    for n in range(Lt):
        toks.append([float(z) for z in ctx[n]])
        pos.append(None)
    for f in range(Fr):
        for i in range(Hp):
            for j in range(Wp):
                pv = []
                for c in range(C):
                    for dy in range(ps):
                        for dx in range(ps):
                            pv.append(x[c, f, i * ps + dy, j * ps + dx])
                toks.append(_linear(W["W_pe"], W["b_pe"], pv))
                pos.append((f, i, j))
    N = len(toks)

    widths = (d // 4, 3 * d // 8, 3 * d // 8)

    def rotate(vec, p3):
        out = list(vec)
        base = 0
        for axis in range(3):
            dA = widths[axis]
            for m in range(dA // 2):
                ang = p3[axis] * cfg.rope_theta ** (-2.0 * m / dA)
                z = complex(vec[base + 2 * m], vec[base + 2 * m + 1]) * cmath.exp(1j * ang)
                out[base + 2 * m], out[base + 2 * m + 1] = z.real, z.imag
            base += dA
        return out

    for l in range(cfg.layers):
        mod = _linear(W[f"W_mod.{l}"], W[f"b_mod.{l}"], cvec)

        def chunk(k, n):
            s = 6 if n < Lt else 0          # text tokens use the second set of six
            return mod[(s + k) * D:(s + k + 1) * D]

        qs, ks, vs = [], [], []
        for n in range(N):
            y = _ln(toks[n], cfg.ln_eps)
            sh, sc = chunk(0, n), chunk(1, n)
            hvec = [y[e] * (1.0 + sc[e]) + sh[e] for e in range(D)]
            qkv = _linear(W[f"W_qkv.{l}"], W[f"b_qkv.{l}"], hvec)
            qh, kh, vh = [], [], []
            for hd in range(H):
                qv = qkv[0 * D + hd * d:0 * D + (hd + 1) * d]
                kv = qkv[1 * D + hd * d:1 * D + (hd + 1) * d]
                vv = qkv[2 * D + hd * d:2 * D + (hd + 1) * d]
                if pos[n] is not None:
                    qv, kv = rotate(qv, pos[n]), rotate(kv, pos[n])
                qh.append(qv); kh.append(kv); vh.append(vv)
            qs.append(qh); ks.append(kh); vs.append(vh)
        new = []
        for n in range(N):
            att = []
            for hd in range(H):
                logit = [_dot(qs[n][hd], ks[j][hd]) / math.sqrt(d) for j in range(N)]
                mx = max(logit)
                w = [math.exp(z - mx) for z in logit]
                tot = sum(w)
                for e in range(d):
                    att.append(sum(w[j] * vs[j][hd][e] for j in range(N)) / tot)
            proj = _linear(W[f"W_o.{l}"], W[f"b_o.{l}"], att)
            g = chunk(2, n)
            xa = [toks[n][e] + g[e] * proj[e] for e in range(D)]
            y = _ln(xa, cfg.ln_eps)
            sh, sc, g2 = chunk(3, n), chunk(4, n), chunk(5, n)
            h2 = [y[e] * (1.0 + sc[e]) + sh[e] for e in range(D)]
            u = [_gelu(z) for z in _linear(W[f"W_1.{l}"], W[f"b_1.{l}"], h2)]
            m2 = _linear(W[f"W_2.{l}"], W[f"b_2.{l}"], u)
            new.append([xa[e] + g2[e] * m2[e] for e in range(D)])
        toks = new

    modf = _linear(W["W_fm"], W["b_fm"], cvec)
    eps = np.zeros((C, Fr, Hh, Ww), dtype=np.float64)
    for n in range(Lt, N):
        f, i, j = pos[n]
        y = _ln(toks[n], cfg.ln_eps)
        yv = [y[e] * (1.0 + modf[D + e]) + modf[e] for e in range(D)]
        o = _linear(W["W_out"], W["b_out"], yv)
        idx = 0
        for c in range(C):
            for dy in range(ps):
                for dx in range(ps):
                    eps[c, f, i * ps + dy, j * ps + dx] = o[idx]
                    idx += 1
    return eps
