// C ABI: argument validation, the DiT forward schedule, and the reuse-then-predict run
// (Algorithm 1 with every rank of a cycle simulated on one device).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"

using namespace ps;

namespace {

constexpr int MAX_BATCH = 16;
constexpr int MAX_LAYERS = 64;
constexpr int N_CLASSES = 7;
enum KClass { KC_ATTN = 0, KC_QKV = 1, KC_OPROJ = 2, KC_FC1 = 3, KC_FC2 = 4, KC_LN = 5, KC_OTHER = 6 };

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

struct LayerW { const void *W_mod, *W_qkv, *W_o, *W_1, *W_2; const float *b_mod, *b_qkv, *b_o, *b_1, *b_2; };

}  // namespace

struct dit {
    dit_config cfg;
    const void *W_pe, *W_t1, *W_t2, *W_fm, *W_out;
    const float *b_pe, *b_t1, *b_t2, *b_fm, *b_out;
    std::vector<LayerW> layers;
    int Hp, Wp, Nv, N, P;
    size_t esize;
    int kernel_path = 0;            // see kernel_path_valid(); dit_set_kernel_path
    // profiling
    int profiling = 0;              // 0 off, 1 every class, 2 the attention class only
    std::vector<hipEvent_t> ev;           // pairs: start, stop
    std::vector<int> ev_class;
    size_t ev_used = 0;
    double prof_ms[N_CLASSES] = {0};
    int64_t prof_n[N_CLASSES] = {0};
};

namespace {

struct WsLayout {
    size_t X, H, QKV, mod, modf, sinus, hid, cvec, rope, attn, gemm, gemm_bytes, total;
};

WsLayout ws_layout(const dit* d, int batch) {
    const dit_config& c = d->cfg;
    size_t M = (size_t)batch * d->N, D = c.hidden;
    WsLayout w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    w.X = take(M * D * 4);
    w.H = take(M * D * d->esize);                                  // LN output / attention output
    size_t wide = (size_t)(c.mlp_ratio > 3 ? c.mlp_ratio : 3);
    w.QKV = take(M * wide * D * d->esize);                         // qkv, later the MLP hidden
    w.mod = take((size_t)batch * c.layers * 12 * D * 4);
    w.modf = take((size_t)batch * 2 * D * 4);
    w.sinus = take((size_t)batch * D * 4);
    w.hid = take((size_t)batch * c.time_embed_dim * 4);
    w.cvec = take((size_t)batch * c.time_embed_dim * 4);
    w.rope = take(rope_table_floats(c.frames, d->Hp, d->Wp, c.head_dim) * 4);   // (cos, sin) per axis position and pair
    w.attn = take(attention_workspace_bytes(c.dtype, batch, d->N, c.heads, c.head_dim));
    {   // K-split scratch of the projections: the largest need of the four shapes of a layer, under any tile
        // variant a kernel path can force (so the size does not change when the handle's path does)
        const int Di = (int)D, Fi = (int)(c.mlp_ratio * D);
        size_t g = 0;
        for (int v = 0; v <= PS_PATH_MAX_VARIANT; ++v) {
            const int path = v << 8;
            g = std::max(g, gemm_split_workspace_bytes(c.dtype, batch, d->N, 3 * Di, Di, path));
            g = std::max(g, gemm_split_workspace_bytes(c.dtype, batch, d->N, Di, Di, path));
            g = std::max(g, gemm_split_workspace_bytes(c.dtype, batch, d->N, Fi, Di, path));
            g = std::max(g, gemm_split_workspace_bytes(c.dtype, batch, d->N, Di, Fi, path));
        }
        w.gemm_bytes = g;
        w.gemm = take(g);
    }
    w.total = off;
    return w;
}

struct Prof {
    dit* d;
    hipStream_t st;
    hipError_t begin(int cls, hipEvent_t* stop) {
        *stop = nullptr;
        if (!d->profiling || (d->profiling == 2 && cls != KC_ATTN)) return hipSuccess;
        if (d->ev_used + 2 > d->ev.size()) {
            // timing-only events: without the system-scope fence (cache write-back and invalidation) an event
            // otherwise performs when it is recorded, which delays the launch that follows
            hipEvent_t a, b;
            hipError_t e = hipEventCreateWithFlags(&a, hipEventDisableSystemFence);
            if (e != hipSuccess) return e;
            e = hipEventCreateWithFlags(&b, hipEventDisableSystemFence);
            if (e != hipSuccess) { hipEventDestroy(a); return e; }
            d->ev.push_back(a);
            d->ev.push_back(b);
            d->ev_class.push_back(cls);
        }
        d->ev_class[d->ev_used / 2] = cls;
        hipError_t e = hipEventRecord(d->ev[d->ev_used], st);
        *stop = d->ev[d->ev_used + 1];
        d->ev_used += 2;
        return e;
    }
    hipError_t end(hipEvent_t stop) { return stop ? hipEventRecord(stop, st) : hipSuccess; }
};

#define PS_TRY(expr)                         \
    do {                                     \
        hipError_t e__ = (expr);             \
        if (e__ != hipSuccess) return PS_ERR_HIP; \
    } while (0)

#define PS_TIMED(cls, expr)                  \
    do {                                     \
        hipEvent_t stop__;                   \
        PS_TRY(prof.begin(cls, &stop__));    \
        PS_TRY(expr);                        \
        PS_TRY(prof.end(stop__));            \
    } while (0)

int validate_forward(const dit* d, const float* x, const void* ctx, const int32_t* t_host,
                     const float* eps_out, int batch, const void* ws, size_t ws_bytes) {
    if (!d || !x || !t_host || !eps_out) return PS_ERR_NULL;
    if (d->cfg.text_tokens > 0 && !ctx) return PS_ERR_NULL;
    if (batch < 1 || batch > MAX_BATCH) return PS_ERR_SHAPE;
    if (x == eps_out) return PS_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(eps_out, 16) || (ctx && !aligned(ctx, 16))) return PS_ERR_SHAPE;
    for (int b = 0; b < batch; ++b)
        if (t_host[b] < 0 || t_host[b] >= 100000) return PS_ERR_SHAPE;
    if (!ws || !aligned(ws, 256) || ws_bytes < dit_workspace_bytes(d, batch)) return PS_ERR_WORKSPACE;
    return PS_OK;
}

// ctx_shared: every sample reads the same [text_tokens, hidden] context (the ranks of a
// reuse-then-predict cycle share one prompt).
int forward_impl(dit* d, const float* x, const void* ctx, const int32_t* t_host, float* eps_out,
                 int batch, void* workspace, hipStream_t st, bool ctx_shared = false) {
    const dit_config& c = d->cfg;
    const int D = c.hidden, Dt = c.time_embed_dim, L = c.layers, N = d->N, M = batch * N;
    const int dt = c.dtype, path = d->kernel_path;
    WsLayout w = ws_layout(d, batch);
    char* base = (char*)workspace;
    float* X = (float*)(base + w.X);
    void* Hb = base + w.H;
    void* QKV = base + w.QKV;
    float* mod = (float*)(base + w.mod);
    float* modf = (float*)(base + w.modf);
    float* sinus = (float*)(base + w.sinus);
    float* hid = (float*)(base + w.hid);
    float* cvec = (float*)(base + w.cvec);
    float* rope = (float*)(base + w.rope);
    void* attn_ws = attention_workspace_bytes(dt, batch, N, c.heads, c.head_dim) ? base + w.attn : nullptr;
    float* gemm_ws = w.gemm_bytes ? (float*)(base + w.gemm) : nullptr;
    Prof prof{d, st};
    TokenGeom geom{N, c.text_tokens};
    const long mod_bs = (long)L * 12 * D;

    // time conditioning: c = SiLU(W_t2 SiLU(W_t1 s(t) + b_t1) + b_t2); all modulation vectors
    PS_TIMED(KC_OTHER, launch_sinusoid(t_host, sinus, batch, D, st));
    PS_TIMED(KC_OTHER, launch_gemv(dt, d->W_t1, d->b_t1, sinus, hid, Dt, D, batch, D, Dt, 1, st));
    PS_TIMED(KC_OTHER, launch_gemv(dt, d->W_t2, d->b_t2, hid, cvec, Dt, Dt, batch, Dt, Dt, 1, st));
    for (int l0 = 0; l0 < L; l0 += GEMV_SET) {           // the layers' modulation matrices, 32 per launch
        GemvSet set{};
        const int cnt = L - l0 < GEMV_SET ? L - l0 : GEMV_SET;
        for (int i = 0; i < cnt; ++i) {
            set.W[i] = d->layers[l0 + i].W_mod; set.bias[i] = d->layers[l0 + i].b_mod;
            set.out[i] = mod + (long)(l0 + i) * 12 * D;
        }
        PS_TIMED(KC_OTHER, launch_gemv_set(dt, set, cnt, cvec, 12 * D, Dt, batch, Dt, mod_bs, 0, st));
    }
    PS_TIMED(KC_OTHER, launch_gemv(dt, d->W_fm, d->b_fm, cvec, modf, 2 * D, Dt, batch, Dt, 2 * D, 0, st));
    PS_TIMED(KC_OTHER, launch_rope_table(rope, c.frames, d->Hp, d->Wp, c.head_dim, c.rope_theta, st));
    PS_TIMED(KC_OTHER, launch_patch_embed(dt, x, ctx, d->W_pe, d->b_pe, X, batch, c.in_channels, c.frames,
                                          c.height, c.width, c.patch, c.text_tokens, D,
                                          ctx_shared ? 0L : (long)c.text_tokens * D, st));

    const size_t es = d->esize;
    AttnStrides as;
    as.q_tok = as.k_tok = as.v_tok = 3L * D;
    as.q_head = as.k_head = as.v_head = c.head_dim;
    as.q_batch = as.k_batch = as.v_batch = (long)N * 3 * D;
    as.o_tok = D; as.o_head = c.head_dim; as.o_batch = (long)N * D;
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    // the MFMA attention kernel takes queries that already carry scale*log2(e); the QKV
    // projection applies the factor in fp32, before its single rounding to bf16
    const bool prescale = attention_uses_mfma(dt, c.head_dim, path);

    for (int l = 0; l < L; ++l) {
        const LayerW& lw = d->layers[l];
        const float* mod_l = mod + (long)l * 12 * D;
        // the attention kernels mark heads in a small flag array; the LayerNorm kernel in front of the QKV projection
        // clears it instead of a launch of its own
        int nflags = 0;
        float* flags = attention_head_flags(dt, batch, c.heads, c.head_dim, attn_ws, path, st, false, &nflags);
        // h = LN(X)(1+scale_a)+shift_a
        PS_TIMED(KC_LN, launch_ln_modulate(dt, X, Hb, M, D, c.ln_eps, mod_l, mod_bs, 0, 1, geom, st, flags, nflags));
        // [q|k|v] = W_qkv h + b, rotary on video q,k
        Epilogue eq{};
        eq.kind = EPI_QKV_ROPE; eq.bias = lw.b_qkv; eq.D = D; eq.geom = geom;
        eq.rope_cs = rope; eq.head_dim = c.head_dim; eq.rope_F = c.frames; eq.rope_Hp = d->Hp; eq.rope_Wp = d->Wp;
        eq.q_scale = prescale ? scale * 1.4426950408889634f : 1.0f;
        eq.split_ws = gemm_ws; eq.split_ws_bytes = w.gemm_bytes;
        PS_TIMED(KC_QKV, launch_gemm(dt, Hb, lw.W_qkv, QKV, batch, N, 3 * D, D, eq, path, st));
        // o = attention(q, k, v) -> Hb (token-major, heads concatenated)
        const char* qp = (const char*)QKV;
        PS_TIMED(KC_ATTN, launch_attention(dt, qp, qp + (size_t)D * es, qp + (size_t)2 * D * es, Hb, batch, N,
                                           c.heads, c.head_dim, scale, as, attn_ws, path, st, prescale,
                                           flags != nullptr));
        // X += gate_a * (W_o o + b_o)
        Epilogue eo{};
        eo.kind = EPI_GATE_RESIDUAL; eo.bias = lw.b_o; eo.resid = X; eo.mod_layer = mod_l;
        eo.mod_batch_stride = mod_bs; eo.gate_chunk = 2; eo.D = D; eo.geom = geom;
        eo.split_ws = gemm_ws; eo.split_ws_bytes = w.gemm_bytes;
        PS_TIMED(KC_OPROJ, launch_gemm(dt, Hb, lw.W_o, nullptr, batch, N, D, D, eo, path, st));
        // h2 = LN(X)(1+scale_m)+shift_m ; u = GELU(W_1 h2 + b_1) ; X += gate_m * (W_2 u + b_2)
        PS_TIMED(KC_LN, launch_ln_modulate(dt, X, Hb, M, D, c.ln_eps, mod_l, mod_bs, 3, 4, geom, st));
        Epilogue e1{};
        e1.kind = EPI_BIAS_GELU; e1.bias = lw.b_1;
        e1.split_ws = gemm_ws; e1.split_ws_bytes = w.gemm_bytes;
        PS_TIMED(KC_FC1, launch_gemm(dt, Hb, lw.W_1, QKV, batch, N, c.mlp_ratio * D, D, e1, path, st));
        Epilogue e2 = eo;
        e2.bias = lw.b_2; e2.gate_chunk = 5;
        PS_TIMED(KC_FC2, launch_gemm(dt, QKV, lw.W_2, nullptr, batch, N, D, c.mlp_ratio * D, e2, path, st));
    }
    // eps = unpatchify(W_out (LN(X)(1+scale_f)+shift_f) + b_out) over the video tokens
    const int P = c.in_channels * c.patch * c.patch;
    if (gemm_uses_mfma(dt, N, P, D, path)) {
        // as every other projection: normalised rows in bf16 (text rows included, dropped by the epilogue)
        PS_TIMED(KC_LN, launch_ln_modulate(dt, X, Hb, M, D, c.ln_eps, modf, 2L * D, 0, 1, TokenGeom{N, 0}, st));
        Epilogue ef{};
        ef.kind = EPI_UNPATCHIFY; ef.bias = d->b_out; ef.resid = eps_out; ef.geom = geom;
        ef.pg = PatchGeom{c.in_channels, c.frames, c.height, c.width, c.patch};
        PS_TIMED(KC_OTHER, launch_gemm(dt, Hb, d->W_out, nullptr, batch, N, P, D, ef, path, st));
    } else {
        PS_TIMED(KC_OTHER, launch_final_proj(dt, X, modf, d->W_out, d->b_out, eps_out, batch, c.in_channels,
                                             c.frames, c.height, c.width, c.patch, c.text_tokens, D, c.ln_eps, st));
    }
    return PS_OK;
}

}  // namespace

extern "C" {

const char* ps_strerror(int status) {
    switch (status) {
        case PS_OK: return "ok";
        case PS_ERR_NULL: return "a required pointer is NULL";
        case PS_ERR_SHAPE: return "inconsistent or unsupported sizes";
        case PS_ERR_DTYPE: return "unknown dtype";
        case PS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case PS_ERR_SCHEDULE: return "invalid sampling schedule";
        case PS_ERR_HIP: return "HIP runtime call or kernel launch failed";
        default: return "unknown status";
    }
}

int dit_get_kernel_path(const dit* d) { return d ? d->kernel_path : PS_ERR_NULL; }

int dit_set_kernel_path(dit* d, int path) {
    if (!d) return PS_ERR_NULL;
    if (!kernel_path_valid(path)) return PS_ERR_SHAPE;
    d->kernel_path = path;
    return PS_OK;
}

int dit_num_weights(int layers) { return layers < 0 ? 0 : 6 + 10 * layers + 4; }

int dit_create(const dit_config* cfg, const void* const* weights, int n_weights, dit** out) {
    if (!cfg || !weights || !out) return PS_ERR_NULL;
    *out = nullptr;
    const dit_config& c = *cfg;
    if (c.dtype != PS_F32 && c.dtype != PS_BF16) return PS_ERR_DTYPE;
    if (c.layers < 1 || c.layers > MAX_LAYERS || c.hidden < 1 || c.heads < 1 || c.head_dim < 1) return PS_ERR_SHAPE;
    if (c.hidden != c.heads * c.head_dim || c.head_dim % 16 != 0) return PS_ERR_SHAPE;
    if (c.head_dim != 16 && c.head_dim != 32 && c.head_dim != 64) return PS_ERR_SHAPE;
    if (c.hidden % 8 != 0 || c.hidden > 2048) return PS_ERR_SHAPE;
    if (c.mlp_ratio < 1 || c.mlp_ratio > 8) return PS_ERR_SHAPE;
    if (c.in_channels < 1 || c.patch < 1 || c.frames < 1 || c.height < 1 || c.width < 1) return PS_ERR_SHAPE;
    if (c.height % c.patch || c.width % c.patch) return PS_ERR_SHAPE;
    if (c.text_tokens < 0 || c.time_embed_dim < 1) return PS_ERR_SHAPE;
    // the patch-embedding kernel stages 16 patch vectors in LDS (64 bytes per patch value, 64 KB at most)
    if ((long)c.in_channels * c.patch * c.patch > 1024) return PS_ERR_SHAPE;
    if (!(c.ln_eps > 0.f) || !(c.rope_theta > 1.f)) return PS_ERR_SHAPE;
    if ((long)c.in_channels * c.frames * c.height * c.width % 4 != 0) return PS_ERR_SHAPE;
    if (n_weights != dit_num_weights(c.layers)) return PS_ERR_SHAPE;
    for (int i = 0; i < n_weights; ++i) {
        if (!weights[i]) return PS_ERR_NULL;
        if (!aligned(weights[i], 16)) return PS_ERR_SHAPE;
    }
    long nv = (long)c.frames * (c.height / c.patch) * (c.width / c.patch);
    if (nv + c.text_tokens > (1L << 24)) return PS_ERR_SHAPE;
    // the bf16 projections address a sample's activations with 32-bit element offsets
    if (c.dtype == PS_BF16 && (nv + c.text_tokens) * (long)c.hidden * std::max(c.mlp_ratio, 3) >= (1L << 31))
        return PS_ERR_SHAPE;
    dit* d = new (std::nothrow) dit();
    if (!d) return PS_ERR_HIP;
    d->cfg = c;
    d->Hp = c.height / c.patch;
    d->Wp = c.width / c.patch;
    d->Nv = (int)nv;
    d->N = d->Nv + c.text_tokens;
    d->P = c.in_channels * c.patch * c.patch;
    d->esize = c.dtype == PS_BF16 ? 2 : 4;
    int i = 0;
    d->W_pe = weights[i++]; d->b_pe = (const float*)weights[i++];
    d->W_t1 = weights[i++]; d->b_t1 = (const float*)weights[i++];
    d->W_t2 = weights[i++]; d->b_t2 = (const float*)weights[i++];
    d->layers.resize(c.layers);
    for (int l = 0; l < c.layers; ++l) {
        LayerW& lw = d->layers[l];
        lw.W_mod = weights[i++]; lw.b_mod = (const float*)weights[i++];
        lw.W_qkv = weights[i++]; lw.b_qkv = (const float*)weights[i++];
        lw.W_o = weights[i++];   lw.b_o = (const float*)weights[i++];
        lw.W_1 = weights[i++];   lw.b_1 = (const float*)weights[i++];
        lw.W_2 = weights[i++];   lw.b_2 = (const float*)weights[i++];
    }
    d->W_fm = weights[i++]; d->b_fm = (const float*)weights[i++];
    d->W_out = weights[i++]; d->b_out = (const float*)weights[i++];
    *out = d;
    return PS_OK;
}

int dit_destroy(dit* d) {
    if (!d) return PS_ERR_NULL;
    for (hipEvent_t e : d->ev) hipEventDestroy(e);
    delete d;
    return PS_OK;
}

size_t dit_workspace_bytes(const dit* d, int batch) {
    if (!d || batch < 1 || batch > MAX_BATCH) return 0;
    return ws_layout(d, batch).total;
}

int dit_forward(dit* d, const float* x, const void* ctx, const int32_t* t_host, float* eps_out,
                int batch, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int rc = validate_forward(d, x, ctx, t_host, eps_out, batch, workspace, workspace_bytes);
    if (rc != PS_OK) return rc;
    return forward_impl(d, x, ctx, t_host, eps_out, batch, workspace, (hipStream_t)hip_stream);
}

int ps_mfma_probe(int iters, float* sink, double* flops_out, void* hip_stream) {
    if (!sink || !flops_out) return PS_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return PS_ERR_SHAPE;
    hipError_t e = launch_mfma_probe(iters, sink, flops_out, (hipStream_t)hip_stream);
    return e == hipSuccess ? PS_OK : PS_ERR_HIP;
}

int dit_profile_enable(dit* d, int on) {
    if (!d) return PS_ERR_NULL;
    if (on < 0 || on > 2) return PS_ERR_SHAPE;
    d->profiling = on;
    if (on) {
        d->ev_used = 0;
        for (int k = 0; k < N_CLASSES; ++k) { d->prof_ms[k] = 0; d->prof_n[k] = 0; }
    }
    return PS_OK;
}

int dit_profile_read(dit* d, double* ms_out, int64_t* launches_out) {
    if (!d || !ms_out || !launches_out) return PS_ERR_NULL;
    for (size_t i = 0; i + 1 < d->ev_used; i += 2) {
        if (hipEventSynchronize(d->ev[i + 1]) != hipSuccess) return PS_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, d->ev[i], d->ev[i + 1]) != hipSuccess) return PS_ERR_HIP;
        int cls = d->ev_class[i / 2];
        d->prof_ms[cls] += ms;
        d->prof_n[cls] += 1;
    }
    d->ev_used = 0;
    for (int k = 0; k < N_CLASSES; ++k) { ms_out[k] = d->prof_ms[k]; launches_out[k] = d->prof_n[k]; }
    return PS_OK;
}

size_t attn3d_workspace_bytes(int batch, int seq, int heads, int head_dim, int dtype) {
    if (batch < 1 || seq < 1 || heads < 1 || head_dim < 1) return 0;
    return align256(attention_workspace_bytes(dtype, batch, seq, heads, head_dim));
}

int attn3d(const void* q, const void* k, const void* v, void* o, int batch, int seq, int heads,
           int head_dim, float scale, int dtype, int kernel_path, void* workspace, size_t workspace_bytes,
           void* hip_stream) {
    if (!q || !k || !v || !o) return PS_ERR_NULL;
    if (dtype != PS_F32 && dtype != PS_BF16) return PS_ERR_DTYPE;
    if (!kernel_path_valid(kernel_path)) return PS_ERR_SHAPE;
    if (batch < 1 || seq < 1 || heads < 1) return PS_ERR_SHAPE;
    if (head_dim != 16 && head_dim != 32 && head_dim != 64) return PS_ERR_SHAPE;
    if (batch > 65535 || heads > 65535 || seq > (1 << 24)) return PS_ERR_SHAPE;
    if (!(scale > 0.f) || !std::isfinite(scale)) return PS_ERR_SHAPE;
    if (o == q || o == k || o == v) return PS_ERR_SHAPE;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16)) return PS_ERR_SHAPE;
    size_t need = attn3d_workspace_bytes(batch, seq, heads, head_dim, dtype);
    if (need > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < need)) return PS_ERR_WORKSPACE;
    AttnStrides s;
    s.q_tok = s.k_tok = s.v_tok = s.o_tok = (long)heads * head_dim;
    s.q_head = s.k_head = s.v_head = s.o_head = head_dim;
    s.q_batch = s.k_batch = s.v_batch = s.o_batch = (long)seq * heads * head_dim;
    hipError_t e = launch_attention(dtype, q, k, v, o, batch, seq, heads, head_dim, scale, s,
                                    need ? workspace : nullptr, kernel_path, (hipStream_t)hip_stream);
    return e == hipSuccess ? PS_OK : PS_ERR_HIP;
}

size_t dit_linear_workspace_bytes(int m, int n_out, int k, int dtype, int kernel_path) {
    if (m < 1 || n_out < 2 || k < 8 || (dtype != PS_F32 && dtype != PS_BF16) || !kernel_path_valid(kernel_path)) return 0;
    return align256(gemm_split_workspace_bytes(dtype, 1, m, n_out, k, kernel_path));
}

int dit_linear(const void* a, const void* w, const float* bias, void* out, int m, int n_out, int k, int act,
               int dtype, int kernel_path, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!a || !w || !bias || !out) return PS_ERR_NULL;
    if (dtype != PS_F32 && dtype != PS_BF16) return PS_ERR_DTYPE;
    if (!kernel_path_valid(kernel_path)) return PS_ERR_SHAPE;
    if (m < 1 || n_out < 2 || k < 8 || (n_out & 1) || (k % 8) || (act != 0 && act != 1)) return PS_ERR_SHAPE;
    if (!aligned(a, 16) || !aligned(w, 16) || !aligned(out, 16) || !aligned(bias, 16) || out == a || out == w)
        return PS_ERR_SHAPE;
    if (workspace && !aligned(workspace, 256)) return PS_ERR_WORKSPACE;
    // a bf16 shape that belongs to the MFMA kernel but whose output exceeds its 32-bit offsets is refused, not
    // handed to the slow generic kernel
    if (dtype == PS_BF16 && (kernel_path & 0xff) != 1 && k % 64 == 0 && n_out % 4 == 0 && n_out >= 64 &&
        (long)m * n_out >= (1L << 31))
        return PS_ERR_SHAPE;
    Epilogue ep{};
    ep.kind = act ? EPI_BIAS_GELU : EPI_BIAS;
    ep.bias = bias;
    ep.geom = TokenGeom{m, 0};
    ep.split_ws = (float*)workspace;                 // used only if large enough for the shape's split
    ep.split_ws_bytes = workspace ? workspace_bytes : 0;
    hipError_t e = launch_gemm(dtype, a, w, out, 1, m, n_out, k, ep, kernel_path, (hipStream_t)hip_stream);
    return e == hipSuccess ? PS_OK : PS_ERR_HIP;
}

size_t sampler_step_workspace_bytes(size_t n) { return align256(reduce_workspace_bytes(n)); }
size_t rel_mae_workspace_bytes(size_t n) { return align256(reduce_workspace_bytes(n)); }

int sampler_step(const float* x, const float* eps, const float* eps_prev, float* x_out, double a, double b,
                 size_t n, float* sums4, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n > 0 && (!x || !eps || !x_out)) return PS_ERR_NULL;      // an empty input has nothing to point at
    if (!aligned(x, 16) || !aligned(eps, 16) || !aligned(x_out, 16) || (eps_prev && !aligned(eps_prev, 16)))
        return PS_ERR_SHAPE;
    if (n > 0 && (eps == x_out || (eps_prev && eps_prev == x_out))) return PS_ERR_SHAPE;
    if (sums4 && (!workspace || !aligned(workspace, 256) || workspace_bytes < sampler_step_workspace_bytes(n)))
        return PS_ERR_WORKSPACE;
    hipError_t e = launch_sampler_step(x, eps, eps_prev, x_out, a, b, n, sums4, workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? PS_OK : PS_ERR_HIP;
}

int sampler_step_noalloc(const float* x, const float* eps, const float* eps_prev, float* x_out, double a, double b,
                         size_t n, float* sums4, void* hip_stream) {
    if (n > SAMPLER_STEP_NOALLOC_MAX_N) return PS_ERR_SHAPE;
    if (n > 0 && (!x || !eps || !x_out)) return PS_ERR_NULL;
    if (!aligned(x, 16) || !aligned(eps, 16) || !aligned(x_out, 16) || (eps_prev && !aligned(eps_prev, 16)))
        return PS_ERR_SHAPE;
    if (n > 0 && (eps == x_out || (eps_prev && eps_prev == x_out))) return PS_ERR_SHAPE;
    hipError_t e = launch_sampler_step_static(x, eps, eps_prev, x_out, a, b, n, sums4, (hipStream_t)hip_stream);
    return e == hipSuccess ? PS_OK : PS_ERR_HIP;
}

int rel_mae(const float* a, const float* b, size_t n, float* out3, void* workspace, size_t workspace_bytes,
            void* hip_stream) {
    if (!out3 || (n > 0 && (!a || !b))) return PS_ERR_NULL;
    if (!aligned(a, 16) || !aligned(b, 16)) return PS_ERR_SHAPE;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < rel_mae_workspace_bytes(n)) return PS_ERR_WORKSPACE;
    hipError_t e = launch_rel_mae(a, b, n, out3, workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? PS_OK : PS_ERR_HIP;
}

int ddim_coefficients(int train_steps, double beta_start, double beta_end, int steps, int32_t* timesteps_out,
                      double* a_out, double* b_out) {
    if (!timesteps_out || !a_out || !b_out) return PS_ERR_NULL;
    if (train_steps < 2 || steps < 1 || steps > train_steps) return PS_ERR_SCHEDULE;
    if (!(beta_start > 0.0) || !(beta_end >= beta_start) || !(beta_end < 1.0)) return PS_ERR_SCHEDULE;
    std::vector<double> abar(train_steps);
    double prod = 1.0;
    for (int k = 0; k < train_steps; ++k) {
        double beta = beta_start + (double)k * (beta_end - beta_start) / (double)(train_steps - 1);
        prod *= 1.0 - beta;
        abar[k] = prod;
    }
    int stride = train_steps / steps;
    for (int i = 0; i < steps; ++i) {
        int tau = (steps - 1 - i) * stride;
        double ab_t = abar[tau];
        double ab_p = i + 1 < steps ? abar[(steps - 2 - i) * stride] : 1.0;
        double a = std::sqrt(ab_p / ab_t);
        double b = std::sqrt(1.0 - ab_p) - a * std::sqrt(1.0 - ab_t);
        timesteps_out[i] = tau;
        a_out[i] = a;
        b_out[i] = b;
    }
    return PS_OK;
}

int euler_discrete_coefficients(int train_steps, double beta_start, double beta_end, int steps,
                                int32_t* timesteps_out, double* a_out, double* b_out) {
    if (!timesteps_out || !a_out || !b_out) return PS_ERR_NULL;
    if (train_steps < 2 || steps < 1 || steps > train_steps) return PS_ERR_SCHEDULE;
    if (!(beta_start > 0.0) || !(beta_end >= beta_start) || !(beta_end < 1.0)) return PS_ERR_SCHEDULE;
    std::vector<double> sigma(train_steps);
    double prod = 1.0;
    for (int k = 0; k < train_steps; ++k) {
        double beta = beta_start + (double)k * (beta_end - beta_start) / (double)(train_steps - 1);
        prod *= 1.0 - beta;
        sigma[k] = std::sqrt((1.0 - prod) / prod);
    }
    int stride = train_steps / steps;
    for (int i = 0; i < steps; ++i) {
        int tau = (steps - 1 - i) * stride;
        double s_next = i + 1 < steps ? sigma[(steps - 2 - i) * stride] : 0.0;
        timesteps_out[i] = tau;
        a_out[i] = 1.0;
        b_out[i] = s_next - sigma[tau];
    }
    return PS_OK;
}

int flow_euler_coefficients(int train_steps, int steps, int32_t* timesteps_out, double* a_out, double* b_out) {
    if (!timesteps_out || !a_out || !b_out) return PS_ERR_NULL;
    if (train_steps < 2 || steps < 1 || steps > train_steps) return PS_ERR_SCHEDULE;
    for (int i = 0; i < steps; ++i) {
        timesteps_out[i] = (int32_t)(((long)i * train_steps) / steps);
        a_out[i] = 1.0;
        b_out[i] = 1.0 / (double)steps;
    }
    return PS_OK;
}

}  // extern "C"

// ----------------------------------------------------------------- reuse-then-predict run
namespace {

struct RunPlan {
    std::vector<int> cycles;   // cycle lengths actually entered after warm-up
    int pmax = 1;
    int warm = 0;
};

int plan_schedule(const sampler_schedule* s, RunPlan* plan) {
    if (!s) return PS_ERR_NULL;
    if (s->steps < 1 || !s->timesteps || !s->coef_a || !s->coef_b) return s->steps < 1 ? PS_ERR_SCHEDULE : PS_ERR_NULL;
    if (s->warmup < 0 || (s->mode < 0 || s->mode > 2) || (s->batched != 0 && s->batched != 1)) return PS_ERR_SCHEDULE;
    if (s->batched && s->mode == 1) return PS_ERR_SCHEDULE;
    for (int i = 0; i < s->steps; ++i) {
        if (s->timesteps[i] < 0 || s->timesteps[i] >= 100000) return PS_ERR_SCHEDULE;
        if (i > 0 && s->timesteps[i] == s->timesteps[i - 1]) return PS_ERR_SCHEDULE;
        if (i > 1 && (s->timesteps[i] > s->timesteps[i - 1]) != (s->timesteps[1] > s->timesteps[0]))
            return PS_ERR_SCHEDULE;                           // strictly monotonic, either way
    }
    plan->warm = s->warmup < s->steps ? s->warmup : s->steps;
    int left = s->steps - plan->warm;
    plan->pmax = 1;
    if (left > 0) {
        if (s->n_cycles < 1 || !s->cycle_len) return PS_ERR_SCHEDULE;
        for (int c = 0; c < s->n_cycles && left > 0; ++c) {
            int p = s->cycle_len[c];
            if (p < 1 || p > MAX_BATCH) return PS_ERR_SCHEDULE;
            plan->cycles.push_back(p);
            if (p > plan->pmax) plan->pmax = p;
            left -= p;
        }
        if (left > 0) return PS_ERR_SCHEDULE;                 // cycles do not cover the run
        if (plan->pmax > 1 && s->warmup < 1) return PS_ERR_SCHEDULE;   // eps_cache undefined
    }
    return PS_OK;
}

// [per-rank samples | per-rank eps_cache | two eps buffers] is the state a run carries from step to step
// (Algorithm 1: x and eps_cache of every rank, plus the eps of the last step for the adjacent-step sums);
// everything after `state_end` is scratch.
struct RunWs { size_t xbuf, cache, pp, state_end, xb, eb, red, dit, total; };

RunWs run_layout(const dit* d, const sampler_schedule* s, const RunPlan& plan) {
    size_t n = (size_t)d->cfg.in_channels * d->cfg.frames * d->cfg.height * d->cfg.width;
    size_t nb = align256(n * 4);
    RunWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    int p = plan.pmax;
    w.xbuf = take(nb * p);        // per-rank samples (rank 0 = true trajectory)
    w.cache = take(nb * p);       // per-rank eps_cache
    w.pp = take(nb * 2);          // ping-pong eps buffers / eps_prev copy
    w.state_end = off;
    w.xb = take(s->batched ? nb * p : 0);
    w.eb = take(s->batched ? nb * p : 0);
    w.red = take(reduce_workspace_bytes(n));
    w.dit = take(dit_workspace_bytes(d, s->batched ? p : 1));
    w.total = off;
    return w;
}

// (cycle, round) at which step `step` runs; false if `step` lies inside warm-up (then both are 0)
bool position_of(const RunPlan& plan, int step, int* cyc, int* rnd) {
    *cyc = 0; *rnd = 0;
    if (step < plan.warm) return false;
    int left = step - plan.warm;
    size_t c = 0;
    while (c < plan.cycles.size() && left >= plan.cycles[c]) { left -= plan.cycles[c]; ++c; }
    *cyc = (int)c; *rnd = left;
    return true;
}

}  // namespace

extern "C" {

size_t sampler_workspace_bytes(const dit* d, const sampler_schedule* s) {
    RunPlan plan;
    if (!d || plan_schedule(s, &plan) != PS_OK) return 0;
    return run_layout(d, s, plan).total;
}

size_t sampler_state_bytes(const dit* d, const sampler_schedule* s) {
    RunPlan plan;
    if (!d || plan_schedule(s, &plan) != PS_OK) return 0;
    return run_layout(d, s, plan).state_end;
}

int sampler_run_steps(dit* d, const sampler_schedule* s, sampler_state* state, int stop_step, const float* x_T,
                      const void* ctx, float* x_out, float* step_sums, float* trajectory_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    if (!d || !s || !state) return PS_ERR_NULL;
    if (d->cfg.text_tokens > 0 && !ctx) return PS_ERR_NULL;
    RunPlan plan;
    int rc = plan_schedule(s, &plan);
    if (rc != PS_OK) return rc;
    const int P = plan.pmax;
    const bool fresh = state->step == 0;
    if (fresh && !x_T) return PS_ERR_NULL;
    if (state->step < 0 || state->step >= s->steps || stop_step <= state->step || stop_step > s->steps)
        return PS_ERR_SCHEDULE;
    if ((x_T && !aligned(x_T, 16)) || (x_out && !aligned(x_out, 16)) || (step_sums && !aligned(step_sums, 16)))
        return PS_ERR_SHAPE;
    if (trajectory_out && (!aligned(trajectory_out, 16) || trajectory_out == x_T || trajectory_out == x_out))
        return PS_ERR_SHAPE;
    int cyc = 0, rnd = 0;
    position_of(plan, state->step, &cyc, &rnd);
    if (!fresh) {
        // a state that does not belong to this schedule is an error, not a different run
        if (state->cycle != cyc || state->round != rnd || (state->toggle != 0 && state->toggle != 1)) return PS_ERR_SCHEDULE;
        if (state->eps_prev < 0 || state->eps_prev >= 2 + P || state->calls < 0) return PS_ERR_SCHEDULE;
        for (int r = 0; r < P; ++r)
            if (state->src[r] != 0 && state->src[r] != r) return PS_ERR_SCHEDULE;
    }
    if (s->batched) {               // a cycle is one predictor call: a run can only pause between cycles
        int c2, r2;
        if (position_of(plan, state->step, &c2, &r2) && r2 != 0) return PS_ERR_SCHEDULE;
        if (stop_step < s->steps && position_of(plan, stop_step, &c2, &r2) && r2 != 0) return PS_ERR_SCHEDULE;
    }
    RunWs w = run_layout(d, s, plan);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < w.total) return PS_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)hip_stream;
    const size_t n = (size_t)d->cfg.in_channels * d->cfg.frames * d->cfg.height * d->cfg.width;
    const size_t nb = align256(n * 4);
    char* base = (char*)workspace;
    auto xbuf = [&](int r) { return (float*)(base + w.xbuf + nb * r); };
    // mode 2 (latest eps): every rank reuses the eps applied in the step before the cycle;
    // it is kept in slot 0, which Algorithm 1 never reads (rank 0 has no reuse update)
    const bool latest = s->mode == 2;
    auto cache = [&](int r) { return (float*)(base + w.cache + nb * (latest ? 0 : r)); };
    auto pp = [&](int i) { return (float*)(base + w.pp + nb * i); };
    auto xb = [&](int r) { return (float*)(base + w.xb + n * 4 * r); };     // contiguous [p, n]
    auto eb = [&](int r) { return (float*)(base + w.eb + n * 4 * r); };
    void* red = base + w.red;
    void* dws = base + w.dit;

    auto step = [&](const float* x, const float* e, const float* eprev, float* xo, int i, bool record) -> int {
        float* sums = (record && step_sums) ? step_sums + 4 * (size_t)i : nullptr;
        hipError_t err = launch_sampler_step(x, e, eprev, xo, s->coef_a[i], s->coef_b[i], n, sums, red, st);
        if (err == hipSuccess && record && trajectory_out)       // rank 0's sample after step i
            err = hipMemcpyAsync(trajectory_out + (size_t)i * n, xo, n * 4, hipMemcpyDeviceToDevice, st);
        return err == hipSuccess ? PS_OK : PS_ERR_HIP;
    };
    auto copy = [&](float* dst, const float* src) -> int {
        if (dst == src) return PS_OK;
        return hipMemcpyAsync(dst, src, n * 4, hipMemcpyDeviceToDevice, st) == hipSuccess ? PS_OK : PS_ERR_HIP;
    };
#define PS_RC(expr) do { int rc__ = (expr); if (rc__ != PS_OK) return rc__; } while (0)

    // the eps of the last step: nowhere yet (-1), eps buffer 0 / 1, or rank r's cache (2 + r)
    auto eps_at = [&](int code) -> float* { return code < 0 ? nullptr : code < 2 ? pp(code) : cache(code - 2); };
    int calls = fresh ? 0 : state->calls;
    int eprev_code = fresh ? -1 : state->eps_prev;
    int toggle = fresh ? 0 : state->toggle;
    std::vector<int> src(P, 0);
    if (!fresh) for (int r = 0; r < P; ++r) src[r] = state->src[r];
    if (fresh) PS_RC(copy(xbuf(0), x_T));
    int i = state->step;

    if (!s->batched) {
        // rank r's current sample lives in xbuf[src[r]] (after a broadcast every rank reads
        // rank 0's buffer until its next own update)
        for (; i < stop_step; ++i) {
            int32_t t = s->timesteps[i];
            const float* eprev = eps_at(eprev_code);
            if (i < plan.warm) {
                const int ecode = toggle;
                float* e = pp(toggle); toggle ^= 1;
                PS_RC(forward_impl(d, xbuf(0), ctx, &t, e, 1, dws, st)); ++calls;
                PS_RC(step(xbuf(0), e, eprev, xbuf(0), i, true));
                eprev_code = ecode;
                if (i == plan.warm - 1) {                                   // eps_cache of every rank
                    if (latest) PS_RC(copy(cache(0), e));
                    else for (int r = 1; r < P; ++r) PS_RC(copy(cache(r), e));
                }
                continue;
            }
            const int p = plan.cycles[cyc];
            if (s->mode == 1) {                      // direct reuse: predict only in round 0
                const float* e = eprev;
                if (rnd == 0) {
                    const int ecode = toggle;
                    float* en = pp(toggle); toggle ^= 1;
                    PS_RC(forward_impl(d, xbuf(0), ctx, &t, en, 1, dws, st)); ++calls;
                    e = en;
                    eprev_code = ecode;
                }
                PS_RC(step(xbuf(0), e, eprev, xbuf(0), i, true));
            } else {
                const int master = rnd;
                float* e;
                int ecode;
                if (master == 0 || latest) { ecode = toggle; e = pp(toggle); toggle ^= 1; }
                else { ecode = 2 + master; e = cache(master); }
                PS_RC(forward_impl(d, xbuf(src[master]), ctx, &t, e, 1, dws, st)); ++calls;
                // ranks that still have to predict in this cycle advance with their own cache;
                // they may read rank 0's buffer, so they go before rank 0's in-place update
                for (int r = master + 1; r < p; ++r) {
                    PS_RC(step(xbuf(src[r]), cache(r), nullptr, xbuf(r), i, false));
                    src[r] = r;
                }
                PS_RC(step(xbuf(0), e, eprev, xbuf(0), i, true));   // rank 0 applies the master's eps
                eprev_code = ecode;
            }
            if (rnd == p - 1) {                      // broadcast rank 0's sample
                for (int r = 1; r < P; ++r) src[r] = 0;
                if (latest && P > 1) PS_RC(copy(cache(0), eps_at(eprev_code)));
                ++cyc; rnd = 0;
            } else {
                ++rnd;
            }
        }
    } else {
        // batched: rank 0's sample lives in xbuf(0); inputs of a cycle in xb(r); the eps of the last step in pp(0)
        float* eprev_buf = pp(0);
        int32_t tb[MAX_BATCH];
        for (; i < plan.warm && i < stop_step; ++i) {
            tb[0] = s->timesteps[i];
            PS_RC(forward_impl(d, xbuf(0), ctx, tb, eb(0), 1, dws, st)); ++calls;
            PS_RC(step(xbuf(0), eb(0), eprev_code >= 0 ? eprev_buf : nullptr, xbuf(0), i, true));
            PS_RC(copy(eprev_buf, eb(0)));
            eprev_code = 0;
            if (i == plan.warm - 1)
                for (int r = 0; r < (latest ? 1 : P); ++r) PS_RC(copy(cache(r), eb(0)));
        }
        for (; (size_t)cyc < plan.cycles.size() && i < stop_step; ++cyc) {
            int p = plan.cycles[cyc];
            int nn = p < s->steps - i ? p : s->steps - i;
            // rank r's input: the current sample advanced r times with that rank's cached eps
            PS_RC(copy(xb(0), xbuf(0)));
            for (int r = 1; r < nn; ++r) {
                PS_RC(step(xbuf(0), cache(r), nullptr, xb(r), i, false));
                for (int jj = 1; jj < r; ++jj) PS_RC(step(xb(r), cache(r), nullptr, xb(r), i + jj, false));
            }
            for (int r = 0; r < nn; ++r) tb[r] = s->timesteps[i + r];
            // the text context is shared by all ranks of the cycle
            PS_RC(forward_impl(d, xb(0), ctx, tb, eb(0), nn, dws, st, true)); ++calls;
            for (int r = 0; r < nn; ++r) {
                const float* prev = r == 0 ? (eprev_code >= 0 ? eprev_buf : nullptr) : eb(r - 1);
                PS_RC(step(xbuf(0), eb(r), prev, xbuf(0), i + r, true));
            }
            if (latest) PS_RC(copy(cache(0), eb(nn - 1)));
            else for (int r = 0; r < nn; ++r) PS_RC(copy(cache(r), eb(r)));
            PS_RC(copy(eprev_buf, eb(nn - 1)));
            eprev_code = 0;
            i += nn;
        }
        rnd = 0;
    }
    if (x_out) PS_RC(copy(x_out, xbuf(0)));
#undef PS_RC
    state->step = i;
    state->cycle = cyc;
    state->round = rnd;
    state->toggle = toggle;
    state->eps_prev = eprev_code;
    state->calls = calls;
    for (int r = 0; r < MAX_BATCH; ++r) state->src[r] = r < P ? src[r] : 0;
    return PS_OK;
}

int sampler_run(dit* d, const sampler_schedule* s, const float* x_T, const void* ctx, float* x0_out,
                float* step_sums, float* trajectory_out, int* calls_out, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
    if (!d || !s || !x_T || !x0_out) return PS_ERR_NULL;
    sampler_state state;
    memset(&state, 0, sizeof(state));
    int rc = sampler_run_steps(d, s, &state, s->steps, x_T, ctx, x0_out, step_sums, trajectory_out, workspace,
                               workspace_bytes, hip_stream);
    if (rc == PS_OK && calls_out) *calls_out = state.calls;
    return rc;
}

}  // extern "C"
