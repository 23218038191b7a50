// Internal declarations shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/parastep.h"

namespace ps {

typedef __hip_bfloat16 bf16_t;

// ---- element conversion (device) ---------------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __bfloat162float(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return __float2bfloat16(v); }

__device__ __forceinline__ float gelu_tanh_f(float x) {
    const float k0 = 0.7978845608028654f, k1 = 0.044715f;
    float u = k0 * (x + k1 * x * x * x);
    return 0.5f * x * (1.0f + tanhf(u));
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

// ---- modulation addressing -----------------------------------------------------------
// mod is fp32 [B][layers][12][D]; chunks 0..5 are the video set (shift_a, scale_a,
// gate_a, shift_m, scale_m, gate_m), 6..11 the same for text tokens.
struct TokenGeom {
    int tokens;        // N = text + video tokens per sample
    int text_tokens;   // L_txt
};

// ---- GEMM epilogues ------------------------------------------------------------------
enum EpiKind { EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_GATE_RESIDUAL = 2, EPI_QKV_ROPE = 3, EPI_UNPATCHIFY = 4 };

struct PatchGeom { int C, F, H, W, patch; };   // latent [C, F, H, W], patch x patch pixels per video token

struct Epilogue {
    int kind;
    const float* bias;        // [Nn]
    // EPI_GATE_RESIDUAL: X[m, col] += gate[b, stream, col] * (acc + bias)
    float* resid;             // fp32 [M, Nn]
    const float* mod_layer;   // fp32, points at mod[0][layer][0][0]
    long mod_batch_stride;    // layers*12*D
    int gate_chunk;           // 2 (attention) or 5 (mlp); text uses +6
    int D;                    // hidden
    TokenGeom geom;
    // EPI_QKV_ROPE: rotate pairs of q and k columns of video tokens
    // rotary table, factored by axis: (cos, sin) float pairs, first [F][d/8] for the frame axis, then [Hp][3d/16]
    // for the patch row, then [Wp][3d/16] for the patch column (video token nv = (f * Hp + i) * Wp + j)
    const float* rope_cs;
    int rope_F, rope_Hp, rope_Wp;
    int head_dim;
    float q_scale;            // factor applied to the q columns (col < D) after the rotation
    // EPI_UNPATCHIFY (bf16 MFMA kernel only): columns are (c, dy, dx) of a video token's patch; rows of text
    // tokens are dropped; resid is the fp32 output latent [B, C, F, H, W]
    PatchGeom pg;
    // optional scratch for the bf16 MFMA kernel: with it, the output tiles of the last, partial round of
    // workgroups are split along K and their fp32 partial sums pass through this buffer
    float* split_ws;
    size_t split_ws_bytes;
};

// Kernel path: a per-call selector handed down from the entry points (a field of the `dit` handle, an argument of
// the stand-alone calls); nothing process-wide selects kernels.  Low byte = mode: 0 the fastest kernel for each
// shape, 1 the generic fp32-FMA kernels, 2 bf16 attention without the key split of its last partial round,
// 3 bf16 head-dim-64 attention always through the kernel that tracks a softmax reference, 4 projections whose
// last partial round is not divided along K.  Bits 8-11: tile variant of the bf16 MFMA GEMM (0 automatic,
// 1: 256x256, 2: 128x128, 3: 192x256, 4: 192x128).
constexpr int PS_PATH_MAX_VARIANT = 4;
inline bool kernel_path_valid(int path) {
    return path >= 0 && (path & ~0xfff) == 0 && (path & 0xff) <= 4 && ((path >> 8) & 0xf) <= PS_PATH_MAX_VARIANT;
}

// The M rows of a projection are `batch` samples of `tokens` rows each; every sample is tiled on its own, so a
// sample's result is bit-identical whatever batch it is computed in.
// scratch that lets launch_gemm split its last partial round along K (0: the shape does not profit)
size_t gemm_split_workspace_bytes(int dtype, int batch, int tokens, int Nn, int K, int path);
// whether launch_gemm sends a bf16 shape to the MFMA kernel (EPI_UNPATCHIFY exists only there)
bool gemm_uses_mfma(int dtype, int tokens, int Nn, int K, int path);

// ---- launchers (each validates nothing; callers have checked shapes) -----------------
// C[batch * tokens, Nn] = A[batch * tokens, K] * W[Nn, K]^T with epilogue.  A, W, C in `dtype` (C ignored for
// EPI_GATE_RESIDUAL).
hipError_t launch_gemm(int dtype, const void* A, const void* W, void* C, int batch, int tokens, int Nn, int K,
                       const Epilogue& epi, int path, hipStream_t st);

// Full attention with explicit strides (in elements) for token, head and batch.
struct AttnStrides { long q_tok, q_head, q_batch, k_tok, k_head, k_batch, v_tok, v_head, v_batch,
                     o_tok, o_head, o_batch; };
// `ws` is scratch of attention_workspace_bytes() bytes (may be NULL when that is 0).
size_t attention_workspace_bytes(int dtype, int batch, int seq, int heads, int head_dim);
// q_prescaled: q already carries scale*log2(e) (only valid when attention_uses_mfma()).
bool attention_uses_mfma(int dtype, int head_dim, int path);
// flags_cleared: the per-(batch, head) flags at the head of `ws` are already zero (see attention_head_flags()), so
// the launch that clears them is skipped.
hipError_t launch_attention(int dtype, const void* q, const void* k, const void* v, void* o,
                            int batch, int seq, int heads, int head_dim, float scale,
                            const AttnStrides& s, void* ws, int path, hipStream_t st, bool q_prescaled = false,
                            bool flags_cleared = false);
// The per-(batch, head) flag array of the bf16 head-dim-64 attention inside ws (nullptr if this shape or path has
// none); *count = its length in 4-byte words; clear: zero it with a launch of its own (else the caller zeroes it
// before the attention call, e.g. from a kernel that runs anyway).
float* attention_head_flags(int dtype, int batch, int heads, int head_dim, void* ws, int path, hipStream_t st,
                            bool clear = true, int* count = nullptr);

hipError_t launch_sinusoid(const int32_t* t_host, float* out, int batch, int D, hipStream_t st);
// out[b, r] = act(W[r,:] . in[b,:] + bias[r]);  act: 0 none, 1 SiLU.  W in dtype, in/out fp32.
// up to GEMV_SET matrices of one shape applied to one input in a single launch
constexpr int GEMV_SET = 32;
struct GemvSet { const void* W[GEMV_SET]; const float* bias[GEMV_SET]; float* out[GEMV_SET]; };
hipError_t launch_gemv_set(int dtype, const GemvSet& set, int count, const float* in, int rows, int cols, int batch,
                           long in_bs, long out_bs, int act, hipStream_t st);
// Rotary (cos, sin) of pair `pair` (0 .. d/2-1) for video token nv: which axis the pair belongs to, its index on
// that axis and the token's position on it.  Pairs 0 .. d/8-1 rotate with the frame, the next 3d/16 with the patch
// row, the last 3d/16 with the patch column.
struct RopeAxis { int base, stride, axis; };      // float offset of (position 0, this pair), floats per position
__host__ __device__ inline RopeAxis rope_axis_of(int pair, int head_dim, int F, int Hp) {
    const int p0 = head_dim / 8, p1 = 3 * head_dim / 16;
    RopeAxis r;
    if (pair < p0) { r.axis = 0; r.base = 2 * pair; r.stride = 2 * p0; }
    else if (pair < p0 + p1) { r.axis = 1; r.base = 2 * (F * p0 + (pair - p0)); r.stride = 2 * p1; }
    else { r.axis = 2; r.base = 2 * (F * p0 + Hp * p1 + (pair - p0 - p1)); r.stride = 2 * p1; }
    return r;
}
hipError_t launch_gemv(int dtype, const void* W, const float* bias, const float* in, float* out,
                       int rows, int cols, int batch, long in_bstride, long out_bstride, int act,
                       hipStream_t st);
size_t rope_table_floats(int F, int Hp, int Wp, int head_dim);
hipError_t launch_rope_table(float* table, int F, int Hp, int Wp, int head_dim,
                             float theta, hipStream_t st);
hipError_t launch_patch_embed(int dtype, const float* x, const void* ctx, const void* W_pe,
                              const float* b_pe, float* X, int batch, int C, int F, int H, int Wd,
                              int patch, int text_tokens, int D, long ctx_batch_stride,
                              hipStream_t st);
// out[m, :] = LN(X[m, :]) * (1 + scale) + shift with per-token stream selection.
hipError_t launch_ln_modulate(int dtype, const float* X, void* out, int M, int D, float eps,
                              const float* mod_layer, long mod_batch_stride, int shift_chunk,
                              int scale_chunk, TokenGeom geom, hipStream_t st, float* zero_buf = nullptr, int zero_n = 0);
hipError_t launch_final_proj(int dtype, const float* X, const float* modf, const void* W_out,
                             const float* b_out, float* eps_out, int batch, int C, int F, int H,
                             int Wd, int patch, int text_tokens, int D, float eps, hipStream_t st);

// measurement aid: a launch of nothing but bf16 MFMAs (see probe.hip)
hipError_t launch_mfma_probe(int iters, float* sink, double* flops, hipStream_t st);

size_t reduce_workspace_bytes(size_t n);
hipError_t launch_sampler_step(const float* x, const float* e, const float* e_prev, float* x_out,
                               double a, double b, size_t n, float* sums4, void* ws, hipStream_t st);
// the same update with its partial sums in a file-scope device array of the library (no workspace, no allocation)
hipError_t launch_sampler_step_static(const float* x, const float* e, const float* e_prev, float* x_out,
                                      double a, double b, size_t n, float* sums4, hipStream_t st);
hipError_t launch_rel_mae(const float* a, const float* b, size_t n, float* out3, void* ws,
                          hipStream_t st);

}  // namespace ps
