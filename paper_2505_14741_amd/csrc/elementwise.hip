// HBM-bound kernels of the denoising step: time conditioning, patch embedding,
// LayerNorm + adaLN modulation, final projection, the fused DDIM update with the
// relative-MAE sums of paper Eq. (1), and the stand-alone relative MAE.
#include "common.h"

#include <mutex>

namespace ps {

static constexpr int WAVE = 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// ------------------------------------------------------------------ time conditioning
struct TList { int t[16]; };

// s(t) = [cos(t w_j) | sin(t w_j)], w_j = 10000^(-j/(D/2)); double precision because
// t*w reaches ~1e3 rad and the result feeds an fp32 MLP compared at 1e-4.
__global__ void sinusoid_kernel(TList tl, float* __restrict__ out, int D) {
    int b = blockIdx.y;
    int half = D / 2;
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= half) return;
    double w = exp(-(double)j / (double)half * 9.210340371976184);   // ln(10000)
    double ang = (double)tl.t[b] * w;
    out[(long)b * D + j] = (float)cos(ang);
    out[(long)b * D + half + j] = (float)sin(ang);
}

hipError_t launch_sinusoid(const int32_t* t_host, float* out, int batch, int D, hipStream_t st) {
    TList tl;
    for (int i = 0; i < 16; ++i) tl.t[i] = i < batch ? t_host[i] : 0;
    dim3 grid((D / 2 + 127) / 128, batch);
    sinusoid_kernel<<<grid, 128, 0, st>>>(tl, out, D);
    return hipGetLastError();
}

// One wave per GEMV_ROWS consecutive output rows (8 for a single input vector, 4 for batches); weights stream once from HBM (16 bytes per lane and load when
// the row length allows, the loads of the wave's rows in flight together), inputs stay in cache and are read once
// for the wave's rows.  Each row's sum is formed as if the wave had that row alone (same lanes, same order).
// blockIdx.y picks one of up to GEMV_SET matrices of the same shape applied to the same input (the modulation
// matrices of all layers in one launch).
template <typename T, int MAXB, int GEMV_ROWS>
__global__ void gemv_kernel(GemvSet set, const float* __restrict__ in, int rows,
                            int cols, int batch, long in_bs, long out_bs, int act) {
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const int lane = threadIdx.x % WAVE;
    const int row0 = wave * GEMV_ROWS;
    if (row0 >= rows) return;
    const T* __restrict__ W = static_cast<const T*>(set.W[blockIdx.y]);
    const float* __restrict__ bias = set.bias[blockIdx.y];
    float* __restrict__ out = set.out[blockIdx.y];
    const T* w[GEMV_ROWS];
#pragma unroll
    for (int r = 0; r < GEMV_ROWS; ++r) w[r] = W + (long)min(row0 + r, rows - 1) * cols;   // rows past the end: recomputed, not stored
    float acc[GEMV_ROWS][MAXB];
#pragma unroll
    for (int r = 0; r < GEMV_ROWS; ++r)
#pragma unroll
        for (int b = 0; b < MAXB; ++b) acc[r][b] = 0.f;
    constexpr int VEC = 16 / sizeof(T);                      // elements per 16-byte load
    if (cols % VEC == 0 && in_bs % 4 == 0) {
        for (int c = lane * VEC; c < cols; c += WAVE * VEC) {
            float wv[GEMV_ROWS][VEC];
#pragma unroll
            for (int r = 0; r < GEMV_ROWS; ++r) {
                if constexpr (sizeof(T) == 2) {
                    typedef __attribute__((ext_vector_type(8))) __bf16 b8;
                    const b8 v = *reinterpret_cast<const b8*>(w[r] + c);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) wv[r][e] = (float)v[e];
                } else {
                    const float4 v = *reinterpret_cast<const float4*>(w[r] + c);
                    wv[r][0] = v.x; wv[r][1] = v.y; wv[r][2] = v.z; wv[r][3] = v.w;
                }
            }
#pragma unroll
            for (int b = 0; b < MAXB; ++b) {
                if (b < batch) {
                    const float* ip = in + b * in_bs + c;
#pragma unroll
                    for (int e4 = 0; e4 < VEC; e4 += 4) {
                        const float4 x = *reinterpret_cast<const float4*>(ip + e4);
#pragma unroll
                        for (int r = 0; r < GEMV_ROWS; ++r)
                            acc[r][b] += (wv[r][e4] * x.x + wv[r][e4 + 1] * x.y) + (wv[r][e4 + 2] * x.z + wv[r][e4 + 3] * x.w);
                    }
                }
            }
        }
    } else {
        for (int c = lane; c < cols; c += WAVE) {
#pragma unroll
            for (int r = 0; r < GEMV_ROWS; ++r) {
                const float wv = to_f32(w[r][c]);
#pragma unroll
                for (int b = 0; b < MAXB; ++b)
                    if (b < batch) acc[r][b] += wv * in[b * in_bs + c];
            }
        }
    }
#pragma unroll
    for (int r = 0; r < GEMV_ROWS; ++r) {
        if (row0 + r >= rows) break;
#pragma unroll
        for (int b = 0; b < MAXB; ++b) {
            if (b < batch) {
                float v = wave_sum(acc[r][b]);
                if (lane == 0) {
                    v += bias[row0 + r];
                    if (act == 1) v = silu_f(v);
                    out[b * out_bs + row0 + r] = v;
                }
            }
        }
    }
}

hipError_t launch_gemv_set(int dtype, const GemvSet& set, int count, const float* in, int rows, int cols, int batch,
                           long in_bs, long out_bs, int act, hipStream_t st) {
    if (count < 1 || count > GEMV_SET) return hipErrorInvalidValue;
    int threads = 256;
    auto go = [&](auto kernel, int rows_per_wave) {
        const int per_block = (threads / WAVE) * rows_per_wave;
        dim3 blocks((rows + per_block - 1) / per_block, count);
        kernel<<<blocks, threads, 0, st>>>(set, in, rows, cols, batch, in_bs, out_bs, act);
    };
    if (batch < 1 || batch > 16) return hipErrorInvalidValue;
    if (dtype == PS_BF16) {
        if (batch == 1) go(gemv_kernel<bf16_t, 1, 8>, 8);
        else if (batch <= 4) go(gemv_kernel<bf16_t, 4, 4>, 4);
        else go(gemv_kernel<bf16_t, 16, 4>, 4);
    } else {
        if (batch == 1) go(gemv_kernel<float, 1, 8>, 8);
        else if (batch <= 4) go(gemv_kernel<float, 4, 4>, 4);
        else go(gemv_kernel<float, 16, 4>, 4);
    }
    return hipGetLastError();
}

hipError_t launch_gemv(int dtype, const void* W, const float* bias, const float* in, float* out,
                       int rows, int cols, int batch, long in_bs, long out_bs, int act,
                       hipStream_t st) {
    GemvSet set{};
    set.W[0] = W; set.bias[0] = bias; set.out[0] = out;
    return launch_gemv_set(dtype, set, 1, in, rows, cols, batch, in_bs, out_bs, act, st);
}

// ------------------------------------------------------------------------- 3D RoPE table
// (cos, sin) of pos * theta^(-2m/d_A), axis widths d/4, 3d/8, 3d/8 over (frame, row, col), double precision
// angles.  The angle of a pair depends on the token only through its position on the pair's axis, so the table is
// stored per axis -- [F][d/8], [Hp][3d/16], [Wp][3d/16] entries of (cos, sin) -- about 1 KB instead of 256 bytes
// per token: the projection epilogue that rotates q and k finds it in the nearest cache.
__global__ void rope_table_kernel(float2* __restrict__ table, int F, int Hp, int Wp, int head_dim, float theta) {
    const int p0 = head_dim / 8, p1 = 3 * head_dim / 16;
    const int total = F * p0 + (Hp + Wp) * p1;
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int pos, m, dA;
    if (idx < F * p0) { pos = idx / p0; m = idx % p0; dA = 2 * p0; }
    else if (idx < F * p0 + Hp * p1) { int r = idx - F * p0; pos = r / p1; m = r % p1; dA = 2 * p1; }
    else { int r = idx - F * p0 - Hp * p1; pos = r / p1; m = r % p1; dA = 2 * p1; }
    double ang = (double)pos * exp(-2.0 * (double)m / (double)dA * log((double)theta));
    table[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

size_t rope_table_floats(int F, int Hp, int Wp, int head_dim) {
    return 2 * ((size_t)F * (head_dim / 8) + (size_t)(Hp + Wp) * (3 * head_dim / 16));
}

hipError_t launch_rope_table(float* table, int F, int Hp, int Wp, int head_dim,
                             float theta, hipStream_t st) {
    const int total = (int)(rope_table_floats(F, Hp, Wp, head_dim) / 2);
    if (total == 0) return hipSuccess;
    rope_table_kernel<<<(total + 255) / 256, 256, 0, st>>>(reinterpret_cast<float2*>(table), F, Hp, Wp, head_dim, theta);
    return hipGetLastError();
}

// ------------------------------------------------------------------------ patch embedding
// X[b, L_txt + (f,i,j), :] = W_pe . patch(c,dy,dx) + b_pe ; X[b, n < L_txt, :] = ctx[b, n, :].
// One workgroup per TOK tokens; patch vectors staged in LDS, threads stride over D.
template <typename T, int TOK>
__global__ void patch_embed_kernel(const float* __restrict__ x, const T* __restrict__ ctx,
                                   const T* __restrict__ W_pe, const float* __restrict__ b_pe,
                                   float* __restrict__ X, int C, int F, int H, int Wd, int patch,
                                   int text_tokens, int D, long ctx_bs) {
    extern __shared__ float pv[];        // [P][TOK]: the TOK values one weight multiplies are contiguous
    int Hp = H / patch, Wp = Wd / patch;
    int Nv = F * Hp * Wp;
    int N = text_tokens + Nv;
    int P = C * patch * patch;
    int b = blockIdx.y;
    int tok0 = blockIdx.x * TOK;         // token index within the sample (text first)
    for (int e = threadIdx.x; e < TOK * P; e += blockDim.x) {
        int tl = e / P, pi = e % P;
        int n = tok0 + tl;
        float val = 0.f;
        if (n < N && n >= text_tokens) {
            int nv = n - text_tokens;
            int j = nv % Wp, i = (nv / Wp) % Hp, f = nv / (Wp * Hp);
            int dx = pi % patch, dy = (pi / patch) % patch, c = pi / (patch * patch);
            val = x[((((long)b * C + c) * F + f) * H + (i * patch + dy)) * Wd + (j * patch + dx)];
        }
        pv[pi * TOK + tl] = val;
    }
    __syncthreads();
    for (int col = threadIdx.x; col < D; col += blockDim.x) {
        float acc[TOK];
#pragma unroll
        for (int tl = 0; tl < TOK; ++tl) acc[tl] = b_pe[col];
        const T* w = W_pe + (long)col * P;
        int pi = 0;
        if ((P & 7) == 0 && (reinterpret_cast<size_t>(W_pe) & 15) == 0) {   // rows of W_pe start 16-byte aligned: 8 weights per load
            for (; pi < P; pi += 8) {
                float wv[8];
                if constexpr (sizeof(T) == 2) {
                    union { uint4 u; bf16_t h[8]; } pk;
                    pk.u = *reinterpret_cast<const uint4*>(w + pi);
#pragma unroll
                    for (int k = 0; k < 8; ++k) wv[k] = to_f32(pk.h[k]);
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) wv[k] = to_f32(w[pi + k]);
                }
#pragma unroll
                for (int k = 0; k < 8; ++k)              // same order of additions as the one-by-one loop
#pragma unroll
                    for (int tl = 0; tl < TOK; ++tl) acc[tl] += wv[k] * pv[(pi + k) * TOK + tl];
            }
        }
        for (; pi < P; ++pi) {
            float wv = to_f32(w[pi]);
#pragma unroll
            for (int tl = 0; tl < TOK; ++tl) acc[tl] += wv * pv[pi * TOK + tl];
        }
#pragma unroll
        for (int tl = 0; tl < TOK; ++tl) {
            int n = tok0 + tl;
            if (n >= N) continue;
            float v = n < text_tokens ? to_f32(ctx[b * ctx_bs + (long)n * D + col]) : acc[tl];
            X[((long)b * N + n) * D + col] = v;
        }
    }
}

hipError_t launch_patch_embed(int dtype, const float* x, const void* ctx, const void* W_pe,
                              const float* b_pe, float* X, int batch, int C, int F, int H, int Wd,
                              int patch, int text_tokens, int D, long ctx_bs, hipStream_t st) {
    constexpr int TOK = 16;
    int N = text_tokens + F * (H / patch) * (Wd / patch);
    int P = C * patch * patch;
    dim3 grid((N + TOK - 1) / TOK, batch);
    size_t sh = (size_t)TOK * P * sizeof(float);
    if (dtype == PS_BF16)
        patch_embed_kernel<bf16_t, TOK><<<grid, 256, sh, st>>>(x, (const bf16_t*)ctx, (const bf16_t*)W_pe,
                                                               b_pe, X, C, F, H, Wd, patch, text_tokens, D, ctx_bs);
    else
        patch_embed_kernel<float, TOK><<<grid, 256, sh, st>>>(x, (const float*)ctx, (const float*)W_pe, b_pe,
                                                              X, C, F, H, Wd, patch, text_tokens, D, ctx_bs);
    return hipGetLastError();
}

// ------------------------------------------------------------------- LayerNorm + modulate
// One wave per token row.  fp32 statistics (mean, then centred second moment), biased
// variance, no affine; out = y*(1+scale)+shift with the text or video chunk.
// The row is held in registers between the passes: D <= 64*4*MAXV.
// (Two rows per wave, both loaded before the first reduction, measured 18 % slower at 17776 x 1920: 48 against 41 us.)
template <typename T, int MAXV>
__global__ void ln_modulate_kernel(const float* __restrict__ X, T* __restrict__ out, int M, int D,
                                   float eps, const float* __restrict__ mod_layer, long mod_bs,
                                   int shift_chunk, int scale_chunk, TokenGeom g, float* __restrict__ zero_buf,
                                   int zero_n) {
    // a few words some later kernel sets (the attention kernels' per-head flags) are cleared here
    // instead of by a launch of their own
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < zero_n; i += blockDim.x) zero_buf[i] = 0.f;
    int row = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    int lane = threadIdx.x % WAVE;
    if (row >= M) return;
    const float4* xr = reinterpret_cast<const float4*>(X + (long)row * D);
    int nvec = D / 4;
    float4 v[MAXV];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int c = lane + i * WAVE;
        if (c < nvec) {
            v[i] = xr[c];
            s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        }
    }
    float mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int c = lane + i * WAVE;
        if (c < nvec) {
            float a = v[i].x - mean, b = v[i].y - mean, cc = v[i].z - mean, d = v[i].w - mean;
            q += (a * a + b * b) + (cc * cc + d * d);
        }
    }
    float rstd = 1.0f / sqrtf(wave_sum(q) / (float)D + eps);
    int b = row / g.tokens, n = row % g.tokens;
    int off = n < g.text_tokens ? 6 : 0;
    const float4* sh = reinterpret_cast<const float4*>(mod_layer + b * mod_bs + (long)(shift_chunk + off) * D);
    const float4* sc = reinterpret_cast<const float4*>(mod_layer + b * mod_bs + (long)(scale_chunk + off) * D);
    T* orow = out + (long)row * D;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int c = lane + i * WAVE;
        if (c < nvec) {
            float4 h = sh[c], k = sc[c];
            float y0 = (v[i].x - mean) * rstd * (1.f + k.x) + h.x;
            float y1 = (v[i].y - mean) * rstd * (1.f + k.y) + h.y;
            float y2 = (v[i].z - mean) * rstd * (1.f + k.z) + h.z;
            float y3 = (v[i].w - mean) * rstd * (1.f + k.w) + h.w;
            if constexpr (sizeof(T) == 2) {
                union { bf16_t h4[4]; uint2 u; } pk;
                pk.h4[0] = __float2bfloat16(y0); pk.h4[1] = __float2bfloat16(y1);
                pk.h4[2] = __float2bfloat16(y2); pk.h4[3] = __float2bfloat16(y3);
                *reinterpret_cast<uint2*>(orow + 4 * c) = pk.u;
            } else {
                *reinterpret_cast<float4*>(orow + 4 * c) = make_float4(y0, y1, y2, y3);
            }
        }
    }
}

hipError_t launch_ln_modulate(int dtype, const float* X, void* out, int M, int D, float eps,
                              const float* mod_layer, long mod_bs, int shift_chunk, int scale_chunk,
                              TokenGeom geom, hipStream_t st, float* zero_buf, int zero_n) {
    int threads = 256;
    int blocks = (M + 3) / 4;
    if (D % 4 != 0 || D > 64 * 4 * 8) return hipErrorInvalidValue;
    if (dtype == PS_BF16)
        ln_modulate_kernel<bf16_t, 8><<<blocks, threads, 0, st>>>(X, (bf16_t*)out, M, D, eps, mod_layer, mod_bs,
                                                                 shift_chunk, scale_chunk, geom, zero_buf, zero_n);
    else
        ln_modulate_kernel<float, 8><<<blocks, threads, 0, st>>>(X, (float*)out, M, D, eps, mod_layer, mod_bs,
                                                                shift_chunk, scale_chunk, geom, zero_buf, zero_n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------ final projection
// Video tokens only: y = LN(X_n)(1+scale)+shift with modf = [shift | scale] (fp32 [B][2D]),
// out = W_out y + b_out (C*ps*ps values in (c,dy,dx) order) scattered into eps[C,F,H,W].
// One workgroup (256 threads) per token; y kept in LDS.
template <typename T>
__global__ void final_proj_kernel(const float* __restrict__ X, const float* __restrict__ modf,
                                  const T* __restrict__ W_out, const float* __restrict__ b_out,
                                  float* __restrict__ eps_out, int C, int F, int H, int Wd, int patch,
                                  int text_tokens, int D, float eps) {
    extern __shared__ float y[];     // [D] + 8 partials
    float* red = y + D;
    int Hp = H / patch, Wp = Wd / patch;
    int Nv = F * Hp * Wp, N = text_tokens + Nv;
    int b = blockIdx.y, nv = blockIdx.x;
    const float* xr = X + ((long)b * N + text_tokens + nv) * D;
    int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
    float s = 0.f;
    for (int c = threadIdx.x; c < D; c += blockDim.x) { float v = xr[c]; y[c] = v; s += v; }
    s = wave_sum(s);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < nw; ++w) tot += red[w];
    float mean = tot / (float)D;
    __syncthreads();
    float q = 0.f;
    for (int c = threadIdx.x; c < D; c += blockDim.x) { float dlt = y[c] - mean; q += dlt * dlt; }
    q = wave_sum(q);
    if (lane == 0) red[wave] = q;
    __syncthreads();
    float qt = 0.f;
    for (int w = 0; w < nw; ++w) qt += red[w];
    float rstd = 1.0f / sqrtf(qt / (float)D + eps);
    const float* shift = modf + (long)b * 2 * D;
    const float* scale = shift + D;
    for (int c = threadIdx.x; c < D; c += blockDim.x)
        y[c] = (y[c] - mean) * rstd * (1.f + scale[c]) + shift[c];
    __syncthreads();
    int P = C * patch * patch;
    int j = nv % Wp, i = (nv / Wp) % Hp, f = nv / (Wp * Hp);
    for (int o = wave; o < P; o += nw) {
        const T* w = W_out + (long)o * D;
        float acc = 0.f;
        for (int c = lane; c < D; c += WAVE) acc += to_f32(w[c]) * y[c];
        acc = wave_sum(acc);
        if (lane == 0) {
            int dx = o % patch, dy = (o / patch) % patch, c = o / (patch * patch);
            eps_out[((((long)b * C + c) * F + f) * H + (i * patch + dy)) * Wd + (j * patch + dx)] = acc + b_out[o];
        }
    }
}

hipError_t launch_final_proj(int dtype, const float* X, const float* modf, const void* W_out,
                             const float* b_out, float* eps_out, int batch, int C, int F, int H,
                             int Wd, int patch, int text_tokens, int D, float eps, hipStream_t st) {
    int Nv = F * (H / patch) * (Wd / patch);
    dim3 grid(Nv, batch);
    size_t sh = (size_t)(D + 8) * sizeof(float);
    if (dtype == PS_BF16)
        final_proj_kernel<bf16_t><<<grid, 256, sh, st>>>(X, modf, (const bf16_t*)W_out, b_out, eps_out, C, F, H,
                                                        Wd, patch, text_tokens, D, eps);
    else
        final_proj_kernel<float><<<grid, 256, sh, st>>>(X, modf, (const float*)W_out, b_out, eps_out, C, F, H, Wd,
                                                       patch, text_tokens, D, eps);
    return hipGetLastError();
}

// ------------------------------------------------- scheduler update + relative-MAE sums
// Two-stage deterministic reduction.  Stage 1 streams the tensors once with non-temporal
// 16-byte accesses.  A workgroup takes contiguous chunks of 256 x 4 float4 (16 KB of every
// tensor), each thread four float4 per tensor 4 KB apart, all loads of a chunk in flight
// before the first use; the grid has one workgroup per chunk up to 32768 (measured on MI355X
// at 2^28 elements: 6.1 TB/s for the update with sums, against 5.3 for a grid-stride walk with
// two float4 in flight and 4.3-5.0 for grids of 2048-8192 long-running workgroups); each
// workgroup leaves its partial sums in the workspace.  Stage 2 (one workgroup of 1024) adds
// the partials in a fixed order in double.
static constexpr int RED_THREADS = 256;
static constexpr int RED_MAX_BLOCKS = 32768;
static constexpr int RED_UNROLL = 4;
static constexpr size_t RED_CHUNK = (size_t)RED_THREADS * RED_UNROLL;      // float4 per workgroup step

typedef __attribute__((ext_vector_type(4))) float v4f_t;
__device__ __forceinline__ float4 stream_load(const float4* p) {
    v4f_t v = __builtin_nontemporal_load(reinterpret_cast<const v4f_t*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void stream_store(float4 r, float4* p) {
    v4f_t v = {r.x, r.y, r.z, r.w};
    __builtin_nontemporal_store(v, reinterpret_cast<v4f_t*>(p));
}
__device__ __forceinline__ float abs4(float4 v) { return (fabsf(v.x) + fabsf(v.y)) + (fabsf(v.z) + fabsf(v.w)); }
__device__ __forceinline__ float absdiff4(float4 a, float4 b) {
    return (fabsf(a.x - b.x) + fabsf(a.y - b.y)) + (fabsf(a.z - b.z) + fabsf(a.w - b.w));
}

static int red_blocks(size_t n) {
    size_t per_block = RED_CHUNK * 4;
    size_t b = (n + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > RED_MAX_BLOCKS) b = RED_MAX_BLOCKS;
    return (int)b;
}

size_t reduce_workspace_bytes(size_t n) { (void)n; return (size_t)RED_MAX_BLOCKS * 4 * sizeof(double); }

template <int NS>
__device__ __forceinline__ void block_store_partials(double (&acc)[NS], double* __restrict__ part) {
    __shared__ double sm[NS][RED_THREADS / WAVE];
    int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        double v = wave_sum_d(acc[k]);
        if (lane == 0) sm[k][wave] = v;
    }
    __syncthreads();
    if (threadIdx.x < NS) {
        double t = 0.0;
        for (int w = 0; w < RED_THREADS / WAVE; ++w) t += sm[threadIdx.x][w];
        part[(long)blockIdx.x * NS + threadIdx.x] = t;
    }
}

// stage 2: NS sums over nblocks partials with one workgroup of FIN_THREADS; thread k adds
// partials k, k+FIN_THREADS, ... (four rows in flight, added in index order) and the per-thread
// results are combined in a fixed tree, so the result does not depend on timing
static constexpr int FIN_THREADS = 1024;
template <int NS>
__device__ __forceinline__ void reduce_partials(const double* __restrict__ part, int nblocks, double (&out)[NS]) {
    __shared__ double sm2[NS][FIN_THREADS / WAVE];
    double acc[NS];
#pragma unroll
    for (int k = 0; k < NS; ++k) acc[k] = 0.0;
    int b = threadIdx.x;
    for (; b + 3 * FIN_THREADS < nblocks; b += 4 * FIN_THREADS) {
        double v[4][NS];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int k = 0; k < NS; ++k) v[u][k] = part[(long)(b + u * FIN_THREADS) * NS + k];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int k = 0; k < NS; ++k) acc[k] += v[u][k];
    }
    for (; b < nblocks; b += FIN_THREADS)
#pragma unroll
        for (int k = 0; k < NS; ++k) acc[k] += part[(long)b * NS + k];
    int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        double v = wave_sum_d(acc[k]);
        if (lane == 0) sm2[k][wave] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        double t = 0.0;
        for (int w = 0; w < FIN_THREADS / WAVE; ++w) t += sm2[k][w];
        out[k] = t;
    }
}

// increment form: d = (a-1)x + b*eps, x' = x + d (a -> 1 near the end of a run, and the sum
// of |x' - x| must not come from a difference of rounded values)
template <bool SUMS, bool PREV>
__global__ void __launch_bounds__(RED_THREADS)
sampler_step_kernel(const float* x, const float* __restrict__ e, const float* __restrict__ ep, float* xo,
                    float am1, float b, size_t n, double* __restrict__ part) {
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    const size_t nvec = n / 4;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    const float4* e4 = reinterpret_cast<const float4*>(e);
    const float4* p4 = reinterpret_cast<const float4*>(ep);
    float4* o4 = reinterpret_cast<float4*>(xo);
    auto one = [&](float4 xv, float4 ev, float4 pv, size_t i) {
        float4 dl, r;
        dl.x = am1 * xv.x + b * ev.x; dl.y = am1 * xv.y + b * ev.y;
        dl.z = am1 * xv.z + b * ev.z; dl.w = am1 * xv.w + b * ev.w;
        r.x = xv.x + dl.x; r.y = xv.y + dl.y; r.z = xv.z + dl.z; r.w = xv.w + dl.w;
        stream_store(r, o4 + i);
        if constexpr (SUMS) {
            s0 += abs4(dl); s1 += abs4(r); s3 += abs4(ev);
            if constexpr (PREV) s2 += absdiff4(ev, pv);
        }
    };
    for (size_t base = (size_t)blockIdx.x * RED_CHUNK; base < nvec; base += (size_t)gridDim.x * RED_CHUNK) {
        const size_t i = base + threadIdx.x;
        if (base + RED_CHUNK <= nvec) {
            float4 xv[RED_UNROLL], ev[RED_UNROLL], pv[RED_UNROLL];
#pragma unroll
            for (int u = 0; u < RED_UNROLL; ++u) {
                xv[u] = stream_load(x4 + i + u * RED_THREADS);
                ev[u] = stream_load(e4 + i + u * RED_THREADS);
                pv[u] = xv[u];
                if constexpr (SUMS && PREV) pv[u] = stream_load(p4 + i + u * RED_THREADS);
            }
#pragma unroll
            for (int u = 0; u < RED_UNROLL; ++u) one(xv[u], ev[u], pv[u], i + u * RED_THREADS);
        } else {
            for (int u = 0; u < RED_UNROLL; ++u) {
                const size_t j = i + u * RED_THREADS;
                if (j < nvec) {
                    float4 xa = stream_load(x4 + j), ea = stream_load(e4 + j), pa = xa;
                    if constexpr (SUMS && PREV) pa = stream_load(p4 + j);
                    one(xa, ea, pa, j);
                }
            }
        }
    }
    // ragged tail (n % 4 elements) handled by the first threads of block 0
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        size_t t = nvec * 4 + threadIdx.x;
        float xv = x[t], ev = e[t];
        float dl = am1 * xv + b * ev;
        float r = xv + dl;
        xo[t] = r;
        if constexpr (SUMS) {
            s0 += fabsf(dl); s1 += fabsf(r); s3 += fabsf(ev);
            if constexpr (PREV) s2 += fabsf(ev - ep[t]);
        }
    }
    if constexpr (SUMS) {
        // a thread adds at most n / (4 * grid * 256) + 1 float4 per sum in fp32 (a few dozen
        // terms at any size the grid cap allows below 2^32 elements), then everything is double
        double acc[4] = {(double)s0, (double)s1, (double)s2, (double)s3};
        block_store_partials<4>(acc, part);
    }
}

__global__ void __launch_bounds__(FIN_THREADS)
finish_sums4_kernel(const double* __restrict__ part, int nblocks, float* __restrict__ out) {
    double t[4];
    reduce_partials<4>(part, nblocks, t);
    if (threadIdx.x < 4) out[threadIdx.x] = (float)t[threadIdx.x];
}

hipError_t launch_sampler_step(const float* x, const float* e, const float* e_prev, float* x_out,
                               double a, double b, size_t n, float* sums4, void* ws, hipStream_t st) {
    if (n == 0) {
        if (sums4) finish_sums4_kernel<<<1, FIN_THREADS, 0, st>>>((const double*)ws, 0, sums4);   // four zeros
        return hipGetLastError();
    }
    int blocks = red_blocks(n);
    double* part = (double*)ws;
    const float am1 = (float)(a - 1.0), bf = (float)b;
    if (!sums4)
        sampler_step_kernel<false, false><<<blocks, RED_THREADS, 0, st>>>(x, e, nullptr, x_out, am1, bf, n, nullptr);
    else if (e_prev)
        sampler_step_kernel<true, true><<<blocks, RED_THREADS, 0, st>>>(x, e, e_prev, x_out, am1, bf, n, part);
    else
        sampler_step_kernel<true, false><<<blocks, RED_THREADS, 0, st>>>(x, e, nullptr, x_out, am1, bf, n, part);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (sums4) finish_sums4_kernel<<<1, FIN_THREADS, 0, st>>>(part, blocks, sums4);
    return hipGetLastError();
}

// Partial sums of sampler_step for callers that may not allocate: a file-scope device array (1 MiB, held by
// every GPU the library runs on until the process ends) instead of a caller-supplied workspace.  In host code the
// array's name is only a stand-in; its device address is looked up once per device, with that device current, and
// kept.  Nothing in it has to start at zero: stage 1 writes the partial sums of every workgroup it launches and
// stage 2 reads exactly those.  Calls that overlap on one GPU share the array and race.
static __device__ __align__(256) double scratch[(size_t)RED_MAX_BLOCKS * 4];
static constexpr int SCRATCH_MAX_DEVICES = 64;
static double* scratch_ptr[SCRATCH_MAX_DEVICES];     // device address of `scratch` on each device (nullptr: not yet asked)
static std::mutex scratch_mutex;

hipError_t launch_sampler_step_static(const float* x, const float* e, const float* e_prev, float* x_out,
                                      double a, double b, size_t n, float* sums4, hipStream_t st) {
    double* ptr = nullptr;
    if (sums4) {
        int dev = -1;
        hipError_t err = hipGetDevice(&dev);
        if (err != hipSuccess) return err;
        if (dev < 0 || dev >= SCRATCH_MAX_DEVICES) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(scratch_mutex);
        if (scratch_ptr[dev] == nullptr) {
            void* p = nullptr;
            err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (err != hipSuccess) return err;
            if (p == nullptr) return hipErrorInvalidSymbol;
            scratch_ptr[dev] = static_cast<double*>(p);
        }
        ptr = scratch_ptr[dev];
    }
    return launch_sampler_step(x, e, e_prev, x_out, a, b, n, sums4, ptr, st);
}

__global__ void __launch_bounds__(RED_THREADS)
rel_mae_kernel(const float* __restrict__ a, const float* __restrict__ b, size_t n, double* __restrict__ part) {
    float s0 = 0.f, s1 = 0.f;
    const size_t nvec = n / 4;
    const float4* a4 = reinterpret_cast<const float4*>(a);
    const float4* b4 = reinterpret_cast<const float4*>(b);
    for (size_t base = (size_t)blockIdx.x * RED_CHUNK; base < nvec; base += (size_t)gridDim.x * RED_CHUNK) {
        const size_t i = base + threadIdx.x;
        if (base + RED_CHUNK <= nvec) {
            float4 av[RED_UNROLL], bv[RED_UNROLL];
#pragma unroll
            for (int u = 0; u < RED_UNROLL; ++u) {
                av[u] = stream_load(a4 + i + u * RED_THREADS);
                bv[u] = stream_load(b4 + i + u * RED_THREADS);
            }
#pragma unroll
            for (int u = 0; u < RED_UNROLL; ++u) { s0 += absdiff4(av[u], bv[u]); s1 += abs4(av[u]); }
        } else {
            for (int u = 0; u < RED_UNROLL; ++u) {
                const size_t j = i + u * RED_THREADS;
                if (j < nvec) {
                    float4 a0 = stream_load(a4 + j), b0 = stream_load(b4 + j);
                    s0 += absdiff4(a0, b0);
                    s1 += abs4(a0);
                }
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        size_t t = nvec * 4 + threadIdx.x;
        s0 += fabsf(a[t] - b[t]); s1 += fabsf(a[t]);
    }
    double acc[2] = {(double)s0, (double)s1};
    block_store_partials<2>(acc, part);
}

__global__ void __launch_bounds__(FIN_THREADS)
finish_rel_mae_kernel(const double* __restrict__ part, int nblocks, float* __restrict__ out3) {
    double t[2];
    reduce_partials<2>(part, nblocks, t);
    if (threadIdx.x == 0) {
        out3[0] = (float)t[0];
        out3[1] = (float)t[1];
        out3[2] = (float)(t[0] / t[1]);     // IEEE: inf or nan when the denominator is 0
    }
}

hipError_t launch_rel_mae(const float* a, const float* b, size_t n, float* out3, void* ws, hipStream_t st) {
    int blocks = n ? red_blocks(n) : 0;
    double* part = (double*)ws;
    if (blocks) {
        rel_mae_kernel<<<blocks, RED_THREADS, 0, st>>>(a, b, n, part);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    finish_rel_mae_kernel<<<1, FIN_THREADS, 0, st>>>(part, blocks, out3);
    return hipGetLastError();
}

}  // namespace ps
