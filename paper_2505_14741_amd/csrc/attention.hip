// Full (unmasked) softmax attention over the flattened text + (frame,row,col) token axis.
//
//  * attn_generic_kernel: one thread per query row, fp32 math, any supported head_dim;
//    serves the fp32 configuration and shapes the MFMA kernel does not cover.
//  * attn_mfma_kernel: flash-style kernel for bf16, head_dim 64, on
//    v_mfma_f32_32x32x16_bf16.  It works on transposed tiles so that a lane owns a QUERY
//    column: S^T = K Q^T puts the keys of one query into one lane's accumulator
//    registers (row statistics need no cross-lane reduction beyond one 32-lane swap),
//    and those registers, converted to bf16, are directly the B operand of
//    O^T += V^T P^T.  V is consumed as V^T [head][d][key] so that its fragments, like
//    K's, are contiguous 16/8-byte LDS reads; K/V^T tiles of 64 keys are double-buffered
//    in LDS and shared by the 4 waves of a workgroup, each wave owning 64 queries.
#include "common.h"

namespace ps {

int get_kernel_path();

// ------------------------------------------------------------------------------ generic
template <typename T, int HD>
__global__ void __launch_bounds__(128)
attn_generic_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                    T* __restrict__ o, int seq, int heads, float scale, AttnStrides s) {
    constexpr int KT = 32;
    __shared__ float Ks[KT][HD];
    __shared__ float Vs[KT][HD];
    int b = blockIdx.z, h = blockIdx.y;
    int qi = blockIdx.x * blockDim.x + threadIdx.x;
    bool active = qi < seq;
    int qr = active ? qi : seq - 1;
    const T* qp = q + b * s.q_batch + (long)qr * s.q_tok + h * s.q_head;
    float qv[HD], acc[HD];
#pragma unroll
    for (int c = 0; c < HD; ++c) { qv[c] = to_f32(qp[c]) * scale; acc[c] = 0.f; }
    float m = -INFINITY, l = 0.f;
    for (int k0 = 0; k0 < seq; k0 += KT) {
        int kn = min(KT, seq - k0);
        for (int e = threadIdx.x; e < KT * HD; e += blockDim.x) {
            int r = e / HD, c = e % HD;
            int kr = k0 + r;
            float kv = 0.f, vv = 0.f;
            if (kr < seq) {
                kv = to_f32(k[b * s.k_batch + (long)kr * s.k_tok + h * s.k_head + c]);
                vv = to_f32(v[b * s.v_batch + (long)kr * s.v_tok + h * s.v_head + c]);
            }
            Ks[r][c] = kv;
            Vs[r][c] = vv;
        }
        __syncthreads();
        float sc[KT];
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < KT; ++r) {
            float d = 0.f;
#pragma unroll
            for (int c = 0; c < HD; ++c) d += qv[c] * Ks[r][c];
            sc[r] = r < kn ? d : -INFINITY;
            tmax = fmaxf(tmax, sc[r]);
        }
        float mn = fmaxf(m, tmax);
        float alpha = expf(m - mn);           // exp(-inf) = 0 on the first tile
        l *= alpha;
#pragma unroll
        for (int c = 0; c < HD; ++c) acc[c] *= alpha;
#pragma unroll
        for (int r = 0; r < KT; ++r) {
            float p = expf(sc[r] - mn);       // masked keys: exp(-inf) = 0
            l += p;
#pragma unroll
            for (int c = 0; c < HD; ++c) acc[c] += p * Vs[r][c];
        }
        m = mn;
        __syncthreads();
    }
    if (active) {
        T* op = o + b * s.o_batch + (long)qi * s.o_tok + h * s.o_head;
        float inv = 1.0f / l;
#pragma unroll
        for (int c = 0; c < HD; ++c) op[c] = from_f32<T>(acc[c] * inv);
    }
}

template <typename T>
static hipError_t launch_generic_attn(const T* q, const T* k, const T* v, T* o, int batch, int seq,
                                      int heads, int head_dim, float scale, const AttnStrides& s,
                                      hipStream_t st) {
    dim3 grid((seq + 127) / 128, heads, batch);
    switch (head_dim) {
        case 16: attn_generic_kernel<T, 16><<<grid, 128, 0, st>>>(q, k, v, o, seq, heads, scale, s); break;
        case 32: attn_generic_kernel<T, 32><<<grid, 128, 0, st>>>(q, k, v, o, seq, heads, scale, s); break;
        case 64: attn_generic_kernel<T, 64><<<grid, 128, 0, st>>>(q, k, v, o, seq, heads, scale, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// --------------------------------------------------------------------------------- MFMA
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

// V [B, seq, H, 64] (strided) -> Vt [B*H][64][npad], keys beyond seq zero-filled.
// One workgroup per (64-key tile, head, batch); transposes through LDS.
__global__ void __launch_bounds__(256)
transpose_v_kernel(const bf16_t* __restrict__ v, bf16_t* __restrict__ vt, int seq, int npad, int heads,
                   long v_tok, long v_head, long v_batch) {
    __shared__ unsigned short tile[64][66];
    int b = blockIdx.z, h = blockIdx.y, k0 = blockIdx.x * 64;
    const unsigned short* vp = reinterpret_cast<const unsigned short*>(v) + b * v_batch + h * v_head;
    for (int e = threadIdx.x; e < 64 * 64; e += 256) {
        int r = e >> 6, c = e & 63;                       // r: key, c: d
        int kr = k0 + r;
        tile[r][c] = kr < seq ? vp[(long)kr * v_tok + c] : (unsigned short)0;
    }
    __syncthreads();
    unsigned short* op = reinterpret_cast<unsigned short*>(vt) + ((long)(b * heads + h) * 64) * npad + k0;
    for (int e = threadIdx.x; e < 64 * 64; e += 256) {
        int c = e >> 6, r = e & 63;                       // c: d row of Vt, r: key
        op[(long)c * npad + r] = tile[r][c];
    }
}

__device__ __forceinline__ int swz8(int row) { return row & 7; }

template <int QT>   // 32-query column tiles per wave
__global__ void __launch_bounds__(256, 2)
attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ vt,
                 bf16_t* __restrict__ o, int seq, int npad, int heads, float scale_log2e,
                 int qblocks, AttnStrides s) {
    constexpr int HD = 64, KV = 64;
    constexpr int BQ = 4 * QT * 32;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][2][KV * 128];   // [buf][K|Vt]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    // workgroup -> (batch*head, query block); consecutive ids of one XCD walk the query
    // blocks of one head so that head's K/V^T stay in that XCD's L2
    const int total = gridDim.x;
    int id = blockIdx.x;
    {
        int per = total / 8, rem = total % 8, x = id % 8, j = id / 8;
        id = x * per + (x < rem ? x : rem) + j;
    }
    const int bh = id / qblocks, qb = id % qblocks;
    const int b = bh / heads, h = bh % heads;
    const int q0 = qb * BQ + wave * (QT * 32);

    const bf16_t* kbase = k + b * s.k_batch + h * s.k_head;
    const bf16_t* vbase = vt + (long)bh * HD * npad;

    // Q fragments (B operand of S^T = K Q^T): lane = query column, 8 consecutive d
    bf16x8_t qf[QT][4];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        int qi = q0 + t * 32 + col;
        qi = qi < seq ? qi : seq - 1;
        const bf16_t* qp = q + b * s.q_batch + (long)qi * s.q_tok + h * s.q_head;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            qf[t][ks] = *reinterpret_cast<const bf16x8_t*>(qp + ks * 16 + half * 8);
    }

    f32x16_t oacc[2][QT];
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[d][t][e] = 0.f;
    float mc[QT], lsum[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) { mc[t] = -1e30f; lsum[t] = 0.f; }

    // staging: thread -> chunk tid%8 of rows tid/8 and tid/8+32, for K and for Vt
    const int lrow = tid >> 3, lchunk = tid & 7;
    uint4 rk[2], rv[2];
    auto load_tile = [&](int kv0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int kr = kv0 + lrow + 32 * i;
            kr = kr < seq ? kr : seq - 1;
            rk[i] = *reinterpret_cast<const uint4*>(kbase + (long)kr * s.k_tok + lchunk * 8);
            rv[i] = *reinterpret_cast<const uint4*>(vbase + (long)(lrow + 32 * i) * npad + kv0 + lchunk * 8);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int r = lrow + 32 * i;
            int off = r * 128 + ((lchunk ^ swz8(r)) << 4);
            *reinterpret_cast<uint4*>(&lds[buf][0][off]) = rk[i];
            *reinterpret_cast<uint4*>(&lds[buf][1][off]) = rv[i];
        }
    };

    const int ntiles = (seq + KV - 1) / KV;
    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int j = 0; j < ntiles; ++j) {
        const int buf = j & 1;
        const int kv0 = j * KV;
        if (j + 1 < ntiles) load_tile(kv0 + KV);
        const unsigned char* lk = &lds[buf][0][0];
        const unsigned char* lv = &lds[buf][1][0];

        // S^T[key tile rt][query tile t]
        f32x16_t sacc[2][QT];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int t = 0; t < QT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) sacc[rt][t][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                int r = rt * 32 + col;
                bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(lk + r * 128 + (((ks * 2 + half) ^ swz8(r)) << 4));
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    sacc[rt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][ks], sacc[rt][t], 0, 0, 0);
            }
        }
        // mask keys beyond the sequence (last tile only)
        if (kv0 + KV > seq) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    int key = kv0 + rt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                    if (key >= seq) {
#pragma unroll
                        for (int t = 0; t < QT; ++t) sacc[rt][t][e] = -INFINITY;
                    }
                }
        }
        // online softmax, per query column
        bf16x8_t pf[QT][4];
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            float mx = sacc[0][t][0];
#pragma unroll
            for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[0][t][e]);
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[1][t][e]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            float mnew = fmaxf(mc[t], mx * scale_log2e);
            if (__any(mnew > mc[t])) {
                float alpha = __builtin_amdgcn_exp2f(mc[t] - mnew);
                lsum[t] *= alpha;
#pragma unroll
                for (int d = 0; d < 2; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[d][t][e] *= alpha;
                mc[t] = mnew;
            }
            float rs = 0.f;
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
                for (int g = 0; g < 2; ++g) {      // k16-step inside the 32-key tile
                    bf16x8_t pk;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float p = __builtin_amdgcn_exp2f(sacc[rt][t][g * 8 + e] * scale_log2e - mc[t]);
                        rs += p;
                        pk[e] = (__bf16)p;
                    }
                    pf[t][rt * 2 + g] = pk;
                }
            }
            lsum[t] += rs;
        }
        // O^T[d tile][query tile] += Vt[d tile][keys] P^T[keys][queries]
        // k-slot (half, e) of step g in key tile rt is key 32rt + 16g + 8(e/4) + 4half + e%4
#pragma unroll
        for (int st = 0; st < 4; ++st) {
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                int r = dt * 32 + col;
                const unsigned char* rowp = lv + r * 128;
                int c0 = (st * 2) ^ swz8(r), c1 = (st * 2 + 1) ^ swz8(r);
                bf16x4_t lo = *reinterpret_cast<const bf16x4_t*>(rowp + (c0 << 4) + half * 8);
                bf16x4_t hi = *reinterpret_cast<const bf16x4_t*>(rowp + (c1 << 4) + half * 8);
                bf16x8_t vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    oacc[dt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t][st], oacc[dt][t], 0, 0, 0);
            }
        }
        if (j + 1 < ntiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // finish: total row sum = both halves; O[query][d] = O^T / l
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        float l = lsum[t] + __shfl_xor(lsum[t], 32, 64);
        float inv = 1.0f / l;
        int qi = q0 + t * 32 + col;
        if (qi < seq) {
            bf16_t* op = o + b * s.o_batch + (long)qi * s.o_tok + h * s.o_head;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4_t w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[dt][t][g * 4 + e] * inv);
                    *reinterpret_cast<bf16x4_t*>(op + dt * 32 + g * 8 + half * 4) = w;
                }
        }
    }
}

size_t attention_workspace_bytes(int dtype, int batch, int seq, int heads, int head_dim) {
    if (dtype != PS_BF16 || head_dim != 64) return 0;
    size_t npad = ((size_t)seq + 63) / 64 * 64;
    return (size_t)batch * heads * 64 * npad * sizeof(bf16_t);
}

hipError_t launch_attention(int dtype, const void* q, const void* k, const void* v, void* o,
                            int batch, int seq, int heads, int head_dim, float scale,
                            const AttnStrides& s, void* ws, hipStream_t st) {
    if (dtype == PS_BF16 && head_dim == 64 && get_kernel_path() == 0 && ws != nullptr) {
        int npad = (seq + 63) / 64 * 64;
        bf16_t* vt = (bf16_t*)ws;
        dim3 tg(npad / 64, heads, batch);
        transpose_v_kernel<<<tg, 256, 0, st>>>((const bf16_t*)v, vt, seq, npad, heads, s.v_tok, s.v_head, s.v_batch);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
        constexpr int QT = 2;
        constexpr int BQ = 4 * QT * 32;
        int qblocks = (seq + BQ - 1) / BQ;
        dim3 grid(qblocks * heads * batch);
        attn_mfma_kernel<QT><<<grid, 256, 0, st>>>((const bf16_t*)q, (const bf16_t*)k, vt, (bf16_t*)o, seq, npad,
                                                   heads, scale * 1.4426950408889634f, qblocks, s);
        return hipGetLastError();
    }
    if (dtype == PS_BF16)
        return launch_generic_attn<bf16_t>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, batch,
                                           seq, heads, head_dim, scale, s, st);
    return launch_generic_attn<float>((const float*)q, (const float*)k, (const float*)v, (float*)o, batch, seq,
                                      heads, head_dim, scale, s, st);
}

}  // namespace ps
