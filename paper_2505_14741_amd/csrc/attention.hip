// Full (unmasked) softmax attention over the flattened text + (frame,row,col) token axis.
//
//  * attn_generic_kernel: one thread per query row, fp32 math, any supported head_dim;
//    serves the fp32 configuration and shapes the MFMA kernel does not cover.
//  * attn_mfma_kernel: flash-style kernel for bf16, head_dim 64, on
//    v_mfma_f32_32x32x16_bf16.  It works on transposed tiles so that a lane owns a QUERY
//    column: S^T = K Q^T puts the keys of one query into one lane's accumulator
//    registers (row statistics need no cross-lane reduction beyond one 32-lane swap),
//    and those registers, converted to bf16, are directly the B operand of
//    O^T += V^T P^T.  K and V tiles of 64 keys go from global memory straight into a
//    three-stage LDS ring (global_load_lds_dwordx4), shared by the 4 waves of a
//    workgroup, each wave owning 64 queries; V stays in its natural [key][d] layout and
//    its transposed fragments come from ds_read_b64_tr_b16.
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
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(2))) int i32x2_t;

#define PS_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define PS_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives, for e = 0..3, the
// 16-bit element (i%4) of the 8 bytes addressed by lane 4*e + i/4 of the same group.
// All 16 transposed V reads of a 64-key tile are issued from one asm statement: through
// the builtin the compiler cannot tell these reads from the in-flight global->LDS loads
// of later tiles and would wait for those (vmcnt(0)) first.  The results are valid only
// after lds_wait_v_frags().
//   f[2*(2*st+dt)+0] : keys 16st + 4h + 0..3,  f[..+1] : keys 16st + 8 + 4h + 0..3
//   a0 / a1: this lane's byte address for d tile 0 / 1 (key row and swizzled slot folded in)
__device__ __forceinline__ void lds_issue_v_frags(i32x2_t (&f)[16], unsigned a0, unsigned a1) {
    asm volatile(
        "ds_read_b64_tr_b16 %0, %16 offset:0\n"
        "ds_read_b64_tr_b16 %1, %16 offset:1024\n"
        "ds_read_b64_tr_b16 %2, %17 offset:0\n"
        "ds_read_b64_tr_b16 %3, %17 offset:1024\n"
        "ds_read_b64_tr_b16 %4, %16 offset:2048\n"
        "ds_read_b64_tr_b16 %5, %16 offset:3072\n"
        "ds_read_b64_tr_b16 %6, %17 offset:2048\n"
        "ds_read_b64_tr_b16 %7, %17 offset:3072\n"
        "ds_read_b64_tr_b16 %8, %16 offset:4096\n"
        "ds_read_b64_tr_b16 %9, %16 offset:5120\n"
        "ds_read_b64_tr_b16 %10, %17 offset:4096\n"
        "ds_read_b64_tr_b16 %11, %17 offset:5120\n"
        "ds_read_b64_tr_b16 %12, %16 offset:6144\n"
        "ds_read_b64_tr_b16 %13, %16 offset:7168\n"
        "ds_read_b64_tr_b16 %14, %17 offset:6144\n"
        "ds_read_b64_tr_b16 %15, %17 offset:7168\n"
        : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&v"(f[4]), "=&v"(f[5]), "=&v"(f[6]), "=&v"(f[7]),
          "=&v"(f[8]), "=&v"(f[9]), "=&v"(f[10]), "=&v"(f[11]), "=&v"(f[12]), "=&v"(f[13]), "=&v"(f[14]),
          "=&v"(f[15])
        : "v"(a0), "v"(a1)
        : "memory");
}
__device__ __forceinline__ void lds_wait_v_frags(i32x2_t (&f)[16]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]),
                   "+v"(f[8]), "+v"(f[9]), "+v"(f[10]), "+v"(f[11]), "+v"(f[12]), "+v"(f[13]), "+v"(f[14]),
                   "+v"(f[15])
                 :
                 : "memory");
}

// max over a query's keys held by lanes l and l^32
__device__ __forceinline__ float max_across_halves(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(v), __float_as_int(v), false, false);
    return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(v), __float_as_int(v), false, false);
    return __int_as_float(r[0]) + __int_as_float(r[1]);
}

template <int QT>   // 32-query column tiles per wave
__global__ void __launch_bounds__(256, 2)
attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                 bf16_t* __restrict__ o, int seq, int heads, float scale_log2e, int qblocks, AttnStrides s) {
    constexpr int KV = 64;
    constexpr int BQ = 4 * QT * 32;
    constexpr int NST = 3;                       // LDS ring depth
    constexpr int STAGE = 2 * KV * 128;          // K tile then V tile, 128-byte rows
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    // workgroup -> (batch*head, query block); consecutive ids of one XCD walk the query
    // blocks of one head so that head's K and V stay in that XCD's L2
    int id = blockIdx.x;
    {
        int total = gridDim.x, per = total / 8, rem = total % 8, x = id % 8, j = id / 8;
        id = x * per + (x < rem ? x : rem) + j;
    }
    const int bh = id / qblocks, qb = id % qblocks;
    const int b = bh / heads, h = bh % heads;
    const int q0 = qb * BQ + wave * (QT * 32);

    const bf16_t* kbase = k + b * s.k_batch + h * s.k_head;
    const bf16_t* vbase = v + b * s.v_batch + h * s.v_head;

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

    // direct global->LDS loads: a wave instruction fills 8 rows of 128 bytes; lane j brings
    // chunk (j%8)^(j/8) of row j/8 (the XOR swizzle is applied on the global side).
    // Per stage: 8 K groups + 8 V groups; wave w takes K groups w, w+4 and V groups w, w+4.
    const int lr = lane >> 3, lc = (lane & 7) ^ lr;
    auto issue = [&](int tile, int buf) {
        unsigned char* st = lds + buf * STAGE;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int g = wave + 4 * i;
            int kr = tile * KV + g * 8 + lr;
            kr = kr < seq ? kr : seq - 1;            // rows past the end re-read the last key (masked later)
            __builtin_amdgcn_global_load_lds(PS_GLOBAL_PTR(kbase + (long)kr * s.k_tok + lc * 8),
                                             PS_LDS_PTR(st + g * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(PS_GLOBAL_PTR(vbase + (long)kr * s.v_tok + lc * 8),
                                             PS_LDS_PTR(st + KV * 128 + g * 1024), 16, 0, 0);
        }
    };

    // V^T fragment addressing for ds_read_b64_tr_b16 (see lds_read_tr16): lane l = 16g + j
    // points at key row 4*(g/2) + j/4 (+16*step, +8 for the second half of a k16-step) and
    // at d columns 16*(g%2) + 4*(j%4) .. +3 (+32 per d tile)
    const int tg = lane >> 4, tj = lane & 15;
    const int trow = 4 * (tg >> 1) + (tj >> 2);
    const int tchunk = 2 * (tg & 1) + ((tj & 3) >> 1);
    const int tsub = (tj & 1) * 8;
    // rows 16*step (+8) keep trow's low 3 bits, so the swizzled slot is the same for every
    // step; d tile 1 flips bit 2 of the slot
    const unsigned lds_base = (unsigned)(size_t)PS_LDS_PTR(lds);
    const unsigned voff0 = KV * 128 + trow * 128 + ((tchunk ^ (trow & 7)) << 4) + tsub;
    const unsigned voff1 = KV * 128 + trow * 128 + (((4 + tchunk) ^ (trow & 7)) << 4) + tsub;

    const int ntiles = (seq + KV - 1) / KV;
    issue(0, 0);
    issue(1, 1);                                   // tiles past the end are harmless re-reads
    int buf = 0;
    for (int j = 0; j < ntiles; ++j) {
        const int kv0 = j * KV;
        // tile j has landed when at most the 4 loads of tile j+1 are still in flight
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        __syncthreads();
        {
            int nb = buf + 2; nb = nb >= NST ? nb - NST : nb;
            issue(j + 2, nb);
        }
        const unsigned char* lk = lds + buf * STAGE;

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
                bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(lk + r * 128 + (((ks * 2 + half) ^ (r & 7)) << 4));
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    sacc[rt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][ks], sacc[rt][t], 0, 0, 0);
            }
        }
        // V^T fragments: issued now, consumed after the softmax
        i32x2_t vfr[16];
        lds_issue_v_frags(vfr, lds_base + buf * STAGE + voff0, lds_base + buf * STAGE + voff1);
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
            mx = max_across_halves(mx);
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
        // O^T[d tile][query tile] += V^T[d tile][keys] P^T[keys][queries]
        // k-slot (half, e) of step st is key 16st + 8(e/4) + 4half + e%4
        lds_wait_v_frags(vfr);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                bf16x4_t lo = __builtin_bit_cast(bf16x4_t, vfr[2 * (2 * st + dt)]);
                bf16x4_t hi = __builtin_bit_cast(bf16x4_t, vfr[2 * (2 * st + dt) + 1]);
                bf16x8_t vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    oacc[dt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t][st], oacc[dt][t], 0, 0, 0);
            }
        }
        buf = buf + 1 == NST ? 0 : buf + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the look-ahead loads before exit

    // finish: total row sum = both halves; O[query][d] = O^T / l
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        float l = sum_across_halves(lsum[t]);
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
    (void)dtype; (void)batch; (void)seq; (void)heads; (void)head_dim;
    return 0;
}

hipError_t launch_attention(int dtype, const void* q, const void* k, const void* v, void* o,
                            int batch, int seq, int heads, int head_dim, float scale,
                            const AttnStrides& s, void* ws, hipStream_t st) {
    (void)ws;
    if (dtype == PS_BF16 && head_dim == 64 && get_kernel_path() != 1) {
        constexpr int QT = 2;
        constexpr int BQ = 4 * QT * 32;
        int qblocks = (seq + BQ - 1) / BQ;
        dim3 grid(qblocks * heads * batch);
        attn_mfma_kernel<QT><<<grid, 256, 0, st>>>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o,
                                                   seq, heads, scale * 1.4426950408889634f, qblocks, s);
        return hipGetLastError();
    }
    if (dtype == PS_BF16)
        return launch_generic_attn<bf16_t>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, batch,
                                           seq, heads, head_dim, scale, s, st);
    return launch_generic_attn<float>((const float*)q, (const float*)k, (const float*)v, (float*)o, batch, seq,
                                      heads, head_dim, scale, s, st);
}

}  // namespace ps
