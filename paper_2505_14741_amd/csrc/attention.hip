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
#include <type_traits>

namespace ps {

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
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
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

__device__ __forceinline__ bf16x4_t lds_read_tr16(const unsigned char* p) {
    s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p));
    return __builtin_bit_cast(bf16x4_t, v);
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

// Softmax bookkeeping.  Every query keeps a reference value r (bf16-representable) and the
// kernel accumulates sum_j 2^(c(s_j - r)) v_j and sum_j 2^(c(s_j - r)); any r gives the same
// quotient, so r is only moved when it has to be:
//  * r starts at 0 and stays there while the exponents c*s of the first tile peak within
//    +-32 and no later tile's sum of 2^(c(s - r)) reaches 2^64 (fp32 sums stay far from
//    overflow, and a row whose maximum is >= -32 cannot sum to zero);
//  * once some query of a wave has r != 0, the subtraction s - r still costs no vector
//    instruction: a fifth k16-step of the QK^T MFMA multiplies a constant "1" slot of the K
//    operand with -r stored in the Q operand (skipped while every r of the wave is 0);
//  * a tile goes through the fast path -- exp2, pack to bf16, row sum with v_dot2c on the
//    packed pairs -- without looking for its maximum; the partial row sums tell whether any
//    2^(c(s - r)) was large or overflowed, and only then (and on the first and on a ragged
//    last tile) the tile is redone through the exact path: true row maximum, new r, rescale
//    of the running sums.
// PRESCALED: q already carries the factor c = scale*log2(e) (the QKV projection applies it
// in fp32 before rounding), so p = exp2(acc) with no multiply; otherwise p = exp2(c*acc).
// ---- fast variant without a reference --------------------------------------------------------
// attn_sp_kernel accumulates sum_j 2^(c s_j) v_j and sum_j 2^(c s_j) as they are: the quotient is the softmax
// whenever no term overflows and the sum does not vanish, which is the case for every head whose exponents c*s
// stay within roughly +-100 of zero.  It does not look for maxima; it checks its result instead.  A query row
// whose key sum l is outside [2^-40, 2^100], or whose accumulators are not finite, marks its (batch, head) in
// a flag array; the launch of attn_mfma_kernel that follows recomputes exactly the marked heads with a tracked
// reference and overwrites them.  (l >= 2^-40 also bounds what flushing tiny terms to zero can cost: with
// l >= 2^-40 the largest term is at least 2^-40 / N, and the terms below the smallest normal number, 2^-126,
// sum to less than N * 2^-126, i.e. a fraction below 2^-58 of l for any sequence this kernel accepts.)
// The check is exact about what went wrong, where a bound on the exponents from the largest query and key
// norms (Cauchy-Schwarz) would send every head with large norms, however harmless its scores, to the slower kernel;
// heads that really overflow are computed twice.
constexpr float SP_SUM_MIN = 0x1p-40f, SP_SUM_MAX = 0x1p+100f;

__global__ void attn_flags_clear_kernel(unsigned* __restrict__ flags, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = 0u;
}

static constexpr int PART_STRIDE = 68;      // floats per row of a partial result (64 + l + r, padded to 16 B)

// Work items of a launch.  Every sample of the batch has the same items -- (head, block of 256 queries), qblocks *
// heads of them -- and the same plan: the first full_ps run whole, the last tail_ps (fewer than half a round of the
// chip's workgroup slots) are each split nsplit ways along the keys.  The plan depends on the sample's shape only,
// never on the batch, so a sample's result is bit-identical whatever batch it is computed in (Section 3.3: the
// batched step must reproduce the per-step process).  Workgroup ids: the batch * full_ps whole items of all samples
// first, then the pieces.
struct AttnGrid { int qblocks, heads, full_ps, tail_ps, nsplit, all_full; };

// id -> sample, head, query block; piece index (-1: whole item) and its share [jt0, jt1) of the nt key tiles
__device__ __forceinline__ void attn_item(const AttnGrid& g, int id, int nt, int& bh, int& qb, int& piece, int& jt0,
                                          int& jt1) {
    int sample, local;
    piece = -1; jt0 = 0; jt1 = nt;
    if (id < g.all_full) {
        // consecutive ids of one XCD walk the query blocks of one head, so that head's K and V stay in that XCD's L2
        const int per = g.all_full / 8, rem = g.all_full % 8, x = id % 8, j = id / 8;
        id = x * per + (x < rem ? x : rem) + j;
        sample = id / g.full_ps;
        local = id - sample * g.full_ps;
    } else {
        piece = id - g.all_full;
        const int per_sample = g.tail_ps * g.nsplit;
        sample = piece / per_sample;
        const int lp = piece - sample * per_sample;
        local = g.full_ps + lp / g.nsplit;
        const int pi = lp % g.nsplit;
        jt0 = (int)((long)nt * pi / g.nsplit);
        jt1 = (int)((long)nt * (pi + 1) / g.nsplit);
    }
    const int h = local / g.qblocks;
    qb = local - h * g.qblocks;
    bh = sample * g.heads + h;
}

// Merge of the key-range pieces of the split items: one thread per (row, 4 output values).
// O = sum_i w_i O_i / sum_i w_i l_i with w_i = 2^(c (r_i - max_i r_i)).
// (a device function: it runs as a kernel of its own and as the trailing workgroups of attn_mfma_kernel)
// g: the plan the pieces were produced under; nitems = batch * g.tail_ps
__device__ __forceinline__ void
attn_merge_rows(int block, const float* __restrict__ part, bf16_t* __restrict__ o, int seq, const AttnGrid& g,
                int nitems, float cexp, int bq, const AttnStrides& s, const unsigned* __restrict__ fail) {
    const int gid = block * 256 + threadIdx.x;
    const int d4 = gid & 15, rowid = gid >> 4;          // 16 threads per row
    const int item = rowid / bq, row = rowid % bq;      // item: over all samples
    if (item >= nitems) return;
    const int sample = item / g.tail_ps;
    const int local = g.full_ps + item % g.tail_ps;
    const int h = local / g.qblocks, qb = local % g.qblocks;
    const int bh = sample * g.heads + h;
    if (fail != nullptr && fail[bh] != 0u) return;      // a marked head is recomputed whole by attn_mfma_kernel
    const int b = sample;
    const int qi = qb * bq + row;
    if (qi >= seq) return;
    const int nsplit = g.nsplit;
    const float* p0 = part + ((long)item * nsplit * bq + row) * PART_STRIDE;
    float rmax = p0[65];
    for (int i = 1; i < nsplit; ++i) rmax = fmaxf(rmax, p0[(long)i * bq * PART_STRIDE + 65]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
    for (int i = 0; i < nsplit; ++i) {
        const float* pi = p0 + (long)i * bq * PART_STRIDE;
        const float w = __builtin_amdgcn_exp2f((pi[65] - rmax) * cexp);
        const float4 v = *reinterpret_cast<const float4*>(pi + d4 * 4);
        acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
        l += w * pi[64];
    }
    const float inv = 1.0f / l;
    bf16x4_t wv;
    wv[0] = (__bf16)(acc.x * inv); wv[1] = (__bf16)(acc.y * inv);
    wv[2] = (__bf16)(acc.z * inv); wv[3] = (__bf16)(acc.w * inv);
    *reinterpret_cast<bf16x4_t*>(o + b * s.o_batch + (long)qi * s.o_tok + h * s.o_head + d4 * 4) = wv;
}

__global__ void __launch_bounds__(256)
attn_merge_kernel(const float* __restrict__ part, bf16_t* __restrict__ o, int seq, AttnGrid g, int nitems, float cexp,
                  int bq, AttnStrides s, const unsigned* __restrict__ fail) {
    attn_merge_rows(blockIdx.x, part, o, seq, g, nitems, cexp, bq, s, fail);
}

// Merge work that rides on a launch of attn_mfma_kernel: its first `blocks` workgroups merge the pieces another,
// earlier launch left in `part` under plan `g` (blocks == 0: none); the items follow.  (In front, because where
// every head is bounded the item workgroups exit at once and the merge is all the launch does.)
struct MergeTail {
    const float* part;
    int blocks, nitems, bq;
    float cexp;
    AttnGrid g;
};

// global->LDS load of 16 bytes per lane: lane j's bytes land at lds_addr + 16*j (lds_addr
// wave-uniform, passed through M0).  _base: scalar 64-bit base + per-lane 32-bit byte offset;
// _ptr: per-lane 64-bit address.
// XOR applied to the 16-byte chunk index of V row r in LDS (low three bits of r matter): bits 0-1 = r & 3,
// bit 2 = bit 1 of r.  A transposing fragment read covers rows 4m..4m+3 with 32 lanes per cycle; rows r and
// r + 2 start in the same bank, and the flipped bit 2 keeps their 64-byte windows apart (with r & 7 instead
// every such read took twice as long: measured as LDS bank conflict cycles).
__device__ __forceinline__ int v_swizzle(int r) { return (r & 3) | ((r & 2) << 1); }

__device__ __forceinline__ void lds_dma16_base(unsigned voff, const void* sbase, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}
__device__ __forceinline__ void lds_dma16_ptr(const void* gptr, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
// acc + sum of eight bf16 values (v_dot2c_f32_bf16 against packed ones)
__device__ __forceinline__ float rowsum_bf16x8(bf16x8_t p, float acc) {
    bf16x2_t ones;
    ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 0, 1), ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 2, 3), ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 4, 5), ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p, p, 6, 7), ones, acc, false);
    return acc;
}

template <int QT, bool PRESCALED>   // QT: 32-query column tiles per wave
__global__ void __launch_bounds__(256, 2)
attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                 bf16_t* __restrict__ o, int seq, float scale_log2e, AttnStrides s, AttnGrid grid,
                 float* __restrict__ part, const unsigned* __restrict__ fail, MergeTail mt) {
    if ((int)blockIdx.x < mt.blocks) {                      // whole workgroup: before any barrier
        attn_merge_rows(blockIdx.x, mt.part, o, seq, mt.g, mt.nitems, mt.cexp, mt.bq, s, fail);
        return;
    }
    const int heads = grid.heads;
    constexpr int KV = 64;
    constexpr int BQ = 4 * QT * 32;
    constexpr int NST = 3;                       // LDS ring depth
    constexpr int STAGE = 2 * KV * 128;          // K tile then V tile, 128-byte rows
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform values stay in scalar registers
    const int col = lane & 31, half = lane >> 5;
    // workgroup -> (batch*head, query block), see AttnGrid.  A whole item takes one workgroup over all keys; a
    // piece of a split item leaves unnormalised sums, row sum and reference in `part` for the merge.
    int bh, qb, piece, jt0, jt1;
    attn_item(grid, blockIdx.x - mt.blocks, (seq + KV - 1) / KV, bh, qb, piece, jt0, jt1);
    // with `fail` given, only the heads attn_sp_kernel marked are (re)computed here
    if (fail != nullptr && fail[bh] == 0u) return;
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
    // pin the Q loads here: the compiler must not place its own vmcnt wait for them inside the
    // loop, where it would also wait for the K/V tile loads in flight
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) asm volatile("" ::"v"(qf[t][ks]));

    f32x16_t oacc[2][QT];
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[d][t][e] = 0.f;
    float mref[QT], lsum[QT];
    bf16x8_t qx[QT];                 // Q operand of the reference step: slot (half 0, e 0) = -r
    bf16x8_t kone;                   // K operand of the reference step: slot (half 0, e 0) = 1
#pragma unroll
    for (int e = 0; e < 8; ++e) kone[e] = (__bf16)((e == 0 && half == 0) ? 1.0f : 0.0f);
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        mref[t] = 0.f; lsum[t] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) qx[t][e] = (__bf16)0.0f;
    }
    const float cexp = PRESCALED ? 1.0f : scale_log2e;
    // Exponents are taken relative to a per-query reference r that stays 0 as long as the scores
    // (in log2 units) of the first tile peak within +-REF_WINDOW and no later tile's sum of
    // 2^(s - r) reaches REF_SUM_LIMIT: fp32 sums over any sequence this kernel accepts stay far
    // from overflow, and a row whose maximum is >= -REF_WINDOW cannot underflow to a zero sum.
    constexpr float REF_WINDOW = 32.0f, REF_SUM_LIMIT = 0x1p+64f;
    bool has_ref = false;                        // wave-uniform: some query of this wave has r != 0

    // direct global->LDS loads: a wave instruction fills 8 rows of 128 bytes (lane j lands
    // at base + 16j), so the XOR swizzles are applied on the global side.  LDS has 64
    // four-byte banks.  K fragments are 16-byte reads of 16 consecutive rows per cycle:
    // slot p of row r holds chunk p ^ ((r>>1)&7).  V fragments are transposing 8-byte
    // reads, 32 lanes per cycle, that touch 4 consecutive rows x 64 bytes: slot p of row r
    // holds chunk p ^ v_swizzle(r), which sends rows r and r+2 (same 32 banks) to different
    // 64-byte halves.
    // Per stage: 8 K groups + 8 V groups; wave w takes K groups w, w+4 and V groups w, w+4.
    // The loads are issued from inline asm (the compiler then never orders LDS reads of other
    // stages behind them; the explicit vmcnt waits and barriers below publish a stage).  A tile
    // that lies entirely inside the sequence is addressed as scalar tile base + a per-lane byte
    // offset fixed for the whole kernel, so the loop spends no vector instruction on addresses;
    // the last, ragged tile and the look-ahead tiles past the end clamp their rows per lane.
    const int lr = lane >> 3;
    const int lc_v = (lane & 7) ^ v_swizzle(lr);
    const unsigned lds_base = (unsigned)(size_t)PS_LDS_PTR(lds);
    unsigned koff[2], voff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int g = wave + 4 * i;
        const int lc_k = (lane & 7) ^ (((g & 1) << 2) | (lane >> 4));
        koff[i] = (unsigned)(((g * 8 + lr) * s.k_tok + lc_k * 8) * 2);
        voff[i] = (unsigned)(((g * 8 + lr) * s.v_tok + lc_v * 8) * 2);
    }
    auto issue = [&](int tile, int buf) {
        const unsigned st = lds_base + buf * STAGE;
        if ((tile + 1) * KV <= seq) {
            const char* kb = reinterpret_cast<const char*>(kbase) + (long)tile * KV * s.k_tok * 2;
            const char* vb = reinterpret_cast<const char*>(vbase) + (long)tile * KV * s.v_tok * 2;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int g = wave + 4 * i;
                lds_dma16_base(koff[i], kb, st + g * 1024);
                lds_dma16_base(voff[i], vb, st + KV * 128 + g * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int g = wave + 4 * i;
                int kr = tile * KV + g * 8 + lr;
                kr = kr < seq ? kr : seq - 1;        // rows past the end re-read the last key (masked later)
                const int lc_k = (lane & 7) ^ (((g & 1) << 2) | (lane >> 4));
                lds_dma16_ptr(kbase + (long)kr * s.k_tok + lc_k * 8, st + g * 1024);
                lds_dma16_ptr(vbase + (long)kr * s.v_tok + lc_v * 8, st + KV * 128 + g * 1024);
            }
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
    const unsigned voff0 = KV * 128 + trow * 128 + ((tchunk ^ v_swizzle(trow)) << 4) + tsub;
    const unsigned voff1 = KV * 128 + trow * 128 + (((4 + tchunk) ^ v_swizzle(trow)) << 4) + tsub;

    issue(jt0, 0);
    issue(jt0 + 1, 1);                             // tiles past the end are harmless re-reads
    int buf = 0;
    for (int j = jt0; j < jt1; ++j) {
        const int kv0 = j * KV;
        // tile j has landed when at most the 4 loads of tile j+1 are still in flight
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        __syncthreads();
        {
            int nb = buf + 2; nb = nb >= NST ? nb - NST : nb;
            issue(j + 2, nb);
        }
        const unsigned char* lk = lds + buf * STAGE;

        // S^T[key tile rt][query tile t] - r, as a function: the exact path recomputes it rather
        // than keeping 64 accumulator registers alive across the fast path
        f32x16_t sacc[2][QT];
        auto scores = [&]() {
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
                    bf16x8_t kf =
                        *reinterpret_cast<const bf16x8_t*>(lk + r * 128 + (((ks * 2 + half) ^ ((r >> 1) & 7)) << 4));
#pragma unroll
                    for (int t = 0; t < QT; ++t)
                        sacc[rt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][ks], sacc[rt][t], 0, 0, 0);
                }
            }
            // reference step: sacc -= r (per query column); skipped while every reference of the wave is 0
            if (has_ref) {
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int t = 0; t < QT; ++t)
                        sacc[rt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kone, qx[t], sacc[rt][t], 0, 0, 0);
            }
        };
        // V^T fragments: issued now, consumed after the softmax
        i32x2_t vfr[16];
        lds_issue_v_frags(vfr, lds_base + buf * STAGE + voff0, lds_base + buf * STAGE + voff1);
        bf16x8_t pf[QT][4];
        const bool ragged = kv0 + KV > seq;
        bool redo = (j == jt0) || ragged;
        if (!redo) {
            scores();
            // fast path: p = 2^(c (s - r)) without a maximum
            float rsv[QT];
#pragma unroll
            for (int t = 0; t < QT; ++t) {
                float rs = 0.f;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int g = 0; g < 2; ++g) {      // k16-step inside the 32-key tile
                        bf16x8_t pk;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            float a = sacc[rt][t][g * 8 + e];
                            pk[e] = (__bf16)__builtin_amdgcn_exp2f(PRESCALED ? a : a * cexp);
                        }
                        pf[t][rt * 2 + g] = pk;
                        rs = rowsum_bf16x8(pk, rs);
                    }
                // large or non-finite partial sum: some exponent was far above the reference
                redo = redo || !(rs < REF_SUM_LIMIT);
                rsv[t] = rs;
            }
            redo = __any(redo);
            if (!redo) {
#pragma unroll
                for (int t = 0; t < QT; ++t) lsum[t] += rsv[t];
            }
        }
        if (redo) {
            scores();
            bool moved = false;
            if (ragged) {
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
#pragma unroll
            for (int t = 0; t < QT; ++t) {
                // exact path: sacc holds s - r_old; move the reference to the row maximum
                float mx = sacc[0][t][0];
#pragma unroll
                for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[0][t][e]);
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[1][t][e]);
                mx = max_across_halves(mx);                       // finite: every tile has a valid key
                if (j > jt0) mx = fmaxf(mx, 0.f);                 // the reference never moves down
                // first tile: keep the reference at 0 while the maximum is within 2^+-REF_WINDOW of it
                if (j == jt0 && fabsf(mx * cexp) <= REF_WINDOW) mx = 0.f;
                const float rnew = (float)(__bf16)(mref[t] + mx); // new reference, bf16-representable
                moved = moved || rnew != 0.f;
                const float d = rnew - mref[t];
                if (j > jt0) {
                    const float alpha = __builtin_amdgcn_exp2f(-d * cexp);
                    lsum[t] *= alpha;
#pragma unroll
                    for (int dd = 0; dd < 2; ++dd)
#pragma unroll
                        for (int e = 0; e < 16; ++e) oacc[dd][t][e] *= alpha;
                }
                mref[t] = rnew;
                qx[t][0] = (__bf16)(half == 0 ? -rnew : 0.0f);
                float rs = 0.f;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        bf16x8_t pk;
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            pk[e] = (__bf16)__builtin_amdgcn_exp2f((sacc[rt][t][g * 8 + e] - d) * cexp);
                        pf[t][rt * 2 + g] = pk;
                        rs = rowsum_bf16x8(pk, rs);
                    }
                lsum[t] += rs;
            }
            has_ref = has_ref || __any(moved);
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
    if (piece >= 0) {
        // partial result of a key range: [piece][row in block][64 sums | row sum | reference | pad]
        float* pp = part + (long)piece * BQ * PART_STRIDE;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            const float l = sum_across_halves(lsum[t]);
            float* pr = pp + (long)(wave * (QT * 32) + t * 32 + col) * PART_STRIDE;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4*>(pr + dt * 32 + g * 8 + half * 4) =
                        make_float4(oacc[dt][t][g * 4], oacc[dt][t][g * 4 + 1], oacc[dt][t][g * 4 + 2],
                                    oacc[dt][t][g * 4 + 3]);
            if (half == 0) { pr[64] = l; pr[65] = mref[t]; }
        }
        return;
    }
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

// The kernel without a softmax reference (see SP_SUM_MIN above): p = 2^(c s), the result checks itself at the end.
// Work split and LDS layout as in attn_mfma_kernel (4 waves x 64 queries, K/V tiles of 64 keys straight into
// an LDS ring, two workgroups per CU), but the loop is software-pipelined over 32-key half tiles.  In
// every step a wave issues the 8 MFMAs of S^T for the NEXT half, the exp2 / pack instructions (and the row-sum MFMAs) of
// the CURRENT half and the 8 MFMAs of O^T += V^T P^T for the PREVIOUS half.  The three are independent,
// so the compiler interleaves them and the instruction stream is a steady mix of MFMA and vector ALU work.
// A wave that alternates long MFMA-only and ALU-only blocks (the other kernel) leaves the matrix pipe
// idle during its ALU blocks even with a second wave on the SIMD, because both waves drift into phase;
// a homogeneous stream keeps both units busy.  Measured on a register-only replica: 1.77 vs 1.37-1.43
// PFLOP/s-equivalent.  (Workgroups of 8 such waves sharing each K/V tile, one per CU, measured 2-3 % slower; 8 waves
// of 32 queries, four per SIMD, 6 % slower; the steps written out in a fixed order, one MFMA with two exp2 and one
// pack per group, 3 % slower than the compiler's order.
// The same loop on v_mfma_f32_16x16x32_bf16 -- query blocks of 16, the eight exponentials of a lane again the B
// fragment of the second product -- measured +1.5 % at 17776 keys, -2.4 % at 33976, -2 to -7 % below 5000: dropped.)
// Steps of iteration j (tile j = halves a, b):
//   A: S(j,b)    | softmax(j,a)  | PV(j-1,b)
//   B: S(j+1,a)  | softmax(j,b)  | PV(j,a)
// so tiles j-1, j, j+1 are read during iteration j and tile j+2 is being loaded: four ring slots.
template <bool PRESCALED>
__global__ void __launch_bounds__(256, 2)
attn_sp_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
               bf16_t* __restrict__ o, int seq, float scale_log2e, AttnStrides s, AttnGrid grid,
               float* __restrict__ part, unsigned* __restrict__ fail) {
    constexpr int QT = 2;                        // 32-query column tiles per wave
    constexpr int KV = 64;                       // keys per tile
    constexpr int BQ = 4 * QT * 32;              // queries per workgroup
    constexpr int NST = 4;                       // LDS ring depth
    constexpr int STAGE = 2 * KV * 128;          // K tile then V tile, 128-byte rows
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    // work items and the key split of the last partial round: as in attn_mfma_kernel
    const int heads = grid.heads;
    int bh, qb, piece, jt0, jt1;
    attn_item(grid, blockIdx.x, (seq + KV - 1) / KV, bh, qb, piece, jt0, jt1);
    const float cexp = PRESCALED ? 1.0f : scale_log2e;
    const int b = bh / heads, h = bh % heads;
    const int q0 = qb * BQ + wave * (QT * 32);

    const bf16_t* kbase = k + b * s.k_batch + h * s.k_head;
    const bf16_t* vbase = v + b * s.v_batch + h * s.v_head;

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
    // pin the Q loads here: the compiler must not place its own vmcnt wait for them inside the
    // loop, where it would also wait for the K/V tile loads in flight
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) asm volatile("" ::"v"(qf[t][ks]));

    f32x16_t oacc[2][QT];
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[d][t][e] = 0.f;
    // Row sums on the matrix pipe.  A P^T fragment (16 keys x 32 queries, lane = query % 32 with 8 keys, the
    // other 8 in lane + 32) read as the B operand of the 16x16x32 product puts queries 0-15 into k-groups 0
    // and 2 and queries 16-31 into k-groups 1 and 3 of column lane % 16.  With an A operand whose row 0 is
    // one over the even groups and row 1 one over the odd groups, rows 0 and 1 of the 16x16 result are the
    // key sums of queries 0-15 and 16-31: one MFMA replaces four v_dot2c and the adds that follow.
    f32x4_t lacc[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) lacc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    bf16x8_t sel;
    {
        const int r16 = lane & 15, grp = lane >> 4;
        const bool on = (r16 == 0 && (grp & 1) == 0) || (r16 == 1 && (grp & 1) == 1);
#pragma unroll
        for (int e = 0; e < 8; ++e) sel[e] = on ? (__bf16)1.0f : (__bf16)0.0f;
    }

    // loads: per tile 8 K + 8 V row groups of 8 rows; wave w takes groups w and w+4 of each
    const int lr = lane >> 3;
    const int lc_v = (lane & 7) ^ v_swizzle(lr);
    const unsigned lds_base = (unsigned)(size_t)PS_LDS_PTR(lds);
    unsigned koff[2], voff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int g = wave + 4 * i;
        const int lc_k = (lane & 7) ^ (((g & 1) << 2) | (lane >> 4));
        koff[i] = (unsigned)(((g * 8 + lr) * s.k_tok + lc_k * 8) * 2);
        voff[i] = (unsigned)(((g * 8 + lr) * s.v_tok + lc_v * 8) * 2);
    }
    auto issue = [&](int tile) {
        const unsigned st = lds_base + ((tile - jt0) & (NST - 1)) * STAGE;
        if ((tile + 1) * KV <= seq) {
            const char* kb = reinterpret_cast<const char*>(kbase) + (long)tile * KV * s.k_tok * 2;
            const char* vb = reinterpret_cast<const char*>(vbase) + (long)tile * KV * s.v_tok * 2;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int g = wave + 4 * i;
                lds_dma16_base(koff[i], kb, st + g * 1024);
                lds_dma16_base(voff[i], vb, st + KV * 128 + g * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int g = wave + 4 * i;
                int kr = tile * KV + g * 8 + lr;
                kr = kr < seq ? kr : seq - 1;        // rows past the end re-read the last key (masked later)
                const int lc_k = (lane & 7) ^ (((g & 1) << 2) | (lane >> 4));
                lds_dma16_ptr(kbase + (long)kr * s.k_tok + lc_k * 8, st + g * 1024);
                lds_dma16_ptr(vbase + (long)kr * s.v_tok + lc_v * 8, st + KV * 128 + g * 1024);
            }
        }
    };

    // V^T fragment addressing for ds_read_b64_tr_b16 (see attn_mfma_kernel)
    const int tg = lane >> 4, tj = lane & 15;
    const int trow = 4 * (tg >> 1) + (tj >> 2);
    const int tchunk = 2 * (tg & 1) + ((tj & 3) >> 1);
    const int tsub = (tj & 1) * 8;
    const int vad0 = KV * 128 + trow * 128 + ((tchunk ^ v_swizzle(trow)) << 4) + tsub;
    const int vad1 = KV * 128 + trow * 128 + (((4 + tchunk) ^ v_swizzle(trow)) << 4) + tsub;
    // K fragment addressing: key row 32*hh + col, chunk (2 ks + half) ^ ((row >> 1) & 7); the row term of
    // the XOR is the same for both halves of a tile (32 rows = 16 * 2)
    const int ksw = (col >> 1) & 7;
    const int kad = col * 128;

    // ---- the three parts of a step
    // S^T of half hh of the tile in ring slot `slot`
    auto scores = [&](f32x16_t (&sacc)[QT], int slot, int hh) {
        const unsigned char* lk = lds + slot * STAGE + hh * (32 * 128) + kad;
#pragma unroll
        for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[t][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(lk + (((ks * 2 + half) ^ ksw) << 4));
#pragma unroll
            for (int t = 0; t < QT; ++t)
                sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][ks], sacc[t], 0, 0, 0);
        }
    };
    // p = 2^(c s), packed to bf16, and the row sums; MASK: keys at or past `seq` get p = 0
    auto softmax = [&](f32x16_t (&sacc)[QT], bf16x8_t (&pf)[QT][2], int key0, bool mask) {
        if (mask) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = key0 + 8 * (e >> 2) + 4 * half + (e & 3);
                if (key >= seq) {
#pragma unroll
                    for (int t = 0; t < QT; ++t) sacc[t][e] = -INFINITY;
                }
            }
        }
#pragma unroll
        for (int t = 0; t < QT; ++t) {
#pragma unroll
            for (int g = 0; g < 2; ++g) {          // k16-step inside the 32-key half
                bf16x8_t pk;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float a = sacc[t][g * 8 + e];
                    pk[e] = (__bf16)__builtin_amdgcn_exp2f(PRESCALED ? a : a * cexp);
                }
                pf[t][g] = pk;
                lacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, pk, lacc[t], 0, 0, 0);
            }
        }
    };
    // O^T += V^T P^T for half hh of the tile in ring slot `slot`; k-slot (half, e) of step g is key
    // 32 hh + 16 g + 8(e/4) + 4 half + e%4
    auto pv = [&](const bf16x8_t (&pf)[QT][2], int slot, int hh) {
        const unsigned char* lv = lds + slot * STAGE + hh * (32 * 128);
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                const unsigned char* a = lv + (dt ? vad1 : vad0) + g * 2048;
                const bf16x4_t lo = lds_read_tr16(a), hi = lds_read_tr16(a + 1024);
                const bf16x8_t vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    oacc[dt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t][g], oacc[dt][t], 0, 0, 0);
            }
    };

    // key sum of this lane's query: row n / 16, column n % 16 of the small product = register n / 16 of lane n % 16
    auto rowsum_of = [&](int t) -> float {
        const float lo = __shfl(lacc[t][0], col & 15, 64), hi = __shfl(lacc[t][1], col & 15, 64);
        return col < 16 ? lo : hi;
    };

    f32x16_t sa[QT], sb[QT];
    bf16x8_t pa[QT][2], pb[QT][2];
    issue(jt0);
    issue(jt0 + 1);                                // tiles past the end are harmless re-reads
    asm volatile("s_waitcnt vmcnt(4)" ::: "memory");   // own share of the first tile
    __syncthreads();
    scores(sa, 0, 0);
    // one iteration; FIRST / LAST are compile-time so that the steps of the steady state are straight-line
    // code the scheduler can interleave
    auto iteration = [&](int j, auto first_c, auto last_c) {
        constexpr bool FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
        const int slot = (j - jt0) & (NST - 1);
        const bool mask = LAST && (j + 1) * KV > seq;
        // tile j+1 has landed (own share), for every wave after the barrier; the slot of tile j-2 is free
        // (the barrier costs 0.5 % of the kernel: timed once without it)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        issue(j + 2);
        // step A
        scores(sb, slot, 1);
        softmax(sa, pa, j * KV, mask);
        if constexpr (!FIRST) pv(pb, (slot + NST - 1) & (NST - 1), 1);
        __builtin_amdgcn_sched_barrier(0);
        // step B
        if constexpr (!LAST) scores(sa, (slot + 1) & (NST - 1), 0);
        softmax(sb, pb, j * KV + 32, mask);
        pv(pa, slot, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    using std::false_type;
    using std::true_type;
    if (jt1 - jt0 == 1) {
        iteration(jt0, true_type{}, true_type{});
    } else {
        iteration(jt0, true_type{}, false_type{});
        for (int j = jt0 + 1; j < jt1 - 1; ++j) iteration(j, false_type{}, false_type{});
        iteration(jt1 - 1, false_type{}, true_type{});
    }
    pv(pb, (jt1 - 1 - jt0) & (NST - 1), 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the look-ahead loads before exit

    // the result checks itself (see SP_SUM_MIN): key sums out of range or accumulators that are not finite mark the
    // head for attn_mfma_kernel.  (A key range of a split item is held to the same limits as a whole row: a range
    // whose keys all lie far below the row's maximum sends the head to the other kernel, which costs time only.)
    {
        bool bad = false;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            const float l = rowsum_of(t);
            float mag = 0.f;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) mag += fabsf(oacc[dt][t][e]);
            bad = bad || !(l >= SP_SUM_MIN && l <= SP_SUM_MAX) || !(mag < INFINITY);
        }
        if (__any(bad) && lane == 0) fail[bh] = 1u;
    }
    if (piece >= 0) {
        // partial result of a key range, reference 0: [piece][row in block][64 sums | row sum | 0 | pad]
        float* pp = part + (long)piece * BQ * PART_STRIDE;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            const float l = rowsum_of(t);
            float* pr = pp + (long)(wave * (QT * 32) + t * 32 + col) * PART_STRIDE;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4*>(pr + dt * 32 + g * 8 + half * 4) =
                        make_float4(oacc[dt][t][g * 4], oacc[dt][t][g * 4 + 1], oacc[dt][t][g * 4 + 2],
                                    oacc[dt][t][g * 4 + 3]);
            if (half == 0) { pr[64] = l; pr[65] = 0.f; }
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        float l = rowsum_of(t);
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

// Split plan for the bf16 head-dim-64 kernels (see AttnGrid): per sample, how many work items run whole and how
// many ways the rest is split along the keys.
struct AttnPlan { int qblocks, items_ps, full_ps, tail_ps, nsplit, bq; };
static int compute_units() {
    // per device, asked once (a constant of the device, not a setting)
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}
// kernel path 3 sends every head to the reference-tracking kernel; otherwise every head first takes the
// software-pipelined kernel without a reference, which marks the heads it could not do
static bool attention_checked_path(int path) { return (path & 0xff) != 3; }
static AttnPlan attention_plan(int seq, int heads) {
    constexpr int KV = 64;
    AttnPlan p;
    p.bq = 256;
    p.qblocks = (seq + p.bq - 1) / p.bq;
    p.items_ps = p.qblocks * heads;
    const int slots = compute_units() * 2;               // two resident workgroups per CU
    const int tail = p.items_ps % slots;
    const int ntiles = (seq + KV - 1) / KV;
    int ns = tail > 0 ? slots / tail : 1;
    if (ns > 8) ns = 8;
    if (ns > ntiles / 2) ns = ntiles / 2;
    if (tail == 0 || p.items_ps < slots || ns < 2) { p.full_ps = p.items_ps; p.tail_ps = 0; p.nsplit = 1; }
    else { p.full_ps = p.items_ps - tail; p.tail_ps = tail; p.nsplit = ns; }
    return p;
}

static size_t flags_bytes(int batch, int heads) { return (((size_t)batch * heads * sizeof(unsigned)) + 255) & ~(size_t)255; }

// workspace of the bf16 head-dim-64 kernels: [one flag per (batch, head) | key-split pieces]
size_t attention_workspace_bytes(int dtype, int batch, int seq, int heads, int head_dim) {
    if (dtype != PS_BF16 || head_dim != 64 || batch < 1 || seq < 1 || heads < 1) return 0;
    const AttnPlan p = attention_plan(seq, heads);
    const size_t need = (size_t)batch * p.tail_ps * p.nsplit * p.bq * PART_STRIDE * sizeof(float);
    return flags_bytes(batch, heads) + need;
}

bool attention_uses_mfma(int dtype, int head_dim, int path) {
    return dtype == PS_BF16 && head_dim == 64 && (path & 0xff) != 1;
}

float* attention_head_flags(int dtype, int batch, int heads, int head_dim, void* ws, int path, hipStream_t st,
                            bool clear, int* count) {
    if (count) *count = 0;
    if (!ws || !attention_uses_mfma(dtype, head_dim, path) || !attention_checked_path(path)) return nullptr;
    const int nb = batch * heads;
    if (count) *count = nb;
    if (!clear) return (float*)ws;
    attn_flags_clear_kernel<<<(nb + 255) / 256, 256, 0, st>>>((unsigned*)ws, nb);
    return hipGetLastError() == hipSuccess ? (float*)ws : nullptr;
}

hipError_t launch_attention(int dtype, const void* q, const void* k, const void* v, void* o,
                            int batch, int seq, int heads, int head_dim, float scale,
                            const AttnStrides& s, void* ws, int path, hipStream_t st, bool q_prescaled,
                            bool flags_cleared) {
    if (attention_uses_mfma(dtype, head_dim, path)) {
        if (ws == nullptr) return hipErrorInvalidValue;
        if (s.k_tok >= (1 << 24) || s.v_tok >= (1 << 24)) return hipErrorInvalidValue;   // 32-bit in-tile offsets
        const bool checked = attention_checked_path(path);
        AttnPlan p = attention_plan(seq, heads);
        if ((path & 0xff) == 2) { p.full_ps = p.items_ps; p.tail_ps = 0; p.nsplit = 1; }
        const float c = scale * 1.4426950408889634f;
        const float cexp = q_prescaled ? 1.0f : c;
        const bf16_t *qq = (const bf16_t*)q, *kk = (const bf16_t*)k, *vv = (const bf16_t*)v;
        unsigned* flags = (unsigned*)ws;
        float* part = (float*)((char*)ws + flags_bytes(batch, heads));
        const int bq = p.bq;
        const AttnGrid split{p.qblocks, heads, p.full_ps, p.tail_ps, p.nsplit, batch * p.full_ps};
        const AttnGrid whole{p.qblocks, heads, p.items_ps, 0, 1, batch * p.items_ps};
        const int split_blocks = batch * (p.full_ps + p.tail_ps * p.nsplit);
        const int nitems = batch * p.tail_ps;
        if (checked) {
            // the kernel without a reference for every head (it marks the heads whose sums left the safe range),
            // then the reference-tracking kernel (unsplit) for the marked heads; each of its workgroups looks its head up
            if (!flags_cleared) {
                const int nb = batch * heads;
                attn_flags_clear_kernel<<<(nb + 255) / 256, 256, 0, st>>>(flags, nb);
            }
            if (q_prescaled)
                attn_sp_kernel<true><<<split_blocks, 256, 0, st>>>(qq, kk, vv, (bf16_t*)o, seq, c, s, split, part, flags);
            else
                attn_sp_kernel<false><<<split_blocks, 256, 0, st>>>(qq, kk, vv, (bf16_t*)o, seq, c, s, split, part, flags);
            // then the reference-tracking kernel (unsplit) for the other heads; the merge of attn_sp_kernel's pieces
            // rides on that launch as workgroups in front of the items
            MergeTail mt{part, 0, nitems, bq, cexp, split};
            // (a multiple of 8 workgroups, so that the items keep their place in the round-robin over the 8 XCDs)
            if (nitems != 0) mt.blocks = ((int)(((long)nitems * bq * 16 + 255) / 256) + 7) & ~7;
            if (q_prescaled)
                attn_mfma_kernel<2, true><<<whole.all_full + mt.blocks, 256, 0, st>>>(qq, kk, vv, (bf16_t*)o, seq, c, s,
                                                                                    whole, nullptr, flags, mt);
            else
                attn_mfma_kernel<2, false><<<whole.all_full + mt.blocks, 256, 0, st>>>(qq, kk, vv, (bf16_t*)o, seq, c, s,
                                                                                     whole, nullptr, flags, mt);
            return hipGetLastError();
        }
        // (one 32-query tile per wave, i.e. 128-query workgroups at three per CU, measured 9 % slower:
        // it doubles the K/V traffic into LDS and the fragment reads per MFMA)
        const MergeTail none{nullptr, 0, 0, 0, 0.f, whole};
        if (q_prescaled)
            attn_mfma_kernel<2, true><<<split_blocks, 256, 0, st>>>(qq, kk, vv, (bf16_t*)o, seq, c, s, split, part, nullptr,
                                                                   none);
        else
            attn_mfma_kernel<2, false><<<split_blocks, 256, 0, st>>>(qq, kk, vv, (bf16_t*)o, seq, c, s, split, part, nullptr,
                                                                    none);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess || nitems == 0) return err;
        const long threads = (long)nitems * bq * 16;
        attn_merge_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, st>>>(part, (bf16_t*)o, seq, split, nitems, cexp, bq,
                                                                            s, nullptr);
        return hipGetLastError();
    }
    if (q_prescaled) return hipErrorInvalidValue;     // only the MFMA kernel takes pre-scaled queries
    if (dtype == PS_BF16)
        return launch_generic_attn<bf16_t>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, batch,
                                           seq, heads, head_dim, scale, s, st);
    return launch_generic_attn<float>((const float*)q, (const float*)k, (const float*)v, (float*)o, batch, seq,
                                      heads, head_dim, scale, s, st);
}

}  // namespace ps
