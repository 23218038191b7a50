// GEMM epilogues applied to a pair of adjacent output columns (col even), so that the
// interleaved rotary pairs (2m, 2m+1) of a head are handled by one thread.  v0, v1 already
// include the bias.
#pragma once
#include "common.h"

namespace ps {

template <int KIND, typename T>
__device__ __forceinline__ void epilogue_pair(const Epilogue& ep, T* __restrict__ C, int Nn, int m,
                                              int col, float v0, float v1) {
    if constexpr (KIND == EPI_BIAS_GELU) {
        v0 = gelu_tanh_f(v0);
        v1 = gelu_tanh_f(v1);
    }
    if constexpr (KIND == EPI_GATE_RESIDUAL) {
        int b = m / ep.geom.tokens, n = m - b * ep.geom.tokens;
        int chunk = ep.gate_chunk + (n < ep.geom.text_tokens ? 6 : 0);
        const float* gate = ep.mod_layer + b * ep.mod_batch_stride + (long)chunk * ep.D;
        float2* xp = reinterpret_cast<float2*>(ep.resid + (long)m * Nn + col);
        float2 xv = *xp;
        xv.x += gate[col] * v0;
        xv.y += gate[col + 1] * v1;
        *xp = xv;
        return;
    }
    if constexpr (KIND == EPI_QKV_ROPE) {
        int n = m % ep.geom.tokens;
        if (n >= ep.geom.text_tokens && col < 2 * ep.D) {
            int nv = n - ep.geom.text_tokens;
            int pr = (col % ep.head_dim) >> 1;
            const RopeAxis ra = rope_axis_of(pr, ep.head_dim, ep.rope_F, ep.rope_Hp);
            const int q1 = nv / ep.rope_Wp, q2 = q1 / ep.rope_Hp;
            const int pos = ra.axis == 0 ? q2 : ra.axis == 1 ? q1 - q2 * ep.rope_Hp : nv - q1 * ep.rope_Wp;
            float cs = ep.rope_cs[ra.base + pos * ra.stride], sn = ep.rope_cs[ra.base + pos * ra.stride + 1];
            float r0 = v0 * cs - v1 * sn;
            float r1 = v0 * sn + v1 * cs;
            v0 = r0;
            v1 = r1;
        }
        if (col < ep.D) { v0 *= ep.q_scale; v1 *= ep.q_scale; }
    }
    if constexpr (sizeof(T) == 2) {
        union { bf16_t h[2]; uint32_t u; } pk;
        pk.h[0] = __float2bfloat16(v0);
        pk.h[1] = __float2bfloat16(v1);
        *reinterpret_cast<uint32_t*>(C + (long)m * Nn + col) = pk.u;
    } else {
        *reinterpret_cast<float2*>(C + (long)m * Nn + col) = make_float2(v0, v1);
    }
}

}  // namespace ps
