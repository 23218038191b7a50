// bf16 MFMA GEMM for gfx950:  C[M, Nn] = A[M, K] * W[Nn, K]^T, fp32 accumulate, fused epilogue.
//
// Both operands are K-contiguous, so each lane's MFMA fragment (8 consecutive k of one
// row) is a single 16-byte LDS read.  One workgroup per CU computes a BM x BN tile with
// WR x WC waves, every wave owning (BM/WR) x (BN/WC) outputs as 32x32
// v_mfma_f32_32x32x16_bf16 tiles.  K is consumed 64 at a time through a two-stage LDS ring
// filled by direct global->LDS loads (global_load_lds_dwordx4: no staging registers, no
// ds_write): the loads of slice k+1 are in flight while slice k is multiplied, one
// barrier per slice.
//
// LDS rows are 128 bytes (64 bf16).  A direct load writes lane j's 16 bytes at
// base + 16*j, so one wave instruction fills 8 rows.  LDS has 64 four-byte banks and a
// 16-byte read is served 16 lanes at a time, so the 16 consecutive rows a fragment read
// touches must land in 16 different 16-byte bank groups: slot p of row r holds chunk
// p ^ ((r >> 1) & 7) (row parity picks the half of the banks, the XOR the group).  The
// swizzle is applied on the global side: lane j of row group g fetches chunk
// (j%8) ^ (4*(g%2) + j/16) of row 8g + j/8.
//
// Output mapping of the 32x32 accumulator: lane l holds column l%32 and rows
// 8*(i/4) + 4*(l/32) + i%4 for i < 16; activations are the row operand, so a lane's
// column is an output feature and stores of one accumulator register are contiguous
// across lanes (bf16 stores cover 64 bytes per row, fp32 residual updates 128).  The
// rotary epilogue gets a pair's other element from the neighbouring lane with one DPP move.
#include "common.h"
#include "epilogue.h"

namespace ps {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

#define PS_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define PS_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Consecutive workgroup ids go to different XCDs (8 of them, each with its own L2).
// Give each XCD a contiguous range of tiles so co-resident workgroups share operand panels.
__device__ __forceinline__ int xcd_remap(int id, int total) {
    int per = total / 8, rem = total % 8;
    int x = id % 8, j = id / 8;
    return x * per + (x < rem ? x : rem) + j;
}

// tanh-form GELU written as x * sigmoid(2u), u = sqrt(2/pi)(x + 0.044715 x^3): two
// transcendentals and four FMAs; used where the result is rounded to bf16.
__device__ __forceinline__ float gelu_fast(float x) {
    const float c0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    const float c1 = c0 * 0.044715f;
    float t = x * (c0 + c1 * x * x);
    return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

__device__ __forceinline__ unsigned short bf16_bits(float v) {
    return __builtin_bit_cast(unsigned short, (__bf16)v);
}

// Writes the TM x TN accumulator tiles of one wave.  row0/col0: first row (incl. the
// lane's 4*half offset) and the lane's column of tile (0,0).  Offsets are 32-bit element
// indices from the uniform base pointers (the launcher guarantees M*Nn < 2^31).
template <int TM, int TN, int KIND, bool CHECK>
__device__ __forceinline__ void tile_epilogue(f32x16_t (&acc)[TM][TN], const Epilogue& ep, bf16_t* __restrict__ C,
                                              int M, int Nn, int row0, int col0, int lane) {
    unsigned short* __restrict__ Cb = reinterpret_cast<unsigned short*>(C);
    const int tokens = ep.geom.tokens, text = ep.geom.text_tokens;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32;
        if (CHECK && col >= Nn) continue;
        const float bias = ep.bias[col];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rb = row0 + i * 32;
            if constexpr (KIND == EPI_BIAS || KIND == EPI_BIAS_GELU) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = rb + 8 * (e >> 2) + (e & 3);
                    if (CHECK && m >= M) continue;
                    float v = acc[i][j][e] + bias;
                    if constexpr (KIND == EPI_BIAS_GELU) v = gelu_fast(v);
                    Cb[(unsigned)(m * Nn + col)] = bf16_bits(v);
                }
            } else if constexpr (KIND == EPI_GATE_RESIDUAL) {
                // X[m, col] += gate[batch(m), stream(m), col] * (acc + bias)
                const int b_lo = rb / tokens, b_hi = (rb + 27) / tokens;
                if (b_lo == b_hi) {
                    const float* g = ep.mod_layer + b_lo * ep.mod_batch_stride + col;
                    const float gv = g[ep.gate_chunk * ep.D], gt = g[(ep.gate_chunk + 6) * ep.D];
                    const int n0r = rb - b_lo * tokens;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int dr = 8 * (e >> 2) + (e & 3);
                        const int m = rb + dr;
                        if (CHECK && m >= M) continue;
                        const float gate = (n0r + dr) < text ? gt : gv;
                        const unsigned off = (unsigned)(m * Nn + col);
                        ep.resid[off] += gate * (acc[i][j][e] + bias);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int m = rb + 8 * (e >> 2) + (e & 3);
                        if (CHECK && m >= M) continue;
                        const int b = m / tokens, n = m - b * tokens;
                        const int chunk = ep.gate_chunk + (n < text ? 6 : 0);
                        const float gate = ep.mod_layer[b * ep.mod_batch_stride + (long)chunk * ep.D + col];
                        const unsigned off = (unsigned)(m * Nn + col);
                        ep.resid[off] += gate * (acc[i][j][e] + bias);
                    }
                }
            } else {   // EPI_QKV_ROPE: rotate (even, odd) column pairs of q and k of video tokens
                const bool rot = col < 2 * ep.D;
                const int pr = (col % ep.head_dim) >> 1;
                const int hd2 = ep.head_dim >> 1;
                const bool odd = lane & 1;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = rb + 8 * (e >> 2) + (e & 3);
                    float v = acc[i][j][e] + bias;
                    const float partner = swap_adjacent_lanes(v);      // before any divergence
                    if (CHECK && m >= M) continue;
                    const int n = m % tokens;
                    if (rot && n >= text) {
                        const unsigned ti = (unsigned)((n - text) * hd2 + pr);
                        const float cs = ep.rope_cos[ti], sn = ep.rope_sin[ti];
                        v = odd ? (v * cs + partner * sn) : (v * cs - partner * sn);
                    }
                    if (col < ep.D) v *= ep.q_scale;
                    Cb[(unsigned)(m * Nn + col)] = bf16_bits(v);
                }
            }
        }
    }
}

template <int BM, int BN, int WR, int WC, int KIND>
__global__ void __launch_bounds__(WR * WC * 64, 1)
gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, bf16_t* __restrict__ C,
                 int M, int Nn, int K, int tiles_m, int tiles_n, Epilogue ep) {
    constexpr int BK = 64;
    constexpr int NW = WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int GROUPS = (BM + BN) / 8;          // 8-row groups per stage, one wave instruction each
    constexpr int GPW = GROUPS / NW;               // groups per wave
    constexpr int STAGE = (BM + BN) * BK * 2;      // bytes
    static_assert(GROUPS % NW == 0, "rows must split evenly over waves");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WC, wn = wave % WC;
    // tiles walk column-fastest inside groups of 8 tile rows, so the workgroups resident on
    // one XCD cover a compact block of the output and reuse each other's panels in L2
    int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    int m0, n0;
    {
        constexpr int GM = 8;
        int per_band = GM * tiles_n;
        int band = tile / per_band, in_band = tile % per_band;
        int rows_here = min(GM, tiles_m - band * GM);
        m0 = (band * GM + in_band % rows_here) * BM;
        n0 = (in_band / rows_here) * BN;
    }

    // direct global->LDS loads: this wave fills row groups wave, wave+NW, ...
    const int lr = lane >> 3;
    const bf16_t* gp[GPW];
#pragma unroll
    for (int i = 0; i < GPW; ++i) {
        int g = wave + NW * i;
        int row = g * 8 + lr;                       // row within [A rows | W rows]
        const int lc = (lane & 7) ^ (((g & 1) << 2) | (lane >> 4));
        if (row < BM) {
            int r = m0 + row;
            r = r < M ? r : M - 1;
            gp[i] = A + (long)r * K + lc * 8;
        } else {
            int r = n0 + row - BM;
            r = r < Nn ? r : Nn - 1;
            gp[i] = W + (long)r * K + lc * 8;
        }
    }
    auto issue = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < GPW; ++i) {
            int g = wave + NW * i;
            __builtin_amdgcn_global_load_lds(PS_GLOBAL_PTR(gp[i] + (long)kt * BK),
                                             PS_LDS_PTR(lds + buf * STAGE + g * 1024), 16, 0, 0);
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int frow = lane & 31, fhalf = lane >> 5;
    // fragment byte offsets inside a stage (row*128 + swizzled chunk); the k16-step only
    // changes the chunk: c = 2*ks + fhalf, slot = c ^ ((row >> 1) & 7)
    int aoff[TM], boff[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) aoff[i] = (wm * WM + i * 32 + frow) * 128;
#pragma unroll
    for (int j = 0; j < TN; ++j) boff[j] = (BM + wn * WN + j * 32 + frow) * 128;
    const int sw = (frow >> 1) & 7;

    const int nk = K / BK;
    issue(0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 1 < nk) issue(kt + 1, buf ^ 1);
        const unsigned char* st = lds + buf * STAGE;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[TM], fb[TN];
            const int slot = ((ks * 2 + fhalf) ^ sw) << 4;
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8_t*>(st + aoff[i] + slot);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const bf16x8_t*>(st + boff[j] + slot);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // epilogue: a lane owns one output column (feature) of each 32x32 tile and 16 of its rows
    const bool interior = (m0 + BM <= M) && (n0 + BN <= Nn);
    if (interior)
        tile_epilogue<TM, TN, KIND, false>(acc, ep, C, M, Nn, m0 + wm * WM + 4 * fhalf, n0 + wn * WN + frow, lane);
    else
        tile_epilogue<TM, TN, KIND, true>(acc, ep, C, M, Nn, m0 + wm * WM + 4 * fhalf, n0 + wn * WN + frow, lane);
}

bool gemm_mfma_supported(int M, int Nn, int K) {
    return K % 64 == 0 && Nn % 2 == 0 && M >= 1 && Nn >= 64 && K >= 64 && (long)M * Nn < (1L << 31);
}

template <int BM, int BN, int WR, int WC>
static hipError_t launch_tile(const bf16_t* A, const bf16_t* W, bf16_t* C, int M, int Nn, int K,
                              const Epilogue& ep, hipStream_t st) {
    int tm = (M + BM - 1) / BM, tn = (Nn + BN - 1) / BN;
    dim3 grid(tm * tn), block(WR * WC * 64);
    switch (ep.kind) {
        case EPI_BIAS:
            gemm_mfma_kernel<BM, BN, WR, WC, EPI_BIAS><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        case EPI_BIAS_GELU:
            gemm_mfma_kernel<BM, BN, WR, WC, EPI_BIAS_GELU><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        case EPI_GATE_RESIDUAL:
            gemm_mfma_kernel<BM, BN, WR, WC, EPI_GATE_RESIDUAL><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        case EPI_QKV_ROPE:
            gemm_mfma_kernel<BM, BN, WR, WC, EPI_QKV_ROPE><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static int g_gemm_variant = 0;   // tuning hook: 0 auto
void set_gemm_variant(int v) { g_gemm_variant = v; }

hipError_t launch_gemm_mfma(const bf16_t* A, const bf16_t* W, bf16_t* C, int M, int Nn, int K,
                            const Epilogue& ep, hipStream_t st) {
    int v = g_gemm_variant;
    if (v == 0) {
        // measured at 17776 tokens inside the forward: two co-resident 128x128 workgroups hide
        // each other's epilogue (rotary, fp32 residual read-modify-write); the wide GELU
        // projection is better off with the 256x256 tile's lower L2 traffic
        if (M < 1024) v = 3;
        else if (ep.kind == EPI_BIAS_GELU || (ep.kind == EPI_BIAS && Nn >= 6144)) v = 1;
        else v = 3;
    }
    switch (v) {
        case 1: return launch_tile<256, 256, 2, 4>(A, W, C, M, Nn, K, ep, st);   // 8 waves, 128x64 each
        case 2: return launch_tile<256, 256, 2, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 128x128 each
        case 3: return launch_tile<128, 128, 2, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 64x64 each
        case 4: return launch_tile<256, 128, 2, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 128x64 each
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ps
