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
// base + 16*j, so one wave instruction fills 8 rows; the XOR swizzle that keeps fragment
// reads conflict-free (16-byte slot p of row r holds chunk p ^ (r & 7)) is applied on the
// global side: lane j fetches chunk (j%8) ^ (j/8) of row j/8.
//
// Output mapping of the 32x32 accumulator: lane l holds column l%32 and rows
// 8*(i/4) + 4*(l/32) + i%4 for i < 16; activations are the row operand, so a lane's
// column is an output feature and stores of one accumulator register are contiguous
// across lanes.  Adjacent lanes swap one value so every lane owns an (even, odd) column
// pair -- the unit the epilogues (bias, GELU, gate*residual, rotary pairs) work on.
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

    // direct global->LDS loads: this wave fills row groups wave, wave+NW, ...; lane j of a
    // group fetches chunk (j%8)^(j/8) of row 8*g + j/8
    const int lr = lane >> 3, lc = (lane & 7) ^ lr;
    const bf16_t* gp[GPW];
#pragma unroll
    for (int i = 0; i < GPW; ++i) {
        int g = wave + NW * i;
        int row = g * 8 + lr;                       // row within [A rows | W rows]
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
    // changes the chunk: c = 2*ks + fhalf, slot = c ^ (row & 7)
    int aoff[TM], boff[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) aoff[i] = (wm * WM + i * 32 + frow) * 128;
#pragma unroll
    for (int j = 0; j < TN; ++j) boff[j] = (BM + wn * WN + j * 32 + frow) * 128;
    const int sw = frow & 7;

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

    // epilogue: lanes pair up so each owns two adjacent columns of one row
    const bool odd = lane & 1;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int colbase = n0 + wn * WN + j * 32 + (frow & ~1);
            int rowbase = m0 + wm * WM + i * 32 + 4 * fhalf;
            if (colbase >= Nn) continue;
            const float2 bias2 = *reinterpret_cast<const float2*>(ep.bias + colbase);
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                float mine0 = acc[i][j][e], mine1 = acc[i][j][e + 1];
                float send = odd ? mine0 : mine1;
                float recv = swap_adjacent_lanes(send);
                // even lane: row e   -> (own col, partner col)
                // odd  lane: row e+1 -> (partner col, own col)
                float v0 = odd ? recv : mine0;
                float v1 = odd ? mine1 : recv;
                int ee = odd ? e + 1 : e;
                int m = rowbase + 8 * (ee >> 2) + (ee & 3);
                if (m < M) epilogue_pair<KIND, bf16_t>(ep, C, Nn, m, colbase, v0 + bias2.x, v1 + bias2.y);
            }
        }
    }
}

bool gemm_mfma_supported(int M, int Nn, int K) {
    return K % 64 == 0 && Nn % 2 == 0 && M >= 1 && Nn >= 64 && K >= 64;
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
    if (v == 0) v = (M >= 1024) ? 1 : 3;
    switch (v) {
        case 1: return launch_tile<256, 256, 2, 4>(A, W, C, M, Nn, K, ep, st);   // 8 waves, 128x64 each
        case 2: return launch_tile<256, 256, 2, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 128x128 each
        case 3: return launch_tile<128, 128, 2, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 64x64 each
        case 4: return launch_tile<256, 128, 2, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 128x64 each
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ps
