// bf16 MFMA GEMM for gfx950:  C[M, Nn] = A[M, K] * W[Nn, K]^T, fp32 accumulate, fused epilogue.
//
// Both operands are K-contiguous, so each lane's MFMA fragment (8 consecutive k of one
// row) is a single 16-byte LDS read.  Workgroup = 4 waves in a 2x2 grid over a BM x BN
// tile; every wave owns (BM/2) x (BN/2) outputs as 32x32 v_mfma_f32_32x32x16_bf16 tiles.
// K is consumed 64 at a time: the next slice is fetched from global memory into
// registers while the current one is multiplied out of LDS (single LDS buffer, two
// barriers per slice; a second resident workgroup per CU covers the barrier bubbles).
// LDS rows are 128 bytes (64 bf16); the 16-byte chunk index is XOR-swizzled with the row
// so that the 32 rows a fragment read touches spread over all banks.
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

#ifndef PS_GEMM_SWZ_SHIFT
#define PS_GEMM_SWZ_SHIFT 0
#endif
__device__ __forceinline__ int swz(int row) { return (row >> PS_GEMM_SWZ_SHIFT) & 7; }

// Consecutive workgroup ids go to different XCDs (8 of them, each with its own L2).
// Give each XCD a contiguous range of tiles, and walk tiles column-fastest inside it so
// co-resident workgroups share activation rows and weight panels in that L2.
__device__ __forceinline__ int xcd_remap(int id, int total) {
    int per = total / 8, rem = total % 8;
    int x = id % 8, j = id / 8;
    // XCD x owns `per` tiles (+1 for the first `rem` XCDs)
    int start = x * per + (x < rem ? x : rem);
    return start + j;
}

template <int BM, int BN, int KIND>
__global__ void __launch_bounds__(256, 2)
gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, bf16_t* __restrict__ C,
                 int M, int Nn, int K, int tiles_m, int tiles_n, Epilogue ep) {
    constexpr int BK = 64;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int LA = BM / 32, LB = BN / 32;      // 16-byte loads per thread per slice
    __shared__ __attribute__((aligned(16))) unsigned char lds[(BM + BN) * BK * 2];
    unsigned char* ldsA = lds;
    unsigned char* ldsB = lds + BM * BK * 2;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    // global -> register staging: thread handles chunk (tid%8) of rows tid/8 + 32*i
    const int lrow = tid >> 3, lchunk = tid & 7;
    const bf16_t* aptr[LA];
    const bf16_t* bptr[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int r = m0 + lrow + 32 * i;
        r = r < M ? r : M - 1;
        aptr[i] = A + (long)r * K + lchunk * 8;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        int r = n0 + lrow + 32 * i;
        r = r < Nn ? r : Nn - 1;
        bptr[i] = W + (long)r * K + lchunk * 8;
    }
    uint4 ra[LA], rb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) ra[i] = *reinterpret_cast<const uint4*>(aptr[i]);
#pragma unroll
    for (int i = 0; i < LB; ++i) rb[i] = *reinterpret_cast<const uint4*>(bptr[i]);

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int frow = lane & 31, fhalf = lane >> 5;
    const int nk = K / BK;
    for (int kt = 0; kt < nk; ++kt) {
        // registers -> LDS (swizzled)
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            int r = lrow + 32 * i;
            *reinterpret_cast<uint4*>(ldsA + r * 128 + ((lchunk ^ swz(r)) << 4)) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            int r = lrow + 32 * i;
            *reinterpret_cast<uint4*>(ldsB + r * 128 + ((lchunk ^ swz(r)) << 4)) = rb[i];
        }
        __syncthreads();
        // prefetch the next slice while this one is multiplied
        if (kt + 1 < nk) {
#pragma unroll
            for (int i = 0; i < LA; ++i) ra[i] = *reinterpret_cast<const uint4*>(aptr[i] + (long)(kt + 1) * BK);
#pragma unroll
            for (int i = 0; i < LB; ++i) rb[i] = *reinterpret_cast<const uint4*>(bptr[i] + (long)(kt + 1) * BK);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[TM], fb[TN];
            int c = ks * 2 + fhalf;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int r = wm * WM + i * 32 + frow;
                fa[i] = *reinterpret_cast<const bf16x8_t*>(ldsA + r * 128 + ((c ^ swz(r)) << 4));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int r = wn * WN + j * 32 + frow;
                fb[j] = *reinterpret_cast<const bf16x8_t*>(ldsB + r * 128 + ((c ^ swz(r)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // epilogue: lanes pair up so each owns two adjacent columns of one row
    const bool odd = lane & 1;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int colbase = n0 + wn * WN + j * 32 + (frow & ~1);
            int rowbase = m0 + wm * WM + i * 32 + 4 * fhalf;
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                float mine0 = acc[i][j][e], mine1 = acc[i][j][e + 1];
                float send = odd ? mine0 : mine1;
                float recv = __shfl_xor(send, 1, 64);
                // even lane: row e   -> (own col, partner col)
                // odd  lane: row e+1 -> (partner col, own col)
                float v0 = odd ? recv : mine0;
                float v1 = odd ? mine1 : recv;
                int ee = odd ? e + 1 : e;
                int m = rowbase + 8 * (ee >> 2) + (ee & 3);
                if (m < M && colbase < Nn) epilogue_pair<KIND, bf16_t>(ep, C, Nn, m, colbase, v0, v1);
            }
        }
    }
}

bool gemm_mfma_supported(int M, int Nn, int K) {
    return K % 64 == 0 && Nn % 2 == 0 && M >= 1 && Nn >= 64 && K >= 64;
}

template <int BM, int BN>
static hipError_t launch_tile(const bf16_t* A, const bf16_t* W, bf16_t* C, int M, int Nn, int K,
                              const Epilogue& ep, hipStream_t st) {
    int tm = (M + BM - 1) / BM, tn = (Nn + BN - 1) / BN;
    dim3 grid(tm * tn);
    switch (ep.kind) {
        case EPI_BIAS:
            gemm_mfma_kernel<BM, BN, EPI_BIAS><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        case EPI_BIAS_GELU:
            gemm_mfma_kernel<BM, BN, EPI_BIAS_GELU><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        case EPI_GATE_RESIDUAL:
            gemm_mfma_kernel<BM, BN, EPI_GATE_RESIDUAL><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        case EPI_QKV_ROPE:
            gemm_mfma_kernel<BM, BN, EPI_QKV_ROPE><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gemm_mfma(const bf16_t* A, const bf16_t* W, bf16_t* C, int M, int Nn, int K,
                            const Epilogue& ep, hipStream_t st) {
    if (M >= 2048 && Nn % 128 == 0) return launch_tile<256, 128>(A, W, C, M, Nn, K, ep, st);
    return launch_tile<128, 128>(A, W, C, M, Nn, K, ep, st);
}

}  // namespace ps
