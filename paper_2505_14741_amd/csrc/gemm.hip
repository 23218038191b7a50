// C[M, Nn] = A[M, K] * W[Nn, K]^T with fused epilogue.
// This file holds the dispatcher and the generic LDS-tiled fp32-FMA kernel used for the
// fp32 configuration and for bf16 shapes the MFMA kernel does not cover.
#include "common.h"
#include "epilogue.h"

namespace ps {

// 64x64 output tile, 16-deep K slices, 256 threads, 4x4 outputs per thread.
template <typename T, int KIND>
__global__ void __launch_bounds__(256)
gemm_generic_kernel(const T* __restrict__ A, const T* __restrict__ W, T* __restrict__ C, int M, int Nn,
                    int K, Epilogue ep) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Ws[BK][BN + 4];
    int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    // loader mapping: thread -> (row = tid/4, k group = (tid%4)*4 .. +3)
    int lr = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            int k = k0 + lk + kk;
            int am = m0 + lr, wn = n0 + lr;
            As[lk + kk][lr] = (am < M && k < K) ? to_f32(A[(long)am * K + k]) : 0.f;
            Ws[lk + kk][lr] = (wn < Nn && k < K) ? to_f32(W[(long)wn * K + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = Ws[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; j += 2) {
            int col = n0 + tx * 4 + j;
            if (col < Nn)
                epilogue_pair<KIND, T>(ep, C, Nn, m, col, acc[i][j] + ep.bias[col], acc[i][j + 1] + ep.bias[col + 1]);
        }
    }
}

template <typename T>
static hipError_t launch_generic(const T* A, const T* W, T* C, int M, int Nn, int K, const Epilogue& ep,
                                 hipStream_t st) {
    dim3 grid((Nn + 63) / 64, (M + 63) / 64);
    switch (ep.kind) {
        case EPI_BIAS: gemm_generic_kernel<T, EPI_BIAS><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, ep); break;
        case EPI_BIAS_GELU: gemm_generic_kernel<T, EPI_BIAS_GELU><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, ep); break;
        case EPI_GATE_RESIDUAL:
            gemm_generic_kernel<T, EPI_GATE_RESIDUAL><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, ep); break;
        case EPI_QKV_ROPE: gemm_generic_kernel<T, EPI_QKV_ROPE><<<grid, 256, 0, st>>>(A, W, C, M, Nn, K, ep); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool gemm_mfma_supported(int tokens, int Nn, int K);
hipError_t launch_gemm_mfma(const bf16_t* A, const bf16_t* W, bf16_t* C, int batch, int tokens, int Nn, int K,
                            const Epilogue& ep, int path, hipStream_t st);

bool gemm_uses_mfma(int dtype, int tokens, int Nn, int K, int path) {
    return dtype == PS_BF16 && (path & 0xff) != 1 && gemm_mfma_supported(tokens, Nn, K);
}

hipError_t launch_gemm(int dtype, const void* A, const void* W, void* C, int batch, int tokens, int Nn, int K,
                       const Epilogue& epi, int path, hipStream_t st) {
    if (batch <= 0 || tokens <= 0 || Nn <= 0 || K <= 0 || (Nn & 1)) return hipErrorInvalidValue;
    const bool mfma = gemm_uses_mfma(dtype, tokens, Nn, K, path);
    if (epi.kind == EPI_UNPATCHIFY && !mfma) return hipErrorInvalidValue;
    if (mfma)
        return launch_gemm_mfma((const bf16_t*)A, (const bf16_t*)W, (bf16_t*)C, batch, tokens, Nn, K, epi, path, st);
    const int M = batch * tokens;                    // (the generic kernel forms 64-bit offsets)
    if (dtype == PS_BF16)
        return launch_generic<bf16_t>((const bf16_t*)A, (const bf16_t*)W, (bf16_t*)C, M, Nn, K, epi, st);
    return launch_generic<float>((const float*)A, (const float*)W, (float*)C, M, Nn, K, epi, st);
}

}  // namespace ps
