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

// Residual values of one wave's outputs, requested before the main loop so that the
// read-modify-write epilogue finds them in registers (rows past M re-read the last row).
template <int TM, int TN>
struct ResidualPrefetch {
    float x[TM][TN][16];
};
template <int TM, int TN>
__device__ __forceinline__ void prefetch_residual(ResidualPrefetch<TM, TN>& rp, const float* __restrict__ X, int M,
                                                  int Nn, int row0, int col0) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int col = col0 + j * 32;
        col = col < Nn ? col : Nn - 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int m = row0 + i * 32 + 8 * (e >> 2) + (e & 3);
                m = m < M ? m : M - 1;
                rp.x[i][j][e] = X[(unsigned)(m * Nn + col)];
            }
    }
}

// Writes the TM x TN accumulator tiles of one wave.  row0/col0: first row (incl. the
// lane's 4*half offset) and the lane's column of tile (0,0).  Offsets are 32-bit element
// indices from the uniform base pointers (the launcher guarantees M*Nn < 2^31).
template <int TM, int TN, int KIND, bool CHECK>
__device__ __forceinline__ void tile_epilogue(f32x16_t (&acc)[TM][TN], const Epilogue& ep, bf16_t* __restrict__ C,
                                              int M, int Nn, int row0, int col0, int lane,
                                              const ResidualPrefetch<TM, TN>* rp) {
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
                        ep.resid[off] = rp->x[i][j][e] + gate * (acc[i][j][e] + bias);
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
                        ep.resid[off] = rp->x[i][j][e] + gate * (acc[i][j][e] + bias);
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

// global->LDS load of 16 bytes per lane, issued from inline asm: lane j's bytes land at
// lds_addr + 16*j (lds_addr wave-uniform, passed through M0).  The compiler does not see the
// LDS write, so it never orders LDS reads of other stages behind loads still in flight; the
// explicit vmcnt waits and barriers in the kernel make a stage visible before it is read.
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// BK: K depth of an LDS stage (64 or 32 bf16 = 128- or 64-byte rows); NST: ring depth.
// Stage kt+NST-1 is requested while stage kt is multiplied.
template <int BM, int BN, int WR, int WC, int BK, int NST, int KIND>
__global__ void __launch_bounds__(WR * WC * 64, (WR * WC == 4 && BM * BN <= 128 * 128) ? 2 : 1)
gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, bf16_t* __restrict__ C,
                 int M, int Nn, int K, int tiles_m, int tiles_n, Epilogue ep) {
    static_assert(BK == 64 || BK == 32, "stage depth");
    constexpr int NW = WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWB = BK * 2;                         // bytes per LDS row
    constexpr int RPI = 1024 / ROWB;                     // rows filled by one wave instruction (8 or 16)
    constexpr int CPR = ROWB / 16;                       // 16-byte chunks per row (8 or 4)
    constexpr int GROUPS = (BM + BN) / RPI;
    constexpr int GPW = GROUPS / NW;                     // load instructions per wave per stage
    constexpr int STAGE = (BM + BN) * ROWB;
    static_assert(GROUPS % NW == 0, "rows must split evenly over waves");
    static_assert(BM % RPI == 0, "a load group must not straddle the A/W boundary");
    static_assert((NST - 1) * GPW <= 63, "vmcnt range");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

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

    // Swizzle (LDS has 64 four-byte banks; a 16-byte fragment read is served 16 lanes = 16
    // consecutive rows at a time, which must hit 16 different 16-byte bank groups):
    //   128-byte rows: slot p of row r holds chunk p ^ ((r>>1)&7)
    //    64-byte rows: slot p of row r holds chunk p ^ ((r>>2)&3)
    // applied on the global side of the direct load (lane j lands at base + 16j).
    const int lr = lane / CPR;                           // row inside the load group
    const bf16_t* gp[GPW];
#pragma unroll
    for (int i = 0; i < GPW; ++i) {
        const int g = wave + NW * i;
        const int row = g * RPI + lr;                    // row within [A rows | W rows]
        const int lc = BK == 64 ? ((lane & 7) ^ ((row >> 1) & 7)) : ((lane & 3) ^ ((row >> 2) & 3));
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
    const unsigned lds_base = (unsigned)(size_t)PS_LDS_PTR(lds);
    const int nk = K / BK;
    auto issue = [&](int kt) {
        const int kc = kt < nk ? kt : nk - 1;            // past the end: harmless re-read keeps vmcnt uniform
        const unsigned st = lds_base + (kt % NST) * STAGE;
#pragma unroll
        for (int i = 0; i < GPW; ++i) {
            const int g = wave + NW * i;
            lds_dma16(gp[i] + (long)kc * BK, __builtin_amdgcn_readfirstlane(st + g * 1024));
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
    int aoff[TM], boff[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) aoff[i] = (wm * WM + i * 32 + frow) * ROWB;
#pragma unroll
    for (int j = 0; j < TN; ++j) boff[j] = (BM + wn * WN + j * 32 + frow) * ROWB;
    const int sw = BK == 64 ? ((frow >> 1) & 7) : ((frow >> 2) & 3);

    // the residual read-modify-write epilogue gets its inputs now: these loads are older than
    // every stage load, so the first stage wait also covers them and they cost one memory
    // latency per tile instead of one per output row
    ResidualPrefetch<TM, TN> rp;
    if constexpr (KIND == EPI_GATE_RESIDUAL)
        prefetch_residual<TM, TN>(rp, ep.resid, M, Nn, m0 + wm * WM + 4 * fhalf, n0 + wn * WN + frow);
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) issue(p);
    for (int kt = 0; kt < nk; ++kt) {
        // stage kt has landed once at most the NST-2 younger stages are still in flight
        wait_vmcnt<(NST - 2) * GPW>();
        __syncthreads();                                 // ... for every wave; and stage kt-1 is no longer read
        issue(kt + NST - 1);                             // into the buffer stage kt-1 occupied
        const unsigned char* st = lds + (kt % NST) * STAGE;
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
    wait_vmcnt<0>();                                     // drain the look-ahead loads before the wave ends

    // epilogue: a lane owns one output column (feature) of each 32x32 tile and 16 of its rows
    const bool interior = (m0 + BM <= M) && (n0 + BN <= Nn);
    if (interior)
        tile_epilogue<TM, TN, KIND, false>(acc, ep, C, M, Nn, m0 + wm * WM + 4 * fhalf, n0 + wn * WN + frow, lane, &rp);
    else
        tile_epilogue<TM, TN, KIND, true>(acc, ep, C, M, Nn, m0 + wm * WM + 4 * fhalf, n0 + wn * WN + frow, lane, &rp);
}

bool gemm_mfma_supported(int M, int Nn, int K) {
    return K % 64 == 0 && Nn % 2 == 0 && M >= 1 && Nn >= 64 && K >= 64 && (long)M * Nn < (1L << 31);
}

template <int BM, int BN, int WR, int WC, int BK, int NST>
static hipError_t launch_tile(const bf16_t* A, const bf16_t* W, bf16_t* C, int M, int Nn, int K,
                              const Epilogue& ep, hipStream_t st) {
    int tm = (M + BM - 1) / BM, tn = (Nn + BN - 1) / BN;
    dim3 grid(tm * tn), block(WR * WC * 64);
    switch (ep.kind) {
        case EPI_BIAS:
            gemm_mfma_kernel<BM, BN, WR, WC, BK, NST, EPI_BIAS><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep);
            break;
        case EPI_BIAS_GELU:
            gemm_mfma_kernel<BM, BN, WR, WC, BK, NST, EPI_BIAS_GELU><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep);
            break;
        case EPI_GATE_RESIDUAL:
            gemm_mfma_kernel<BM, BN, WR, WC, BK, NST, EPI_GATE_RESIDUAL><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn,
                                                                                                 ep);
            break;
        case EPI_QKV_ROPE:
            gemm_mfma_kernel<BM, BN, WR, WC, BK, NST, EPI_QKV_ROPE><<<grid, block, 0, st>>>(A, W, C, M, Nn, K, tm, tn, ep);
            break;
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
        case 1: return launch_tile<256, 256, 2, 4, 64, 2>(A, W, C, M, Nn, K, ep, st);   // 8 waves, 128x64 each
        case 2: return launch_tile<256, 256, 2, 4, 32, 4>(A, W, C, M, Nn, K, ep, st);   // same tile, deeper ring
        case 3: return launch_tile<128, 128, 2, 2, 64, 2>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 64x64 each, 2 per CU
        case 4: return launch_tile<128, 128, 2, 2, 32, 4>(A, W, C, M, Nn, K, ep, st);   // same tile, deeper ring
        case 5: return launch_tile<256, 128, 4, 2, 64, 3>(A, W, C, M, Nn, K, ep, st);   // 8 waves, 64x64 each
        case 6: return launch_tile<256, 128, 2, 2, 32, 3>(A, W, C, M, Nn, K, ep, st);   // 4 waves, 128x64, 2 per CU
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ps
