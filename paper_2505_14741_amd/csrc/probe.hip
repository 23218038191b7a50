// Measurement aid: a loop of nothing but bf16 matrix instructions on register operands.  What it sustains is the
// practical ceiling of the matrix pipes on this chip under load (the clock drops under matrix load), which the
// benchmark reports next to the nominal peak the roofline fractions are quoted against.
#include "common.h"

namespace ps {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int PROBE_ACCS = 8;        // independent accumulators per wave: covers the instruction's latency

__global__ void __launch_bounds__(256, 2)
mfma_probe_kernel(int iters, float* __restrict__ sink) {
    // operands: pseudo-random values in (-1, 1), different in every lane (data toggling matters for power and clock)
    unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    bf16x8_t a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        h = h * 1664525u + 1013904223u;
        a[e] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.0f / 32768.0f) - 1.0f);
        h = h * 1664525u + 1013904223u;
        b[e] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.0f / 32768.0f) - 1.0f);
    }
    f32x4_t acc[PROBE_ACCS];
#pragma unroll
    for (int j = 0; j < PROBE_ACCS; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < PROBE_ACCS; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PROBE_ACCS; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == 1.2345e30f) sink[0] = s;    // never true for these operands: keeps the loop alive
}

// launches 2 workgroups of 4 waves per compute unit (two waves per SIMD); *flops = operations the launch performs
hipError_t launch_mfma_probe(int iters, float* sink, double* flops, hipStream_t st) {
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const int blocks = 2 * cus;
    mfma_probe_kernel<<<blocks, 256, 0, st>>>(iters, sink);
    if (flops) *flops = (double)blocks * 4.0 * iters * PROBE_ACCS * (2.0 * 16 * 16 * 32);
    return hipGetLastError();
}

}  // namespace ps
