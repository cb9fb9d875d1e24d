// Measurement aid (not a step of the layer): a register-resident stream of the FP8
// matrix-core instruction that the GEMM kernels are built on, so that a benchmark can
// report the rate the chip sustains for it at its own power state beside the published
// peak.  No memory traffic inside the timed loop.
#include "jet_internal.h"
#include "jet_numerics.h"

namespace jet {

// 8 waves per workgroup (two per SIMD), 32 independent accumulator tiles per wave.
// Operand bytes: a counter-based hash of (lane, register) with the exponent field
// limited to 0..7, i.e. |value| < 2 and never the NaN code, or all zero.
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* __restrict__ out, int iters, int zero_data) {
    v8i a[4], b[8];
#pragma unroll
    for (int f = 0; f < 12; ++f) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t h = (threadIdx.x * 12u + f) * 8u + i + 0x9e3779b9u * (blockIdx.x + 1u);
            h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
            const int v = zero_data ? 0 : (int)(h & 0xbfbfbfbfu);   // bit 6 of every byte clear: exponent <= 7
            if (f < 4) a[f][i] = v; else b[f - 4][i] = v;
        }
    }
    v4f acc[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 32; ++j)
            acc[j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[j & 3], b[j >> 2], acc[j], 0, 0, 0, 0, 0, 0);
    }
    float r = 0.0f;
#pragma unroll
    for (int j = 0; j < 32; ++j) r += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    // one value per wave; keeps the loop alive and lets a caller see that it ran
    if ((threadIdx.x & 63) == 0) out[blockIdx.x * 8 + (threadIdx.x >> 6)] = r;
}

hipError_t launch_mfma_rate(float* out, int workgroups, int iters, int zero_data, hipStream_t st) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)workgroups), dim3(512), 0, st, out, iters, zero_data);
    return hipGetLastError();
}

}  // namespace jet
