// libjet_probe.so -- a measurement aid of the benchmark, built beside libjet.so and not part
// of its ABI: a register-resident stream of the FP8 matrix-core instruction that the GEMM kernels
// are built on, so that a benchmark can report the rate the chip sustains for it at its own power
// state beside the published peak.  No memory traffic inside the timed loop.
//
//   int jet_probe_mfma_rate(float* out, int32_t workgroups, int32_t iters, int32_t zero_data, void* stream)
// launches `workgroups` workgroups of 8 waves that each issue 32 * iters instructions on register
// operands (pseudo-random finite E4M3 bytes, or all zero if zero_data != 0):
// flop = workgroups * 8 * 32 * iters * 65536.  out: device, f32 [workgroups * 8], one value per
// wave (a checksum of no meaning).  1 <= workgroups <= 65536, 1 <= iters <= 2^24.  Returns the
// status codes of include/jet.h (NULL 1, SHAPE 2, ALIGN 3, LAUNCH 5).
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

}  // namespace jet

extern "C" __attribute__((visibility("default")))
int jet_probe_mfma_rate(float* out, int32_t workgroups, int32_t iters, int32_t zero_data, void* stream) {
    if (!out) return 1;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24)) return 2;
    if (reinterpret_cast<uintptr_t>(out) & 15u) return 3;
    (void)hipGetLastError();
    hipLaunchKernelGGL(jet::mfma_rate_kernel, dim3((unsigned)workgroups), dim3(512), 0,
                       static_cast<hipStream_t>(stream), out, iters, zero_data != 0);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}
