// Fused producers: the operator in front of a GEMM writes its output directly as
// 1x128-quantized FP8 (Jet-RL Sec. 4.2: the activation quantization is fused with the
// previous operator; Sec. 4.3 names RMSNorm and the activation function).  The operator's
// bf16 result h is never stored: it is rounded to bf16 in registers and quantized with the
// row quantizer's arithmetic (jet_numerics.h), so the FP8 bytes and scales equal those of
// "operator in bf16, then jet_quant_act".  Both kernels are HBM-bound streams.
#include <algorithm>

#include "jet_internal.h"
#include "jet_numerics.h"

namespace jet {

// ------------------------------------------------------------------------
// bf16 of a binary64 value with one rounding (finite input).  The conversion to binary32
// is monotonic, so the binary32 value lies on the same side of every bf16 tie point as the
// binary64 one -- unless it landed exactly on a tie, where the binary64 value decides.
// ------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bf16_from_double(double v) {
    const float f = (float)v;
    const uint32_t u = __float_as_uint(f);
    if ((u & 0xffffu) == 0x8000u) {
        const double fd = (double)f;
        if (fd != v) return (u >> 16) + (fabs(v) > fabs(fd) ? 1u : 0u);
    }
    return bf16_rne(f);
}

// bf16( g / (1 + e^-g) ) of a bf16 value g, the real function rounded once.
// Fast path in binary32: e^-g = 2^y with y = -g log2(e) split as -g c_hi (exact: 8 x 16
// significant bits) plus a small remainder folded in as a factor 1 + ln2 * (-g c_lo); the
// hardware 2^y and reciprocal are good to 1 ulp each, so the result is within 5 ulp of the
// real value for |g| <= 80 and results above 2^-100.  Where that cannot decide the bf16
// rounding (the binary32 result is within 8 ulp of a tie), and outside that range, binary64
// arithmetic decides.  The function has 65280 finite inputs; the tests check every one.
__device__ __forceinline__ uint32_t silu_bf16(float g) {
    const float c_hi = 0x1.7154p+0f, c_lo = 0x1.d94aep-18f, ln2 = 0x1.62e43p-1f;
    const float p2 = __builtin_amdgcn_exp2f(-g * c_hi);
    const float e = __builtin_fmaf(p2, (-g * c_lo) * ln2, p2);
    const float a = g * __builtin_amdgcn_rcpf(1.0f + e);
    const uint32_t low = __float_as_uint(a) & 0xffffu;
    const bool near_tie = (low - (0x8000u - 8u)) <= 16u;
    const bool in_range = fabsf(g) <= 80.0f && fabsf(a) >= 0x1p-100f;
    if (near_tie || !in_range) {
        const double gd = (double)g;
        return bf16_from_double(gd / (1.0 + exp(-gd)));
    }
    return bf16_rne(a);
}

// quantize the 16 values of a lane (a team of 8 lanes holds one 128-group) and store them
__device__ __forceinline__ void quantize_store(float (&v)[16], uint8_t* q16, float* s1, bool leader) {
    float am = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) am = fmaxf(am, fabsf(v[i]));
    am = team8_max(am);
    const GroupScale gs = make_scale(am);
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = div_by_scale(v[i], gs);
    uint4 o;
    o.x = e4m3_pack4(v[0], v[1], v[2], v[3]);
    o.y = e4m3_pack4(v[4], v[5], v[6], v[7]);
    o.z = e4m3_pack4(v[8], v[9], v[10], v[11]);
    o.w = e4m3_pack4(v[12], v[13], v[14], v[15]);
    *reinterpret_cast<uint4*>(q16) = o;
    if (leader) *s1 = gs.S;
}

__device__ __forceinline__ void unpack16(const uint16_t* p, float (&v)[16]) {
    const uint4* p4 = reinterpret_cast<const uint4*>(p);
    const uint4 u0 = p4[0], u1 = p4[1];
    const uint32_t w[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[2 * i] = bf16_lo(w[i]);
        v[2 * i + 1] = bf16_hi(w[i]);
    }
}

// ------------------------------------------------------------------------
// SiLU(gate) * up -> 1x128 FP8.  a = bf16(silu(g)), h = bf16(a * u) (binary32 product).
// Same decomposition as the row quantizer: a team of 8 lanes owns a group, a lane 16
// consecutive elements (2 x 32 B in, 16 B out).  gate and up share the row stride ld.
// ------------------------------------------------------------------------
__global__ __launch_bounds__(256) void silu_mul_quant_kernel(const uint16_t* __restrict__ gate,
                                                             const uint16_t* __restrict__ up, long ld,
                                                             int groups_per_row, long n_groups,
                                                             uint8_t* __restrict__ q, float* __restrict__ s) {
    const long n_teams = (long)gridDim.x * 32;
    const int l8 = threadIdx.x & 7;
    for (long g = ((long)blockIdx.x * 256 + threadIdx.x) >> 3; g < n_groups; g += n_teams) {
        const long m = g / groups_per_row;
        const long src = m * ld + (g - m * groups_per_row) * kGroup + l8 * 16;
        float a[16], u[16];
        unpack16(gate + src, a);
        unpack16(up + src, u);
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float act0 = __uint_as_float(silu_bf16(a[i]) << 16);
            const float act1 = __uint_as_float(silu_bf16(a[i + 1]) << 16);
            const uint32_t h2 = bf16_pack2(act0 * u[i], act1 * u[i + 1]);
            a[i] = bf16_lo(h2);
            a[i + 1] = bf16_hi(h2);
        }
        quantize_store(a, q + g * kGroup + l8 * 16, s + g, l8 == 0);
    }
}

// ------------------------------------------------------------------------
// RMSNorm -> 1x128 FP8.  A team of kTeam threads owns a row and keeps it in registers
// between the two phases (a thread holds 16-element pieces, one per 16 kTeam columns):
//   1. sum of squares in binary64 (the square of a bf16 value is exact there), reduced over
//      the team; mean rounded once to binary32; r = 1 / sqrt(mean + eps) in binary32;
//   2. n = bf16(x r), h = bf16(gamma n), quantized per 128-group.
// kTeam = 64 (a wave per row, four rows per workgroup, no barrier, up to 128 bytes per lane in
// flight) for rows up to 8192 columns; kTeam = 256 (the workgroup, one barrier) beyond.
// ------------------------------------------------------------------------
template <int kTeam, int MAXCH>
__global__ __launch_bounds__(256) void rmsnorm_quant_kernel(const uint16_t* __restrict__ x,
                                                            const uint16_t* __restrict__ gamma, float eps,
                                                            long M, int K, uint8_t* __restrict__ q,
                                                            float* __restrict__ s) {
    __shared__ double part[4];
    const int t = threadIdx.x, l8 = t & 7;
    const int lane = (kTeam == 64) ? (t & 63) : t;
    const long m = (kTeam == 64) ? (long)blockIdx.x * 4 + (t >> 6) : (long)blockIdx.x;
    if (m >= M) return;                                  // whole waves; only with a wave per row
    const uint16_t* row = x + m * K;
    float v[MAXCH][16];
    double ss = 0.0;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) {
        const int k0 = (c * kTeam + lane) * 16;
        if (k0 < K) unpack16(row + k0, v[c]);
    }
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) {
        const int k0 = (c * kTeam + lane) * 16;
        if (k0 < K) {
#pragma unroll
            for (int i = 0; i < 16; ++i) ss = fma((double)v[c][i], (double)v[c][i], ss);
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) ss += __shfl_xor(ss, d, 64);
    if (kTeam == 256) {
        if ((t & 63) == 0) part[t >> 6] = ss;
        __syncthreads();
        ss = (part[0] + part[1]) + (part[2] + part[3]);
    }
    const float ms = (float)(ss / (double)K);
    const float r = 1.0f / sqrtf(ms + eps);
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) {
        const int k0 = (c * kTeam + lane) * 16;
        if (k0 < K) {   // whole groups: 8 lanes hold one, and K is a multiple of 128
            float gm[16];
            unpack16(gamma + k0, gm);
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const uint32_t n2 = bf16_pack2(v[c][i] * r, v[c][i + 1] * r);
                const uint32_t h2 = bf16_pack2(gm[i] * bf16_lo(n2), gm[i + 1] * bf16_hi(n2));
                v[c][i] = bf16_lo(h2);
                v[c][i + 1] = bf16_hi(h2);
            }
            quantize_store(v[c], q + m * K + k0, s + (m * K + k0) / kGroup, l8 == 0);
        }
    }
}

// ------------------------------------------------------------------------
// Backward of h = bf16(bf16(silu(g)) * u), the element-wise operator between the down projection
// and the gate/up projections of an MLP block (Sec. 4.1: gradients between operators stay bf16):
//   dup = bf16(dh * a),  da = bf16(dh * u),  dgate = bf16(da * silu'(g)),
//   a = bf16(silu(g)) as in the forward,  silu'(g) = s (1 + g (1 - s)),  s = 1 / (1 + e^-g).
// The two products of bf16 values are exact in binary32, so their bf16 rounding is the single
// rounding of the real value.  dgate is the real value da * silu'(g) rounded once: the binary32
// evaluation below carries an error bound (in ulps, growing towards the zero of silu' at
// g = -1.2785 where 1 + g (1 - s) cancels), and whenever the result is closer than that bound to
// a bf16 tie, or outside the range the bound holds in, binary64 decides.
// ------------------------------------------------------------------------
__device__ __forceinline__ uint32_t silu_grad_mul_bf16(float g, float da) {
    const float c_hi = 0x1.7154p+0f, c_lo = 0x1.d94aep-18f, ln2 = 0x1.62e43p-1f;
    const float p2 = __builtin_amdgcn_exp2f(-g * c_hi);
    const float e = __builtin_fmaf(p2, (-g * c_lo) * ln2, p2);     // e^-g, within 4 ulp
    const float r = __builtin_amdgcn_rcpf(1.0f + e);               // s, within 5 ulp
    const float om = e * r;                                        // 1 - s without cancellation, within 9 ulp
    const float gom = g * om;
    const float w = 1.0f + gom;                                    // absolute error <= 10 ulp(g om) + half an ulp of w
    const float prod = da * (r * w);
    // error of prod in its own ulps: <= 7 + 10 |g om| / |w|; doubled as the window around a tie
    const float window = 16.0f + 24.0f * fabsf(gom) * __builtin_amdgcn_rcpf(fabsf(w));
    const float dist = fabsf((float)(int)(__float_as_uint(prod) & 0xffffu) - 32768.0f);
    const bool in_range = fabsf(g) <= 80.0f && fabsf(prod) >= 0x1p-100f;
    if (!(dist > window) || !in_range) {
        const double gd = (double)g;
        const double sd = 1.0 / (1.0 + exp(-gd));
        return bf16_from_double((double)da * (sd * (1.0 + gd * (1.0 - sd))));
    }
    return bf16_rne(prod);
}

__global__ __launch_bounds__(256) void silu_mul_bwd_kernel(const uint16_t* __restrict__ gate,
                                                           const uint16_t* __restrict__ up, long ld,
                                                           const uint16_t* __restrict__ dh, int chunks_per_row,
                                                           long n_chunks, uint16_t* __restrict__ dgate,
                                                           uint16_t* __restrict__ dup, long ld_out) {
    const long stride = (long)gridDim.x * 256;
    for (long c = (long)blockIdx.x * 256 + threadIdx.x; c < n_chunks; c += stride) {
        const long m = c / chunks_per_row;
        const long k = (c - m * chunks_per_row) * 8;
        const uint4 g4 = *reinterpret_cast<const uint4*>(gate + m * ld + k);
        const uint4 u4 = *reinterpret_cast<const uint4*>(up + m * ld + k);
        const uint4 d4 = *reinterpret_cast<const uint4*>(dh + m * (long)chunks_per_row * 8 + k);
        const uint32_t gw[4] = {g4.x, g4.y, g4.z, g4.w}, uw[4] = {u4.x, u4.y, u4.z, u4.w},
                       dw[4] = {d4.x, d4.y, d4.z, d4.w};
        uint32_t og[4], ou[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float g0 = bf16_lo(gw[i]), g1 = bf16_hi(gw[i]);
            const float u0 = bf16_lo(uw[i]), u1 = bf16_hi(uw[i]);
            const float d0 = bf16_lo(dw[i]), d1 = bf16_hi(dw[i]);
            const float a0 = __uint_as_float(silu_bf16(g0) << 16), a1 = __uint_as_float(silu_bf16(g1) << 16);
            ou[i] = bf16_pack2(d0 * a0, d1 * a1);
            const uint32_t da2 = bf16_pack2(d0 * u0, d1 * u1);
            og[i] = silu_grad_mul_bf16(g0, bf16_lo(da2)) | (silu_grad_mul_bf16(g1, bf16_hi(da2)) << 16);
        }
        *reinterpret_cast<uint4*>(dgate + m * ld_out + k) = uint4{og[0], og[1], og[2], og[3]};
        *reinterpret_cast<uint4*>(dup + m * ld_out + k) = uint4{ou[0], ou[1], ou[2], ou[3]};
    }
}

// ----------------------------------------------------------------- launch --

hipError_t launch_silu_mul_quant(const void* gate, const void* up, long ld, long M, long K, uint8_t* q,
                                 float* s, hipStream_t st) {
    const long n_groups = M * (K / kGroup);
    const long blocks = std::min<long>((n_groups + 31) / 32, 256L * 64);
    hipLaunchKernelGGL(silu_mul_quant_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const uint16_t*>(gate), static_cast<const uint16_t*>(up), ld,
                       (int)(K / kGroup), n_groups, q, s);
    return hipGetLastError();
}

hipError_t launch_silu_mul_bwd(const void* gate, const void* up, long ld, const void* dh, long M, long K,
                               void* dgate, void* dup, long ld_out, hipStream_t st) {
    const long n_chunks = M * (K / 8);
    const long blocks = std::min<long>((n_chunks + 255) / 256, 256L * 32);
    hipLaunchKernelGGL(silu_mul_bwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const uint16_t*>(gate), static_cast<const uint16_t*>(up), ld,
                       static_cast<const uint16_t*>(dh), (int)(K / 8), n_chunks,
                       static_cast<uint16_t*>(dgate), static_cast<uint16_t*>(dup), ld_out);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_quant(const void* x, const void* gamma, float eps, long M, long K, uint8_t* q,
                                float* s, hipStream_t st) {
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const uint16_t* gp = static_cast<const uint16_t*>(gamma);
#define JET_RMS(TEAM, N, GRID) \
    hipLaunchKernelGGL((rmsnorm_quant_kernel<TEAM, N>), dim3((unsigned)(GRID)), dim3(256), 0, st, xp, gp, eps, M, (int)K, q, s)
    if (K <= 8192) {
        const int chunks = (int)((K + 1023) / 1024);
        const long grid = (M + 3) / 4;
        if (chunks <= 1) JET_RMS(64, 1, grid);
        else if (chunks <= 2) JET_RMS(64, 2, grid);
        else if (chunks <= 4) JET_RMS(64, 4, grid);
        else JET_RMS(64, 8, grid);
    } else {
        const int chunks = (int)((K + 4095) / 4096);
        if (chunks <= 4) JET_RMS(256, 4, M);
        else JET_RMS(256, 8, M);
    }
#undef JET_RMS
    return hipGetLastError();
}

}  // namespace jet
