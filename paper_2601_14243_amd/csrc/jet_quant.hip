// Fused amax / scale / cast quantizers (Jet-RL Sec. 2.1 formula at the
// granularities of Sec. 4.2).  All of them are HBM-bound streaming kernels:
// every input byte is read once with 16-byte loads, every output byte written
// once, reductions stay in registers (DPP) or LDS.
#include "jet_internal.h"
#include "jet_numerics.h"

namespace jet {

// ------------------------------------------------------------------------
// Row quantizer: 1x128 groups along the contiguous axis.  A team of 8 lanes
// owns one group; a lane owns 16 consecutive elements (32 B of bf16 in, 16 B
// of codes out).  Works for any M (decode shapes included).
// ------------------------------------------------------------------------
template <int SRC>
__global__ __launch_bounds__(256) void quant_row_kernel(const void* __restrict__ x,
                                                        const float* __restrict__ xs,
                                                        uint8_t* __restrict__ q,
                                                        float* __restrict__ s, long n_groups) {
    const long n_teams = (long)gridDim.x * 32;
    const int l8 = threadIdx.x & 7;
    for (long g = ((long)blockIdx.x * 256 + threadIdx.x) >> 3; g < n_groups; g += n_teams) {
        float v[16];
        if (SRC == JET_SRC_BF16) {
            const uint4* p = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(x) + g * kGroup + l8 * 16);
            uint4 u0 = p[0], u1 = p[1];
            const uint32_t w[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[2 * i] = bf16_lo(w[i]);
                v[2 * i + 1] = bf16_hi(w[i]);
            }
        } else {
            const uint4 u = *reinterpret_cast<const uint4*>(static_cast<const uint8_t*>(x) + g * kGroup + l8 * 16);
            const float sc = xs[g];
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float a, b, c, d;
                e4m3_unpack4(w[i], a, b, c, d);
                v[4 * i] = a * sc;
                v[4 * i + 1] = b * sc;
                v[4 * i + 2] = c * sc;
                v[4 * i + 3] = d * sc;
            }
        }
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
        *reinterpret_cast<uint4*>(q + g * kGroup + l8 * 16) = o;
        if (l8 == 0) s[g] = gs.S;
    }
}

// ------------------------------------------------------------------------
// Tile quantizer: one workgroup per 128x128 tile of the source.
//   ROW  : 1x128 groups along the contiguous axis   -> q_row, s_row
//   COL  : 128x1 groups along the row axis, outputs transposed -> q_colT, s_colT
//   BLOCK: one scale for the whole tile (weights); q_row/s_row are the plain
//          outputs, q_colT/s_colT the optional transposed copy (COL says whether
//          it is wanted).
// Thread (rr = t>>4, cc = t&15) holds rows 8rr..8rr+7, columns 8cc..8cc+7 of the
// tile as binary32, so that codes pack along either axis without shuffles; the
// transposed bytes go through LDS once so that global stores are 16 B wide.
// ------------------------------------------------------------------------
constexpr int kTPitch = 136;  // bytes per transposed row in LDS (8-byte aligned, off the bank period)

template <int SRC, bool ROW, bool COL, bool BLOCK>
__global__ __launch_bounds__(256) void quant_tile_kernel(const void* __restrict__ x,
                                                         const float* __restrict__ xs, long M, long K,
                                                         uint8_t* __restrict__ q_row,
                                                         float* __restrict__ s_row,
                                                         uint8_t* __restrict__ q_colT,
                                                         float* __restrict__ s_colT) {
    __shared__ float red[16 * 128];
    __shared__ float scS[128];
    __shared__ __attribute__((aligned(16))) uint8_t T[128 * kTPitch];

    const int t = threadIdx.x, rr = t >> 4, cc = t & 15;
    const long m0 = (long)blockIdx.y * 128, k0 = (long)blockIdx.x * 128;
    const long GK = K / kGroup, GM = M / kGroup;

    float v[8][8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const long row = m0 + 8 * rr + p;
        if (SRC == JET_SRC_BF16) {
            const uint4 u = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(x) + row * K + k0 + 8 * cc);
            v[p][0] = bf16_lo(u.x); v[p][1] = bf16_hi(u.x);
            v[p][2] = bf16_lo(u.y); v[p][3] = bf16_hi(u.y);
            v[p][4] = bf16_lo(u.z); v[p][5] = bf16_hi(u.z);
            v[p][6] = bf16_lo(u.w); v[p][7] = bf16_hi(u.w);
        } else {
            const uint2 u = *reinterpret_cast<const uint2*>(static_cast<const uint8_t*>(x) + row * K + k0 + 8 * cc);
            const float sc = xs[row * GK + blockIdx.x];
            e4m3_unpack4(u.x, v[p][0], v[p][1], v[p][2], v[p][3]);
            e4m3_unpack4(u.y, v[p][4], v[p][5], v[p][6], v[p][7]);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[p][j] *= sc;
        }
    }

    if (BLOCK) {
        // one amax for the tile: lanes -> 16-lane rows -> wave -> workgroup
        float am = 0.0f;
#pragma unroll
        for (int p = 0; p < 8; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) am = fmaxf(am, fabsf(v[p][j]));
        am = team16_max(am);
        am = fmaxf(am, __shfl_xor(am, 16));
        am = fmaxf(am, __shfl_xor(am, 32));
        if ((t & 63) == 0) red[t >> 6] = am;
        __syncthreads();
        am = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const GroupScale gs = make_scale(am);
#pragma unroll
        for (int p = 0; p < 8; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) v[p][j] = div_by_scale(v[p][j], gs);
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            uint2 o;
            o.x = e4m3_pack4(v[p][0], v[p][1], v[p][2], v[p][3]);
            o.y = e4m3_pack4(v[p][4], v[p][5], v[p][6], v[p][7]);
            *reinterpret_cast<uint2*>(q_row + (m0 + 8 * rr + p) * K + k0 + 8 * cc) = o;
        }
        if (t == 0) {
            s_row[(long)blockIdx.y * GK + blockIdx.x] = gs.S;
            if (COL) s_colT[(long)blockIdx.x * GM + blockIdx.y] = gs.S;
        }
        if (COL) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint2 o;
                o.x = e4m3_pack4(v[0][j], v[1][j], v[2][j], v[3][j]);
                o.y = e4m3_pack4(v[4][j], v[5][j], v[6][j], v[7][j]);
                *reinterpret_cast<uint2*>(&T[(8 * cc + j) * kTPitch + 8 * rr]) = o;
            }
        }
    } else {
        if (ROW) {
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                float am = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) am = fmaxf(am, fabsf(v[p][j]));
                am = team16_max(am);
                const GroupScale gs = make_scale(am);
                float tq[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) tq[j] = div_by_scale(v[p][j], gs);
                uint2 o;
                o.x = e4m3_pack4(tq[0], tq[1], tq[2], tq[3]);
                o.y = e4m3_pack4(tq[4], tq[5], tq[6], tq[7]);
                const long row = m0 + 8 * rr + p;
                *reinterpret_cast<uint2*>(q_row + row * K + k0 + 8 * cc) = o;
                if (cc == 0) s_row[row * GK + blockIdx.x] = gs.S;
            }
        }
        if (COL) {
            // column amax: registers -> LDS partials over the 16 row-threads -> 128 scales
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float cm = 0.0f;
#pragma unroll
                for (int p = 0; p < 8; ++p) cm = fmaxf(cm, fabsf(v[p][j]));
                red[rr * 128 + 8 * cc + j] = cm;
            }
            __syncthreads();
            if (t < 128) {
                float am = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) am = fmaxf(am, red[r * 128 + t]);
                const float S = (am == 0.0f) ? 1.0f : am / kDeltaMax;
                scS[t] = am;
                s_colT[(k0 + t) * GM + blockIdx.y] = S;
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const GroupScale gs = make_scale(scS[8 * cc + j]);
                float tq[8];
#pragma unroll
                for (int p = 0; p < 8; ++p) tq[p] = div_by_scale(v[p][j], gs);
                uint2 o;
                o.x = e4m3_pack4(tq[0], tq[1], tq[2], tq[3]);
                o.y = e4m3_pack4(tq[4], tq[5], tq[6], tq[7]);
                *reinterpret_cast<uint2*>(&T[(8 * cc + j) * kTPitch + 8 * rr]) = o;
            }
        }
    }

    if (COL) {
        __syncthreads();
        // T[kl][0..127] holds column k0+kl of the tile along m: write it out 16 B at a time
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int chunk = t + 256 * i, kl = chunk >> 3, part = chunk & 7;
            const uint2 a = *reinterpret_cast<const uint2*>(&T[kl * kTPitch + 16 * part]);
            const uint2 b = *reinterpret_cast<const uint2*>(&T[kl * kTPitch + 16 * part + 8]);
            uint4 o = {a.x, a.y, b.x, b.y};
            *reinterpret_cast<uint4*>(q_colT + (k0 + kl) * M + m0 + 16 * part) = o;
        }
    }
}

// ----------------------------------------------------------------- launch --

template <int SRC>
static hipError_t launch_row(const void* x, const float* xs, long M, long K, uint8_t* q, float* s,
                             hipStream_t st) {
    const long n_groups = M * (K / kGroup);
    long blocks = (n_groups + 31) / 32;
    const long cap = 256L * 32;  // a few waves of workgroups per CU, grid-stride beyond that
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL((quant_row_kernel<SRC>), dim3((unsigned)blocks), dim3(256), 0, st, x, xs, q, s, n_groups);
    return hipGetLastError();
}

template <int SRC, bool ROW, bool COL, bool BLOCK>
static hipError_t launch_tile(const void* x, const float* xs, long M, long K, uint8_t* q_row,
                              float* s_row, uint8_t* q_colT, float* s_colT, hipStream_t st) {
    dim3 grid((unsigned)(K / 128), (unsigned)(M / 128));
    hipLaunchKernelGGL((quant_tile_kernel<SRC, ROW, COL, BLOCK>), grid, dim3(256), 0, st, x, xs, M, K,
                       q_row, s_row, q_colT, s_colT);
    return hipGetLastError();
}

hipError_t launch_quant_act(const void* x, const float* xs, int src, long M, long K, uint8_t* q_row,
                            float* s_row, uint8_t* q_colT, float* s_colT, hipStream_t st) {
    const bool row = q_row != nullptr, col = q_colT != nullptr;
    if (src == JET_SRC_BF16) {
        if (row && col) return launch_tile<JET_SRC_BF16, true, true, false>(x, xs, M, K, q_row, s_row, q_colT, s_colT, st);
        if (col) return launch_tile<JET_SRC_BF16, false, true, false>(x, xs, M, K, q_row, s_row, q_colT, s_colT, st);
        return launch_row<JET_SRC_BF16>(x, xs, M, K, q_row, s_row, st);
    }
    if (row && col) return launch_tile<JET_SRC_FP8_ROW, true, true, false>(x, xs, M, K, q_row, s_row, q_colT, s_colT, st);
    if (col) return launch_tile<JET_SRC_FP8_ROW, false, true, false>(x, xs, M, K, q_row, s_row, q_colT, s_colT, st);
    return launch_row<JET_SRC_FP8_ROW>(x, xs, M, K, q_row, s_row, st);
}

hipError_t launch_quant_weight(const void* w, long N, long K, uint8_t* q, float* s, uint8_t* qT,
                               float* sT, hipStream_t st) {
    if (qT) return launch_tile<JET_SRC_BF16, true, true, true>(w, nullptr, N, K, q, s, qT, sT, st);
    return launch_tile<JET_SRC_BF16, true, false, true>(w, nullptr, N, K, q, s, qT, sT, st);
}

}  // namespace jet
