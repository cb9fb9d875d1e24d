// Block-scaled FP8 GEMMs  OUT[i,j] = sum_r A[i,r] B[j,r]  (Jet-RL Sec. 2.2: FProp,
// DGrad and WGrad all take this form once both operands are stored with the
// reduction axis contiguous, Table 1; operand granularities of Sec. 4.2).
//
// Every kernel here computes an output element with the chain fixed in
// jet_numerics.h: p_g = one 16x16x128 FP8 MFMA over group g (accumulator input 0),
// s_g = sa*sb, acc = fma(p_g, s_g, acc) for g ascending, bf16 RNE.  p_g does not
// depend on any other group, so kernels are free to compute the p_g of different
// groups wherever they like; only the fma chain is ordered.  That keeps a token
// row bit-identical between decode-shaped and training-shaped calls (Sec. 4.1).
#include <mutex>

#include "jet_internal.h"
#include "jet_numerics.h"

namespace jet {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// Lane-linear direct global->LDS copies: lane l's 16 (4) bytes land at lds + 16 l (4 l).
__device__ __forceinline__ void load_to_lds16(const void* g, void* lds) {
    __builtin_amdgcn_global_load_lds((gbl_ptr_t)g, (lds_ptr_t)lds, 16, 0, 0);
}
__device__ __forceinline__ void load_to_lds4(const void* g, void* lds) {
    __builtin_amdgcn_global_load_lds((gbl_ptr_t)g, (lds_ptr_t)lds, 4, 0, 0);
}

// Hardware deals workgroup b to XCD b % 8; give every XCD a contiguous range of
// logical ids so that workgroups sharing operand tiles share an L2.
__device__ __forceinline__ int xcd_contiguous_id(int b, int n) {
    const int x = b & 7, k = b >> 3, q = n >> 3, rem = n & 7;
    return x * q + (x < rem ? x : rem) + k;
}

// ------------------------------------------------------------------------
// Tile kernel: 128x128 output tile per workgroup, 4 waves as 2x2, each wave a
// 64x64 sub-tile = 4x4 MFMA tiles.  Operand tiles of one group (128 rows x 128
// bytes each) are copied global->LDS directly in MFMA fragment order (no VGPR
// staging, conflict-free ds_read_b128), three stages deep.
//
// LDS stage layout: [A tile 16 KB][B tile 16 KB][scales 1 KB]
//   tile: fragment f (rows 16f..16f+15) at f*2048; half h at +h*1024; lane l at +l*16
//         = row (l&15), bytes [64h + 16(l>>4), +16) of the group
//   scales: wave w's 256 B = [sa rows 32w..32w+31][sb rows 32w..32w+31 | block scale]
// ------------------------------------------------------------------------
constexpr int kStages = 3;
constexpr int kTileBytes = 128 * 128;
constexpr int kStageBytes = 2 * kTileBytes + 1024;
constexpr int kLoadsPerStage = 9;  // per wave: 4 A halves, 4 B halves, 1 scale line

template <int SB_MODE>
__global__ __launch_bounds__(256) void gemm_tile_kernel(const uint8_t* __restrict__ A,
                                                        const float* __restrict__ sa,
                                                        const uint8_t* __restrict__ B,
                                                        const float* __restrict__ sb,
                                                        uint16_t* __restrict__ out, int I, int J, int R,
                                                        int tiles_i, int tiles_j) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int t = threadIdx.x, w = t >> 6, l = t & 63, r = l & 15, c4 = l >> 4;
    const int G = R / kGroup;

    // workgroup -> tile: bands of 8 tile rows, walked column by column
    const int lid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    constexpr int kBand = 8;
    const int band = lid / (kBand * tiles_j);
    const int within = lid - band * (kBand * tiles_j);
    const int rows_in_band = min(kBand, tiles_i - band * kBand);
    const int ti = band * kBand + within % rows_in_band;
    const int tj = within / rows_in_band;
    const int i0 = ti * 128, j0 = tj * 128;

    // this wave copies A halves 4w..4w+3 and B halves 4w..4w+3 of every stage
    const uint8_t* ga[4];
    const uint8_t* gb[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int half = 4 * w + x, f = half >> 1, h = half & 1;
        const int row_a = min(i0 + 16 * f + r, I - 1);
        ga[x] = A + (size_t)row_a * R + 64 * h + 16 * c4;
        gb[x] = B + (size_t)(j0 + 16 * f + r) * R + 64 * h + 16 * c4;
    }
    const float* gs;
    if (l < 32) {
        gs = sa + (size_t)min(i0 + 32 * w + l, I - 1) * G;
    } else if (SB_MODE == kSbBlock) {
        gs = sb + (size_t)tj * G;
    } else {
        gs = sb + (size_t)(j0 + 32 * w + (l - 32)) * G;
    }

    auto issue = [&](int g, int slot) {
        uint8_t* st = smem + slot * kStageBytes;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            load_to_lds16(ga[x] + (size_t)g * kGroup, st + (4 * w + x) * 1024);
            load_to_lds16(gb[x] + (size_t)g * kGroup, st + kTileBytes + (4 * w + x) * 1024);
        }
        load_to_lds4(gs + g, st + 2 * kTileBytes + w * 256);
    };

    const int wi = w >> 1, wj = w & 1;
    v4f acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

#pragma unroll
    for (int s = 0; s < kStages - 1; ++s)
        if (s < G) issue(s, s);

    for (int g = 0; g < G; ++g) {
        // group g landed when at most the younger stages' loads are outstanding
        if (g + 1 < G) {
            JET_WAIT_VMCNT(kLoadsPerStage * (kStages - 2));
        } else {
            JET_WAIT_VMCNT(0);
        }
        __syncthreads();
        if (g + kStages - 1 < G) issue(g + kStages - 1, (g + kStages - 1) % kStages);

        const uint8_t* st = smem + (g % kStages) * kStageBytes;
        const uint8_t* sc = st + 2 * kTileBytes;
        v8i xf[4], cf[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint8_t* p = st + (4 * wi + m) * 2048 + l * 16;
            xf[m] = make_frag(*reinterpret_cast<const uint4*>(p), *reinterpret_cast<const uint4*>(p + 1024));
        }
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const uint8_t* p = st + kTileBytes + (4 * wj + n) * 2048 + l * 16;
            cf[n] = make_frag(*reinterpret_cast<const uint4*>(p), *reinterpret_cast<const uint4*>(p + 1024));
        }
        float sai[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int ii = 64 * wi + 16 * m + r;
            sai[m] = *reinterpret_cast<const float*>(sc + (ii >> 5) * 256 + (ii & 31) * 4);
        }
        if (SB_MODE == kSbBlock) {
            const float sbv = *reinterpret_cast<const float*>(sc + 128);
            float s[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) s[m] = sai[m] * sbv;
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const v4f p = group_product(cf[n], xf[m]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[m][n][e] = chain(p[e], s[m], acc[m][n][e]);
                }
        } else {
            v4f sbj[4];
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                const int jj = 64 * wj + 16 * n + 4 * c4;
                sbj[n] = *reinterpret_cast<const v4f*>(sc + (jj >> 5) * 256 + 128 + (jj & 31) * 4);
            }
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const v4f p = group_product(cf[n], xf[m]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[m][n][e] = chain(p[e], sai[m] * sbj[n][e], acc[m][n][e]);
                }
        }
    }

    // epilogue: lane holds 4 consecutive columns of one row per MFMA tile
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int i = i0 + 64 * wi + 16 * m + r;
        if (i < I) {
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                const int j = j0 + 64 * wj + 16 * n + 4 * c4;
                uint2 o;
                o.x = bf16_rne(acc[m][n][0]) | (bf16_rne(acc[m][n][1]) << 16);
                o.y = bf16_rne(acc[m][n][2]) | (bf16_rne(acc[m][n][3]) << 16);
                *reinterpret_cast<uint2*>(out + (size_t)i * J + j) = o;
            }
        }
    }
}

// ------------------------------------------------------------------------
// Skinny kernel for I <= 16 (decode): bound by streaming B (the weights) once.
// One workgroup of 8 waves owns 16 output columns and the whole reduction; the
// waves split the groups, each streaming its weight fragments straight from
// global memory into MFMA registers with a deep prefetch queue.  The p_g and
// s_g of all groups meet in LDS, where waves 0-3 run the ordered fma chain.
// ------------------------------------------------------------------------
constexpr int kSkinnyWaves = 8;
constexpr int kSkinnyPass = 112;                    // groups resident in LDS at once
constexpr int kSkinnyGroupBytes = 4 * 64 * 4 + 64 * 4;  // p[4][64] + s[64]
constexpr int kSkinnyDepth = 8;                     // weight fragments in flight per wave

__global__ __launch_bounds__(512) void gemm_skinny_kernel(const uint8_t* __restrict__ A,
                                                          const float* __restrict__ sa,
                                                          const uint8_t* __restrict__ B,
                                                          const float* __restrict__ sb,
                                                          uint16_t* __restrict__ out, int I, int J, int R) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int t = threadIdx.x, w = t >> 6, l = t & 63, r = l & 15, c4 = l >> 4;
    const int G = R / kGroup;
    const int j0 = blockIdx.x * 16;
    const int ia = min(r, I - 1);

    const uint8_t* gb = B + (size_t)(j0 + r) * R + 16 * c4;
    const uint8_t* ga = A + (size_t)ia * R + 16 * c4;
    const float* gsa = sa + (size_t)ia * G;
    const float* gsb = sb + (size_t)(j0 >> 7) * G;

    float acc = 0.0f;  // waves 0-3: output (row r, column j0 + 4 c4 + w)

    for (int g0 = 0; g0 < G; g0 += kSkinnyPass) {
        const int ng = min(kSkinnyPass, G - g0);
        const int per = (ng + kSkinnyWaves - 1) / kSkinnyWaves;
        const int gbeg = g0 + min(w * per, ng), gend = g0 + min((w + 1) * per, ng);

        if (gbeg < gend) {
            // queue of operand fragments and scales, kSkinnyDepth groups ahead; indices are
            // clamped to the wave's last group, so the tail repeats it (same values, same slot)
            const int last = gend - 1;
            uint4 wlo[kSkinnyDepth], whi[kSkinnyDepth], xlo[kSkinnyDepth], xhi[kSkinnyDepth];
            float qa[kSkinnyDepth], qb[kSkinnyDepth];
            auto fetch = [&](int d, int g) {
                wlo[d] = *reinterpret_cast<const uint4*>(gb + (size_t)g * kGroup);
                whi[d] = *reinterpret_cast<const uint4*>(gb + (size_t)g * kGroup + 64);
                xlo[d] = *reinterpret_cast<const uint4*>(ga + (size_t)g * kGroup);
                xhi[d] = *reinterpret_cast<const uint4*>(ga + (size_t)g * kGroup + 64);
                qa[d] = gsa[g];
                qb[d] = gsb[g];
            };
#pragma unroll
            for (int d = 0; d < kSkinnyDepth; ++d) fetch(d, min(gbeg + d, last));
            for (int gq = gbeg; gq < gend; gq += kSkinnyDepth) {
#pragma unroll
                for (int d = 0; d < kSkinnyDepth; ++d) {
                    const int g = min(gq + d, last);
                    const v4f p = group_product(make_frag(wlo[d], whi[d]), make_frag(xlo[d], xhi[d]));
                    const float s = qa[d] * qb[d];
                    fetch(d, min(gq + d + kSkinnyDepth, last));
                    float* dst = reinterpret_cast<float*>(smem + (g - g0) * kSkinnyGroupBytes);
#pragma unroll
                    for (int e = 0; e < 4; ++e) dst[e * 64 + l] = p[e];
                    dst[256 + l] = s;
                }
            }
        }
        __syncthreads();
        if (w < 4) {
            for (int g = 0; g < ng; ++g) {
                const float* src = reinterpret_cast<const float*>(smem + g * kSkinnyGroupBytes);
                acc = chain(src[w * 64 + l], src[256 + l], acc);
            }
        }
        __syncthreads();
    }
    if (w < 4 && r < I) out[(size_t)r * J + j0 + 4 * c4 + w] = (uint16_t)bf16_rne(acc);
}

// ----------------------------------------------------------------- launch --

template <typename K>
static hipError_t allow_lds(K kernel, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

hipError_t launch_gemm(const uint8_t* A, const float* sa, const uint8_t* B, const float* sb,
                       int sb_mode, void* out, long I, long J, long R, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        hipError_t e = allow_lds(gemm_tile_kernel<kSbBlock>, kStages * kStageBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbRow>, kStages * kStageBytes);
        if (e == hipSuccess) e = allow_lds(gemm_skinny_kernel, kSkinnyPass * kSkinnyGroupBytes);
        attr_err = e;
    });
    if (attr_err != hipSuccess) return attr_err;

    uint16_t* o = static_cast<uint16_t*>(out);
    if (I <= 16 && sb_mode == kSbBlock) {
        hipLaunchKernelGGL(gemm_skinny_kernel, dim3((unsigned)(J / 16)), dim3(512),
                           kSkinnyPass * kSkinnyGroupBytes, st, A, sa, B, sb, o, (int)I, (int)J, (int)R);
        return hipGetLastError();
    }
    const int tiles_i = (int)((I + 127) / 128), tiles_j = (int)(J / 128);
    dim3 grid((unsigned)(tiles_i * tiles_j));
    if (sb_mode == kSbBlock) {
        hipLaunchKernelGGL(gemm_tile_kernel<kSbBlock>, grid, dim3(256), kStages * kStageBytes, st, A, sa,
                           B, sb, o, (int)I, (int)J, (int)R, tiles_i, tiles_j);
    } else {
        hipLaunchKernelGGL(gemm_tile_kernel<kSbRow>, grid, dim3(256), kStages * kStageBytes, st, A, sa, B,
                           sb, o, (int)I, (int)J, (int)R, tiles_i, tiles_j);
    }
    return hipGetLastError();
}

}  // namespace jet
