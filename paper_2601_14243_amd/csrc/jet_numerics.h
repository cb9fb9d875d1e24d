// Device-side numerics contract of libjet (gfx950 only).
//
// Everything that decides an output bit lives here, so that every kernel --
// decode-shaped or training-shaped -- takes the same decisions:
//   * the quantizer step  S = amax/448, t = x/S (IEEE binary32), E4M3 RNE with
//     saturation (Jet-RL Sec. 2.1);
//   * the GEMM element chain: one FP8 MFMA over the 128 products of a group,
//     s = sa*sb, acc = fma(p, s, acc), groups ascending, bf16 RNE at the end
//     (Sec. 2.2 on the 1x128 / 128x128 operands of Sec. 4.2);
//   * the assignment of the 128 bytes of a group to MFMA lanes and registers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jet {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kGroup = 128;          // quantization group length (Sec. 4.2)
constexpr float kDeltaMax = 448.0f;  // largest finite E4M3 value (Sec. 2.1)

// ------------------------------------------------------------------ bf16 --

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// binary32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t bf16_rne(float v) {
    uint32_t u = __float_as_uint(v);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// two floats -> two bf16 (round to nearest even) in one dword, low half first: one
// hardware convert for the pair
__device__ __forceinline__ uint32_t bf16_pack2(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ------------------------------------------------------------- quantizer --

// Scale of a group and the data needed to divide by it.
struct GroupScale {
    float S;    // amax / 448, or 1 for an all-zero group
    float r;    // correctly rounded 1/S (used only when `fast`)
    bool fast;  // S far from the binary32 range limits
};

__device__ __forceinline__ GroupScale make_scale(float amax) {
    GroupScale g;
    g.S = (amax == 0.0f) ? 1.0f : amax / kDeltaMax;  // IEEE division
    g.fast = (g.S >= 0x1p-80f) && (g.S <= 0x1p80f);
    g.r = 1.0f / g.S;                                // IEEE division
    return g;
}

// t = x / S, correctly rounded.  With r = RN(1/S), q0 = RN(x r) and two
// fma residual corrections give RN(x/S) (Markstein's division theorem: the
// first correction makes q faithful, the second makes it correctly rounded)
// as long as nothing leaves the normal range, which `fast` guarantees for
// every t that can round to a non-zero code; otherwise the compiler's IEEE
// division sequence is used.  fma(+0, r, -0) would lose the sign of a zero
// input, so the sign of x is copied back.
__device__ __forceinline__ float div_by_scale(float x, const GroupScale& g) {
    if (g.fast) {
        float q = x * g.r;
        float e = __builtin_fmaf(-g.S, q, x);
        q = __builtin_fmaf(e, g.r, q);
        e = __builtin_fmaf(-g.S, q, x);
        q = __builtin_fmaf(e, g.r, q);
        return __builtin_copysignf(q, x);
    }
    return x / g.S;
}

// Four binary32 values -> four E4M3 codes (little-endian in the result).
// The hardware convert rounds to nearest even, also into the subnormal range,
// and keeps the sign of zero; it does not saturate, so the value is clamped to
// +-448 first (every value in (448, 464) rounds to 448 anyway).
__device__ __forceinline__ uint32_t e4m3_pack4(float a, float b, float c, float d) {
    a = __builtin_amdgcn_fmed3f(a, -kDeltaMax, kDeltaMax);
    b = __builtin_amdgcn_fmed3f(b, -kDeltaMax, kDeltaMax);
    c = __builtin_amdgcn_fmed3f(c, -kDeltaMax, kDeltaMax);
    d = __builtin_amdgcn_fmed3f(d, -kDeltaMax, kDeltaMax);
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (uint32_t)w;
}

// Four E4M3 codes of one dword -> binary32 (exact).
__device__ __forceinline__ void e4m3_unpack4(uint32_t w, float& a, float& b, float& c, float& d) {
    typedef float v2f __attribute__((ext_vector_type(2)));
    v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    v2f hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    a = lo[0]; b = lo[1]; c = hi[0]; d = hi[1];
}

// max over a team of 8 / 16 consecutive lanes (all lanes of the team get it).
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
    int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return fmaxf(v, __int_as_float(o));
}
__device__ __forceinline__ float team8_max(float v) {
    v = dpp_max<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_max<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_max<0x141>(v);  // row_half_mirror
    return v;
}
__device__ __forceinline__ float team16_max(float v) {
    v = team8_max(v);
    v = dpp_max<0x140>(v);  // row_mirror
    return v;
}

// ------------------------------------------------------------------ GEMM --

// MFMA operand fragment of one 16-row x 128-byte group tile.  Lane l serves
// row (l & 15) and 16-byte chunk column c4 = l >> 4: registers 0-3 hold bytes
// [16 c4, 16 c4 + 16) and registers 4-7 hold bytes [64 + 16 c4, 64 + 16 c4 + 16)
// of that row's 128-byte group.  Every kernel loads both operands this way, so
// a given pair of rows always meets the matrix core in the same arrangement.
__device__ __forceinline__ v8i make_frag(uint4 lo, uint4 hi) {
    v8i f = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    return f;
}

// Partial sums of one group for a 16x16 output tile of OUT[i,j] = sum_r A[i,r] B[j,r]:
// p[t] belongs to (B row 4*(lane>>4)+t, A row lane&15).  The operand that indexes
// output columns (the weight in FProp and DGrad, X^T in WGrad) always goes first and
// the operand that indexes output rows second, in every kernel.
__device__ __forceinline__ v4f group_product(v8i col_frag, v8i row_frag) {
    v4f z = {0.0f, 0.0f, 0.0f, 0.0f};
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(col_frag, row_frag, z, 0, 0, 0, 0, 0, 0);
}

// One step of the scaled accumulation chain.
__device__ __forceinline__ float chain(float p, float s, float acc) { return __builtin_fmaf(p, s, acc); }

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding).
#define JET_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | (((n) >> 4) << 14) | (0x7 << 4) | (0xf << 8))

}  // namespace jet
