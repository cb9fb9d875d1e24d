/*
 * jet_oracle.c -- CPU oracle for the block-scaled FP8 linear layer of Jet-RL.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a slow, plain, obviously
 * correct host implementation of what the GPU library computes, written from the
 * paper (Jet-RL, Sec. 2.1 "Quantization Basis", Sec. 2.2 "Quantization of a
 * Linear Layer", Sec. 4.2 "Granularity of GEMM Quantization") and from the OCP
 * 8-bit floating point specification the paper cites for E4M3.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may call it.  It
 * shares no code, header, table or constant generator with the HIP path.
 *
 * Every pointer is a HOST pointer.  All matrices are dense row-major.
 * bf16 values travel as uint16_t (the upper half of the IEEE binary32 pattern).
 *
 * Pins (tests/test_oracle_*.py): all 256 E4M3 codes, hand-worked tie table,
 * torch's float8_e4m3fn CPU conversion, exhaustive bf16-amax scale sweep,
 * lossless integer GEMM against int64 arithmetic, exact rational brute force
 * on tiny shapes, fp64 dequantise-then-matmul, transpose / permutation /
 * power-of-two metamorphic invariants; for the fused producers: closed forms
 * (one-hot rows, constant rows, scale invariance), a binary64 numpy evaluation,
 * and torch's binary64 silu over every finite bf16 input; for its backward: binary64 autograd of
 * torch over every finite bf16 gate value, finite differences, closed forms at 0 and +-infinity.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -fPIC -shared (no -ffast-math: every
 * division, multiplication and fma below must be the IEEE binary32 operation).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#include <stddef.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_NULL 1
#define ORC_ERR_SHAPE 2
#define ORC_ERR_ARG 4
#define ORC_ERR_NONFINITE 6

#define ORC_SRC_BF16 0
#define ORC_SRC_FP8_ROW 1

/* scale layout of the second GEMM operand */
#define ORC_SB_BLOCK 0 /* sb[j/128, g]  : 128x128 blocks (FProp, DGrad) */
#define ORC_SB_ROW 1   /* sb[j, g]      : 1x128 groups   (WGrad)        */

#define GROUP 128
/* Delta_max of E4M3 (Sec. 2.1). */
static const float DELTA_MAX = 448.0f;

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the row loops may use from now on (timing the oracle at one thread and at all). */
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------------------------------------------------------------- bf16 -- */

float orc_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* binary32 -> bf16, round to nearest, ties to even ("output BF16", Sec. 4.2).
 * Written as arithmetic on the value, not as a bit trick: the bf16 neighbours
 * of v are found by truncation and the nearer one is chosen in double. */
uint16_t orc_bf16_rne(float v) {
    uint32_t u;
    memcpy(&u, &v, 4);
    if (isnan(v)) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lo_bits = u & 0xFFFF0000u;          /* toward zero */
    uint32_t hi_bits = lo_bits + 0x00010000u;    /* next bf16 away from zero (may be inf) */
    float lo, hi;
    memcpy(&lo, &lo_bits, 4);
    memcpy(&hi, &hi_bits, 4);
    if (lo == v) return (uint16_t)(lo_bits >> 16);
    double dl = fabs((double)v - (double)lo);
    double dh = isinf(hi) ? fabs(ldexp(1.0, 128) - fabs((double)v)) : fabs((double)hi - (double)v);
    if (dl < dh) return (uint16_t)(lo_bits >> 16);
    if (dh < dl) return (uint16_t)(hi_bits >> 16);
    /* tie: even mantissa */
    return (uint16_t)(((lo_bits >> 16) & 1u) ? (hi_bits >> 16) : (lo_bits >> 16));
}

/* ---------------------------------------------------------------- E4M3 -- */

/* OCP OFP8 E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities;
 * S.1111.111 is NaN; exponent field 0 is subnormal with quantum 2^-9;
 * largest finite value 448 (= Delta_max, Sec. 2.1). */
float orc_e4m3_decode(uint8_t b) {
    int sign = b >> 7;
    int e = (b >> 3) & 15;
    int m = b & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) mag = ldexp((double)m, -9);
    else mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return (float)(sign ? -mag : mag);
}

/* Round the exact value of t to the nearest E4M3 value, ties to the even
 * mantissa, one rounding (also into the subnormal range); results beyond the
 * largest finite value saturate to +-448; the sign is kept even when the
 * magnitude rounds to zero.  The rounding bracket of Sec. 2.1. */
uint8_t orc_e4m3_encode(float t) {
    uint32_t u;
    memcpy(&u, &t, 4);
    uint8_t sign = (uint8_t)((u >> 31) << 7);
    if (isnan(t)) return (uint8_t)(sign | 0x7F);
    double a = fabs((double)t);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);       /* a = f * 2^ex, f in [0.5,1)  =>  floor(log2 a) = ex-1 */
    int e = ex - 1;
    if (e < -6) e = -6;        /* subnormal range shares the quantum of the lowest binade */
    double quantum = ldexp(1.0, e - 3);
    double n = nearbyint(a / quantum); /* exact scaling, then RNE to an integer */
    double r = n * quantum;            /* the rounded magnitude, exact */
    if (r > 448.0) return (uint8_t)(sign | 0x7E);
    if (r == 0.0) return sign;
    /* r is exactly representable: read its fields off */
    (void)frexp(r, &ex);
    int re = ex - 1;
    if (re < -6) { /* subnormal: r = m * 2^-9 */
        int m = (int)ldexp(r, 9);
        return (uint8_t)(sign | m);
    }
    int m = (int)(ldexp(r, -re) * 8.0) - 8; /* (1+m/8) * 2^re */
    return (uint8_t)(sign | ((re + 7) << 3) | m);
}

/* ---------------------------------------------------------- quantizers -- */

/* Scale of one group: S = max|X| / Delta_max (Sec. 2.1), one binary32
 * division.  Reading for a group of zeros (0/0 in the formula): S = 1. */
static float group_scale(float amax) {
    if (amax == 0.0f) return 1.0f;
    volatile float s = amax / DELTA_MAX;
    return s;
}

static uint8_t quant_elem(float v, float S) {
    volatile float t = v / S; /* X / S_X, one binary32 division */
    return orc_e4m3_encode(t);
}

/* value of source element (m,k) as binary32 */
static float src_value(const void* x, const float* xs, int src, int64_t K, int64_t m, int64_t k) {
    if (src == ORC_SRC_BF16) return orc_bf16_to_f32(((const uint16_t*)x)[m * K + k]);
    /* FP8-saved activation (Sec. 4.1): dequantised value q * s, one binary32 multiply */
    volatile float v = orc_e4m3_decode(((const uint8_t*)x)[m * K + k]) * xs[m * (K / GROUP) + k / GROUP];
    return v;
}

/* 1x128 per-group quantization of activations / gradients (Sec. 4.2).
 *   row outputs : groups of 128 consecutive k in one row m  -> q_row[M,K], s_row[M,K/128]
 *   colT outputs: groups of 128 consecutive m in one column k, stored transposed
 *                 -> q_colT[K,M], s_colT[K,M/128]   (the 128x1 scheme of WGrad)
 * Either output pair may be NULL. */
int orc_quant_act(const void* x, const float* x_scales, int src, int64_t M, int64_t K,
                  uint8_t* q_row, float* s_row, uint8_t* q_colT, float* s_colT) {
    if (!x) return ORC_ERR_NULL;
    if (src != ORC_SRC_BF16 && src != ORC_SRC_FP8_ROW) return ORC_ERR_ARG;
    if (src == ORC_SRC_FP8_ROW && !x_scales) return ORC_ERR_ARG;
    int want_row = (q_row != NULL) || (s_row != NULL);
    int want_col = (q_colT != NULL) || (s_colT != NULL);
    if (!want_row && !want_col) return ORC_ERR_ARG;
    if (want_row && (!q_row || !s_row)) return ORC_ERR_NULL;
    if (want_col && (!q_colT || !s_colT)) return ORC_ERR_NULL;
    if (M < 1 || K < 1) return ORC_ERR_SHAPE;
    if (want_row && K % GROUP) return ORC_ERR_SHAPE;
    if (src == ORC_SRC_FP8_ROW && K % GROUP) return ORC_ERR_SHAPE;
    if (want_col && M % GROUP) return ORC_ERR_SHAPE;

    int bad = 0;
    if (want_row) {
        int64_t G = K / GROUP;
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t m = 0; m < M; ++m) {
            for (int64_t g = 0; g < G; ++g) {
                float amax = 0.0f;
                for (int64_t k = g * GROUP; k < (g + 1) * GROUP; ++k) {
                    float v = src_value(x, x_scales, src, K, m, k);
                    if (!isfinite(v)) bad = 1;
                    float a = fabsf(v);
                    if (a > amax) amax = a;
                }
                float S = group_scale(amax);
                s_row[m * G + g] = S;
                for (int64_t k = g * GROUP; k < (g + 1) * GROUP; ++k)
                    q_row[m * K + k] = quant_elem(src_value(x, x_scales, src, K, m, k), S);
            }
        }
    }
    if (want_col) {
        int64_t G = M / GROUP;
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t k = 0; k < K; ++k) {
            for (int64_t g = 0; g < G; ++g) {
                float amax = 0.0f;
                for (int64_t m = g * GROUP; m < (g + 1) * GROUP; ++m) {
                    float v = src_value(x, x_scales, src, K, m, k);
                    if (!isfinite(v)) bad = 1;
                    float a = fabsf(v);
                    if (a > amax) amax = a;
                }
                float S = group_scale(amax);
                s_colT[k * G + g] = S;
                for (int64_t m = g * GROUP; m < (g + 1) * GROUP; ++m)
                    q_colT[k * M + m] = quant_elem(src_value(x, x_scales, src, K, m, k), S);
            }
        }
    }
    return bad ? ORC_ERR_NONFINITE : ORC_OK;
}

/* 128x128 per-block quantization of weights (Sec. 4.2).  w bf16 [N,K] ->
 * q[N,K], s[N/128,K/128]; optional transposed copy qT[K,N], sT[K/128,N/128]
 * holding the same codes and scales (the scheme is symmetric under transpose,
 * so the backward pass only transposes). */
int orc_quant_weight(const uint16_t* w, int64_t N, int64_t K, uint8_t* q, float* s, uint8_t* qT,
                     float* sT) {
    if (!w || !q || !s) return ORC_ERR_NULL;
    if ((qT == NULL) != (sT == NULL)) return ORC_ERR_NULL;
    if (N < 1 || K < 1 || N % GROUP || K % GROUP) return ORC_ERR_SHAPE;
    int64_t NB = N / GROUP, KB = K / GROUP;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t nb = 0; nb < NB; ++nb) {
        for (int64_t kb = 0; kb < KB; ++kb) {
            float amax = 0.0f;
            for (int64_t n = nb * GROUP; n < (nb + 1) * GROUP; ++n)
                for (int64_t k = kb * GROUP; k < (kb + 1) * GROUP; ++k) {
                    float v = orc_bf16_to_f32(w[n * K + k]);
                    if (!isfinite(v)) bad = 1;
                    float a = fabsf(v);
                    if (a > amax) amax = a;
                }
            float S = group_scale(amax);
            s[nb * KB + kb] = S;
            if (sT) sT[kb * NB + nb] = S;
            for (int64_t n = nb * GROUP; n < (nb + 1) * GROUP; ++n)
                for (int64_t k = kb * GROUP; k < (kb + 1) * GROUP; ++k) {
                    uint8_t c = quant_elem(orc_bf16_to_f32(w[n * K + k]), S);
                    q[n * K + k] = c;
                    if (qT) qT[k * N + n] = c;
                }
        }
    }
    return bad ? ORC_ERR_NONFINITE : ORC_OK;
}

/* ---------------------------------------------------------------- GEMM -- */

/* One output element of  OUT[i,j] = sum_r A[i,r] * B[j,r]  on block-scaled FP8
 * operands (the three GEMMs of Sec. 2.2 all have this shape once each operand
 * is stored with the reduction axis contiguous, Table 1).
 *
 * Reference order: within each group of 128 the products (exact in binary32)
 * are added one by one in ascending r into a binary32 partial sum p starting
 * from 0; the group's scale s = sa * sb is one binary32 product; the running
 * result is acc = fma(p, s, acc), groups ascending.
 *
 * Exact companion: the group sum as an integer in units of 2^-18 (every E4M3
 * value is a multiple of 2^-9), times s, summed over groups in long double.
 * sum_abs = sum_g |s_g * p_g(exact)| measures cancellation across groups,
 * sum_abs_prod = sum_g s_g * sum_r |a_r b_r| cancellation down to single products. */
/* decode(b) for all 256 codes, filled from orc_e4m3_decode (a lookup of the
 * definition, so that sampled checks at the large shapes finish in seconds);
 * TABI holds the same values as integers in units of 2^-9. */
static float TAB[256];
static int32_t TABI[256];
static void fill_tables(void) {
    for (int c = 0; c < 256; ++c) {
        float v = orc_e4m3_decode((uint8_t)c);
        TAB[c] = v;
        TABI[c] = isnan(v) ? 0 : (int32_t)lrint(ldexp((double)v, 9));
    }
}

static void gemm_elem(const uint8_t* a, const float* sa, const uint8_t* b, const float* sb,
                      int64_t R, float* acc_out, double* exact_out, double* sum_abs_out,
                      double* sum_abs_prod_out) {
    int64_t G = R / GROUP;
    float acc = 0.0f;
    long double ex = 0.0L, sabs = 0.0L, sprod = 0.0L;
    for (int64_t g = 0; g < G; ++g) {
        volatile float p = 0.0f;
        int64_t pi = 0, pa = 0;
        for (int64_t r = g * GROUP; r < (g + 1) * GROUP; ++r) {
            float va = TAB[a[r]];
            float vb = TAB[b[r]];
            volatile float prod = va * vb; /* exact: two 4-bit significands */
            p = p + prod;
            pi += (int64_t)TABI[a[r]] * (int64_t)TABI[b[r]];
            pa += llabs((int64_t)TABI[a[r]] * (int64_t)TABI[b[r]]);
        }
        volatile float s = sa[g] * sb[g];
        acc = fmaf(p, s, acc);
        long double term = (long double)s * ldexpl((long double)pi, -18);
        ex += term;
        sabs += fabsl(term);
        sprod += fabsl((long double)s) * ldexpl((long double)pa, -18);
    }
    *acc_out = acc;
    if (exact_out) *exact_out = (double)ex;
    if (sum_abs_out) *sum_abs_out = (double)sabs;
    if (sum_abs_prod_out) *sum_abs_prod_out = (double)sprod;
}

/* Sampled / full GEMM.  a u8 [I,R], sa f32 [I,R/128]; b u8 [J,R];
 * sb f32 [J/128,R/128] (ORC_SB_BLOCK) or [J,R/128] (ORC_SB_ROW).
 * rows / cols: index lists into I / J, or NULL for all of them.
 * Outputs (each may be NULL), compact [nrows, ncols] row-major:
 *   acc  binary32 reference-order result      out_bf16  its bf16 rounding
 *   exact  order-independent value (double)   sum_abs   sum_g |s_g p_g|
 *   sum_abs_prod  sum_g s_g sum_r |a_r b_r|                                  */
int orc_gemm(const uint8_t* a, const float* sa, const uint8_t* b, const float* sb, int sb_mode,
             int64_t I, int64_t J, int64_t R, const int64_t* rows, int64_t nrows,
             const int64_t* cols, int64_t ncols, float* acc, uint16_t* out_bf16, double* exact,
             double* sum_abs, double* sum_abs_prod) {
    if (!a || !sa || !b || !sb) return ORC_ERR_NULL;
    if (I < 1 || J < 1 || R < 1 || R % GROUP) return ORC_ERR_SHAPE;
    if (sb_mode == ORC_SB_BLOCK && J % GROUP) return ORC_ERR_SHAPE;
    if (sb_mode != ORC_SB_BLOCK && sb_mode != ORC_SB_ROW) return ORC_ERR_ARG;
    if (!rows) nrows = I;
    if (!cols) ncols = J;
    int64_t G = R / GROUP;
    fill_tables();
    for (int64_t x = 0; rows && x < nrows; ++x)
        if (rows[x] < 0 || rows[x] >= I) return ORC_ERR_ARG;
    for (int64_t x = 0; cols && x < ncols; ++x)
        if (cols[x] < 0 || cols[x] >= J) return ORC_ERR_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t ii = 0; ii < nrows; ++ii) {
        int64_t i = rows ? rows[ii] : ii;
        for (int64_t jj = 0; jj < ncols; ++jj) {
            int64_t j = cols ? cols[jj] : jj;
            const float* sbp = (sb_mode == ORC_SB_BLOCK) ? sb + (j / GROUP) * G : sb + j * G;
            float v;
            double e, sa_abs, sa_prod;
            gemm_elem(a + i * R, sa + i * G, b + j * R, sbp, R, &v, &e, &sa_abs, &sa_prod);
            int64_t o = ii * ncols + jj;
            if (acc) acc[o] = v;
            if (out_bf16) out_bf16[o] = orc_bf16_rne(v);
            if (exact) exact[o] = e;
            if (sum_abs) sum_abs[o] = sa_abs;
            if (sum_abs_prod) sum_abs_prod[o] = sa_prod;
        }
    }
    return ORC_OK;
}

/* FProp  Y[M,N] = X W^T :  (qx,sx)[M,K] 1x128 along K,  (qw,sw)[N,K] 128x128. */
int orc_fp8_linear_fwd(const uint8_t* qx, const float* sx, const uint8_t* qw, const float* sw,
                       int64_t M, int64_t N, int64_t K, float* acc, uint16_t* y) {
    return orc_gemm(qx, sx, qw, sw, ORC_SB_BLOCK, M, N, K, NULL, 0, NULL, 0, acc, y, NULL, NULL, NULL);
}

/* DGrad  dX[M,K] = dY W :  (qdy,sdy)[M,N] 1x128 along N,  (qwT,swT)[K,N] 128x128. */
int orc_fp8_linear_dgrad(const uint8_t* qdy, const float* sdy, const uint8_t* qwT,
                         const float* swT, int64_t M, int64_t N, int64_t K, float* acc,
                         uint16_t* dx) {
    return orc_gemm(qdy, sdy, qwT, swT, ORC_SB_BLOCK, M, K, N, NULL, 0, NULL, 0, acc, dx, NULL,
                    NULL, NULL);
}

/* WGrad  dW[N,K] = dY^T X :  (qdyT,sdyT)[N,M] and (qxT,sxT)[K,M], both in
 * groups of 128 along the token axis. */
int orc_fp8_linear_wgrad(const uint8_t* qdyT, const float* sdyT, const uint8_t* qxT,
                         const float* sxT, int64_t M, int64_t N, int64_t K, float* acc,
                         uint16_t* dw) {
    return orc_gemm(qdyT, sdyT, qxT, sxT, ORC_SB_ROW, N, K, M, NULL, 0, NULL, 0, acc, dw, NULL,
                    NULL, NULL);
}

/* ------------------------------------------------------ fused producers -- */

/* The paper fuses the 1x128 activation quantization with the operator in front of
 * the GEMM (Sec. 4.2) and names RMSNorm and the activation function as those
 * operators (Sec. 4.3); it does not spell out their arithmetic.  The reading taken
 * here is the usual bf16 module semantics: the operator produces a bf16 tensor h,
 * and h is then quantized exactly as any other activation (orc_quant_act).  The
 * functions below produce h; the tests chain them with orc_quant_act. */

/* double -> bf16, one rounding to nearest (ties to even), also into the bf16
 * subnormal range (quantum 2^-133); magnitudes that round to 2^128 give infinity. */
uint16_t orc_bf16_from_double(double v) {
    uint16_t sign = (uint16_t)(signbit(v) ? 0x8000u : 0u);
    if (isnan(v)) return (uint16_t)(sign | 0x7FC0u);
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    int ex;
    (void)frexp(a, &ex);
    int e = ex - 1;                       /* floor(log2 a) */
    if (e < -126) e = -126;
    double quantum = ldexp(1.0, e - 7);   /* spacing of bf16 values in this binade */
    double r = nearbyint(a / quantum) * quantum;   /* exact scaling, RNE to an integer, exact product */
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    float f = (float)r;                   /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(sign | (u >> 16));
}

/* RMSNorm:  h[m,k] = bf16( gamma[k] * bf16( x[m,k] * r[m] ) ),
 *           r[m]   = 1 / sqrt( mean_k x[m,k]^2 + eps ).
 * The mean is formed in binary64 (every square of a bf16 value is exact there) and
 * rounded once to binary32; adding eps, the square root, the reciprocal and the two
 * products are single binary32 operations; both bf16 roundings are to nearest even. */
int orc_rmsnorm(const uint16_t* x, const uint16_t* gamma, float eps, int64_t M, int64_t K, uint16_t* h) {
    if (!x || !gamma || !h) return ORC_ERR_NULL;
    if (M < 1 || K < 1) return ORC_ERR_SHAPE;
    if (!(eps >= 0.0f) || !isfinite(eps)) return ORC_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = (double)orc_bf16_to_f32(x[m * K + k]);
            if (!isfinite(v)) bad = 1;
            ss += v * v;
        }
        volatile float ms = (float)(ss / (double)K);
        volatile float d = ms + eps;
        volatile float rt = sqrtf(d);
        volatile float r = 1.0f / rt;
        if (!isfinite(r) || !isfinite(ms)) bad = 1;   /* an all-zero row with eps = 0; a mean beyond binary32 */
        for (int64_t k = 0; k < K; ++k) {
            volatile float n = orc_bf16_to_f32(x[m * K + k]) * r;
            float nb = orc_bf16_to_f32(orc_bf16_rne(n));
            volatile float t = orc_bf16_to_f32(gamma[k]) * nb;
            h[m * K + k] = orc_bf16_rne(t);
        }
    }
    return bad ? ORC_ERR_NONFINITE : ORC_OK;
}

/* SiLU(gate) * up:  a = bf16( g / (1 + e^-g) )  (the real function, rounded once),
 *                   h = bf16( a * u )           (binary32 product, rounded to bf16).
 * gate and up are bf16 [M,K] with a common row stride ld >= K (in elements), so that the
 * two halves of a fused gate/up projection output can be passed without a copy. */
uint16_t orc_silu_bf16(uint16_t g_bits) {
    double g = (double)orc_bf16_to_f32(g_bits);
    return orc_bf16_from_double(g / (1.0 + exp(-g)));
}

int orc_silu_mul(const uint16_t* gate, const uint16_t* up, int64_t ld, int64_t M, int64_t K, uint16_t* h) {
    if (!gate || !up || !h) return ORC_ERR_NULL;
    if (M < 1 || K < 1 || ld < K) return ORC_ERR_SHAPE;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t k = 0; k < K; ++k) {
            float g = orc_bf16_to_f32(gate[m * ld + k]), u = orc_bf16_to_f32(up[m * ld + k]);
            if (!isfinite(g) || !isfinite(u)) bad = 1;
            float a = orc_bf16_to_f32(orc_silu_bf16(gate[m * ld + k]));
            volatile float t = a * u;
            if (!isfinite(t)) bad = 1;
            h[m * K + k] = orc_bf16_rne(t);
        }
    }
    return bad ? ORC_ERR_NONFINITE : ORC_OK;
}

/* Backward of h = bf16( bf16(silu(g)) * u ) for the MLP block whose saved activations are FP8
 * (Sec. 4.1: the tensors saved for the GEMMs of the backward pass are the FP8 ones, while the
 * gradients that travel between operators stay BF16).  The element-wise operator between the
 * down projection and the gate/up projections receives dh in bf16 and returns dgate and dup in
 * bf16; the paper does not spell out its arithmetic.  Reading, bf16 module semantics as in the
 * forward: with a = bf16(silu(g)) as the forward formed it,
 *     dup   = bf16( dh * a )                    (the product of two bf16 values is exact in binary32)
 *     da    = bf16( dh * u )
 *     dgate = bf16( da * silu'(g) ),  silu'(g) = s (1 + g (1 - s)),  s = 1 / (1 + e^-g),
 * the real value of da * silu'(g) rounded once (evaluated in binary64).
 * gate, up: bf16 [M,K] with row stride ld; dh: bf16 [M,K] dense; dgate, dup: bf16 [M,K] with row
 * stride ld_out (the two halves of one [M,2K] gradient tensor can be written in place). */
double orc_silu_grad(double g) {
    double s = 1.0 / (1.0 + exp(-g));
    return s * (1.0 + g * (1.0 - s));
}

int orc_silu_mul_bwd(const uint16_t* gate, const uint16_t* up, int64_t ld, const uint16_t* dh,
                     int64_t M, int64_t K, uint16_t* dgate, uint16_t* dup, int64_t ld_out) {
    if (!gate || !up || !dh || !dgate || !dup) return ORC_ERR_NULL;
    if (M < 1 || K < 1 || ld < K || ld_out < K) return ORC_ERR_SHAPE;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t k = 0; k < K; ++k) {
            float g = orc_bf16_to_f32(gate[m * ld + k]), u = orc_bf16_to_f32(up[m * ld + k]);
            float d = orc_bf16_to_f32(dh[m * K + k]);
            if (!isfinite(g) || !isfinite(u) || !isfinite(d)) bad = 1;
            float a = orc_bf16_to_f32(orc_silu_bf16(gate[m * ld + k]));
            volatile float pu = d * a;
            volatile float pa = d * u;
            if (!isfinite(pu) || !isfinite(pa)) bad = 1;
            dup[m * ld_out + k] = orc_bf16_rne(pu);
            double da = (double)orc_bf16_to_f32(orc_bf16_rne(pa));
            dgate[m * ld_out + k] = orc_bf16_from_double(da * orc_silu_grad((double)g));
        }
    }
    return bad ? ORC_ERR_NONFINITE : ORC_OK;
}

/* vector helpers for the tests */
void orc_e4m3_encode_n(const float* t, uint8_t* out, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = orc_e4m3_encode(t[i]);
}
void orc_e4m3_decode_n(const uint8_t* b, float* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_e4m3_decode(b[i]);
}
void orc_bf16_rne_n(const float* v, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_rne(v[i]);
}
