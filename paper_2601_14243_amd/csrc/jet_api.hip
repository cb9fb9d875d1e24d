// C ABI of libjet: host-side argument checks, then one kernel launch on the
// caller's stream.  Nothing here allocates, synchronises or keeps a pointer.
#include "jet_internal.h"

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline jet_status after_launch(hipError_t e) { return e == hipSuccess ? JET_OK : JET_ERR_LAUNCH; }

// The launchers report hipGetLastError() after their launch; an error left pending by the caller's
// earlier HIP calls must not be mistaken for this call's, so it is discarded before launching.
inline void discard_stale_error() { (void)hipGetLastError(); }

constexpr int64_t kMaxTileRows = 65535LL * 128;   // the tile quantizers index 128-row tiles with gridDim.y

// shared by the three GEMM entry points: operands (a,sa)[I,R], (b,sb)[J,R], out [I,J]
jet_status gemm_entry(const uint8_t* a, const float* sa, const uint8_t* b, const float* sb, int sb_mode,
                      void* out, int64_t I, int64_t J, int64_t R, bool i_mult_128, void* stream) {
    if (!a || !sa || !b || !sb || !out) return JET_ERR_NULL;
    if (I < 1 || J < 1 || R < 1) return JET_ERR_SHAPE;
    if (J % 128 || R % 128 || (i_mult_128 && I % 128)) return JET_ERR_SHAPE;
    /* kernels form 32-bit byte offsets (row in tile) x R with a 24-bit multiply: reduction length below 2^24 */
    if (I > INT32_MAX / 2 || J > INT32_MAX / 2 || R >= (1 << 24)) return JET_ERR_SHAPE;
    if (misaligned(a) || misaligned(sa) || misaligned(b) || misaligned(sb) || misaligned(out))
        return JET_ERR_ALIGN;
    discard_stale_error();
    return after_launch(jet::launch_gemm(a, sa, b, sb, sb_mode, out, I, J, R, static_cast<hipStream_t>(stream)));
}

}  // namespace

extern "C" {

jet_status jet_quant_act(const void* x, const float* x_scales, jet_src src, int64_t M, int64_t K,
                         uint8_t* q_row, float* s_row, uint8_t* q_colT, float* s_colT, void* stream) {
    if (!x) return JET_ERR_NULL;
    if (src != JET_SRC_BF16 && src != JET_SRC_FP8_ROW) return JET_ERR_ARG;
    if (src == JET_SRC_FP8_ROW && !x_scales) return JET_ERR_ARG;
    const bool any_row = q_row || s_row, any_col = q_colT || s_colT;
    if (!any_row && !any_col) return JET_ERR_ARG;
    if (any_row && (!q_row || !s_row)) return JET_ERR_NULL;
    if (any_col && (!q_colT || !s_colT)) return JET_ERR_NULL;
    if (M < 1 || K < 1) return JET_ERR_SHAPE;
    if (K % 128) return JET_ERR_SHAPE;              /* row groups, FP8-source scales, 128-wide tiles */
    if (any_col && M % 128) return JET_ERR_SHAPE;
    if (M > INT32_MAX / 2 || K > INT32_MAX / 2) return JET_ERR_SHAPE;
    if (any_col && M > kMaxTileRows) return JET_ERR_SHAPE;
    if (misaligned(x) || (src == JET_SRC_FP8_ROW && misaligned(x_scales)) ||
        (any_row && (misaligned(q_row) || misaligned(s_row))) ||
        (any_col && (misaligned(q_colT) || misaligned(s_colT))))
        return JET_ERR_ALIGN;
    discard_stale_error();
    return after_launch(jet::launch_quant_act(x, x_scales, src, M, K, q_row, s_row, q_colT, s_colT,
                                              static_cast<hipStream_t>(stream)));
}

jet_status jet_quant_weight(const void* w, int64_t N, int64_t K, uint8_t* q, float* s, uint8_t* qT,
                            float* sT, void* stream) {
    if (!w || !q || !s) return JET_ERR_NULL;
    if ((qT == nullptr) != (sT == nullptr)) return JET_ERR_ARG;
    if (N < 1 || K < 1 || N % 128 || K % 128) return JET_ERR_SHAPE;
    if (N > kMaxTileRows || K > INT32_MAX / 2) return JET_ERR_SHAPE;
    if (misaligned(w) || misaligned(q) || misaligned(s) || (qT && (misaligned(qT) || misaligned(sT))))
        return JET_ERR_ALIGN;
    discard_stale_error();
    return after_launch(jet::launch_quant_weight(w, N, K, q, s, qT, sT, static_cast<hipStream_t>(stream)));
}

jet_status jet_fp8_linear_fwd(const uint8_t* qx, const float* sx, const uint8_t* qw, const float* sw,
                              void* y, int64_t M, int64_t N, int64_t K, void* stream) {
    return gemm_entry(qx, sx, qw, sw, jet::kSbBlock, y, M, N, K, false, stream);
}

jet_status jet_fp8_linear_dgrad(const uint8_t* qdy, const float* sdy, const uint8_t* qwT,
                                const float* swT, void* dx, int64_t M, int64_t N, int64_t K, void* stream) {
    return gemm_entry(qdy, sdy, qwT, swT, jet::kSbBlock, dx, M, K, N, false, stream);
}

jet_status jet_fp8_linear_wgrad(const uint8_t* qdyT, const float* sdyT, const uint8_t* qxT,
                                const float* sxT, void* dw, int64_t M, int64_t N, int64_t K, void* stream) {
    return gemm_entry(qdyT, sdyT, qxT, sxT, jet::kSbRow, dw, N, K, M, true, stream);
}

jet_status jet_rmsnorm_quant(const void* x, const void* gamma, float eps, int64_t M, int64_t K,
                             uint8_t* q_row, float* s_row, void* stream) {
    if (!x || !gamma || !q_row || !s_row) return JET_ERR_NULL;
    if (!(eps >= 0.0f) || eps > 3.0e38f) return JET_ERR_ARG;   /* negative, NaN or infinite */
    if (M < 1 || K < 1 || K % 128 || K > 32768 || M > INT32_MAX / 2) return JET_ERR_SHAPE;
    if (misaligned(x) || misaligned(gamma) || misaligned(q_row) || misaligned(s_row)) return JET_ERR_ALIGN;
    discard_stale_error();
    return after_launch(jet::launch_rmsnorm_quant(x, gamma, eps, M, K, q_row, s_row, static_cast<hipStream_t>(stream)));
}

jet_status jet_silu_mul_quant(const void* gate, const void* up, int64_t ld, int64_t M, int64_t K,
                              uint8_t* q_row, float* s_row, void* stream) {
    if (!gate || !up || !q_row || !s_row) return JET_ERR_NULL;
    if (M < 1 || K < 1 || K % 128 || ld < K || ld % 8) return JET_ERR_SHAPE;
    if (M > INT32_MAX / 2 || K > INT32_MAX / 2 || ld > INT32_MAX / 2) return JET_ERR_SHAPE;
    if (misaligned(gate) || misaligned(up) || misaligned(q_row) || misaligned(s_row)) return JET_ERR_ALIGN;
    discard_stale_error();
    return after_launch(jet::launch_silu_mul_quant(gate, up, ld, M, K, q_row, s_row, static_cast<hipStream_t>(stream)));
}

jet_status jet_silu_mul_bwd(const void* gate, const void* up, int64_t ld, const void* dh, int64_t M, int64_t K,
                            void* dgate, void* dup, int64_t ld_out, void* stream) {
    if (!gate || !up || !dh || !dgate || !dup) return JET_ERR_NULL;
    if (M < 1 || K < 1 || K % 128 || ld < K || ld % 8 || ld_out < K || ld_out % 8) return JET_ERR_SHAPE;
    if (M > INT32_MAX / 2 || K > INT32_MAX / 2 || ld > INT32_MAX / 2 || ld_out > INT32_MAX / 2) return JET_ERR_SHAPE;
    if (misaligned(gate) || misaligned(up) || misaligned(dh) || misaligned(dgate) || misaligned(dup)) return JET_ERR_ALIGN;
    discard_stale_error();
    return after_launch(jet::launch_silu_mul_bwd(gate, up, ld, dh, M, K, dgate, dup, ld_out, static_cast<hipStream_t>(stream)));
}

const char* jet_status_str(jet_status st) {
    switch (st) {
        case JET_OK: return "ok";
        case JET_ERR_NULL: return "required pointer is NULL";
        case JET_ERR_SHAPE: return "size < 1 or not a multiple of 128 where required";
        case JET_ERR_ALIGN: return "pointer not 16-byte aligned";
        case JET_ERR_ARG: return "bad enum value or inconsistent optional arguments";
        case JET_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

int jet_version(void) { return 101; }

}  // extern "C"
