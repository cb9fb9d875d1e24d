// Internal launch interface between the C ABI (jet_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/jet.h"

namespace jet {

// scale layout of the operand that indexes output columns
enum { kSbBlock = 0,  // sb[j/128, g]: 128x128 blocks (FProp, DGrad)
       kSbRow = 1 };  // sb[j, g]    : 1x128 groups   (WGrad)

hipError_t launch_quant_act(const void* x, const float* xs, int src, long M, long K, uint8_t* q_row,
                            float* s_row, uint8_t* q_colT, float* s_colT, hipStream_t st);
hipError_t launch_quant_weight(const void* w, long N, long K, uint8_t* q, float* s, uint8_t* qT,
                               float* sT, hipStream_t st);

// fused producers: h = SiLU(gate) * up or RMSNorm(x), in bf16 semantics, written as 1x128 FP8
hipError_t launch_silu_mul_quant(const void* gate, const void* up, long ld, long M, long K, uint8_t* q,
                                 float* s, hipStream_t st);
// element-wise backward of h = SiLU(gate) * up in bf16 semantics: dgate, dup from dh
hipError_t launch_silu_mul_bwd(const void* gate, const void* up, long ld, const void* dh, long M, long K,
                               void* dgate, void* dup, long ld_out, hipStream_t st);
hipError_t launch_rmsnorm_quant(const void* x, const void* gamma, float eps, long M, long K, uint8_t* q,
                                float* s, hipStream_t st);

// OUT[i,j] = sum_r A[i,r] B[j,r]; A u8 [I,R] with sa f32 [I,R/128]; B u8 [J,R] with sb as
// sb_mode says; out bf16 [I,J].  I >= 1 arbitrary, J % 128 == 0, R % 128 == 0.
hipError_t launch_gemm(const uint8_t* A, const float* sa, const uint8_t* B, const float* sb,
                       int sb_mode, void* out, long I, long J, long R, hipStream_t st);

}  // namespace jet
