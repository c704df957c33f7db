// Shared declarations of the GPU library's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/moe.h"

namespace moe {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

void set_error(const char *fmt, ...);
moe_status_t check_launch(const char *what);

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return (float)v; }
__device__ __forceinline__ bf16_t f32_to_bf16(float v) { return (bf16_t)v; }   // round to nearest even

// ---- activation (exact erf form or tanh approximation), evaluated in fp32 ----
__device__ __forceinline__ float act_fwd(float x, int act) {
    if (act == MOE_GELU_TANH) {
        float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
        return 0.5f * x * (1.0f + tanhf(u));
    }
    return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f));
}
__device__ __forceinline__ float act_grad(float x, int act) {
    if (act == MOE_GELU_TANH) {
        float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
        float th = tanhf(u);
        float du = 0.7978845608028654f * (1.0f + 0.134145f * x * x);
        return 0.5f * (1.0f + th) + 0.5f * x * (1.0f - th * th) * du;
    }
    return 0.5f * (1.0f + erff(x * 0.7071067811865476f)) + x * expf(-0.5f * x * x) * 0.3989422804014327f;
}

// ---- grouped GEMM description shared by the fp32 and bf16 kernels ----
// For expert e:  C_e[M_e, N] = opA(A_e)[M_e, K_e] * opB(B_e)[K_e, N]
//   a_xc == 0: A_e stored [M, K] (k contiguous), lda = row length;  a_xc == 1: stored [K, M].
//   b_xc == 1: B_e stored [K, N] (n contiguous);                    b_xc == 0: stored [N, K].
//   rows_from_kept == 1: M_e = kept[e] (K_e = K);  == 0: M_e = M and K_e = kept[e] (weight gradient).
enum { EPI_STORE = 0, EPI_GELU = 1, EPI_DGELU = 2 };
struct GemmDesc {
    const void *A, *B;
    void *C;          // main output
    void *C2;         // EPI_GELU: optional second output act'(pre-activation) (may be null)
    const void *Zin;  // EPI_DGELU: act'(pre-activation) as saved by EPI_GELU; the result is multiplied by it
    const int32_t *kept;
    int64_t strideA, strideB, strideC;   // elements between experts
    int32_t M, N, K;                     // upper bounds / fixed sizes
    int32_t lda, ldb, ldc;
    int32_t E;
    int32_t a_xc, b_xc, rows_from_kept, epi, act;
    void *plan;       // bf16 path: device buffer of gemm_bf16_plan_bytes() bytes holding this launch's tile plan
    // bf16 path, optional fusions of the row permutations (rows_from_kept GEMMs with a KC A operand):
    //   a_index != null: row r of expert e's A operand is row a_index[e*M + r] of the one [a_rows, lda]
    //   array A (dispatch folded into the operand load; strideA is unused);
    //   c_index != null (EPI_STORE): row r of expert e's result, times c_scale[e*M + r] and rounded again, is
    //   also written to row c_index[e*M + r] of C_scatter [*, ldc] (combine folded into the epilogue); C may
    //   then be null.
    //   a_dtd_g = G > 1 (instead of a_index): A is the array of the G row shares of duplicate token dropping,
    //   [G, E, a_dtd_cg, lda]: row r of expert e's operand is row r / G of share r % G (a_rows = G * E * a_dtd_cg).
    const int32_t *a_index;
    int64_t a_rows;
    int32_t a_dtd_g, a_dtd_cg;
    const int32_t *c_index;
    const float *c_scale;
    void *C_scatter;
};

moe_status_t launch_gemm_f32(const GemmDesc &d, hipStream_t s);
// bf16 path: write the tile plans of up to 4 GEMMs in one small launch, then launch each GEMM once
size_t gemm_bf16_plan_bytes(const GemmDesc &d);
moe_status_t launch_gemm_bf16_plans(const GemmDesc *descs, int n, hipStream_t s);
moe_status_t launch_gemm_bf16(const GemmDesc &d, hipStream_t s);

}  // namespace moe
