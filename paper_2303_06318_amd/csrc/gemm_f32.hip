// Grouped fp32 GEMM for the fp32 storage type (true fp32 FMA arithmetic, no reduced-precision
// matrix instructions).  It serves the tiny fp32 workload and tight-tolerance checks of the
// layer's formulas; it is LDS-tiled but not tuned: that workload is launch-latency bound.
#include "moe_common.h"

namespace moe {

constexpr int FT = 64;   // tile edge (M and N)
constexpr int FK = 16;   // k step

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmDesc d) {
    const int e = blockIdx.z;
    const int kept = d.kept[e];
    const int Me = d.rows_from_kept ? kept : d.M;
    const int Ke = d.rows_from_kept ? d.K : kept;
    const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;
    if (m0 >= Me) return;
    const float *A = (const float *)d.A + (int64_t)e * d.strideA;
    const float *B = (const float *)d.B + (int64_t)e * d.strideB;
    float *C = (float *)d.C + (int64_t)e * d.strideC;

    __shared__ float As[FK][FT + 1];
    __shared__ float Bs[FK][FT + 1];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    float acc[4][4] = {};

    for (int k0 = 0; k0 < Ke; k0 += FK) {
        for (int i = tid; i < FT * FK; i += 256) {
            int kk, mm;
            if (d.a_xc) { mm = i % FT; kk = i / FT; } else { kk = i % FK; mm = i / FK; }
            int gm = m0 + mm, gk = k0 + kk;
            float v = 0.f;
            if (gm < Me && gk < Ke) v = d.a_xc ? A[(int64_t)gk * d.lda + gm] : A[(int64_t)gm * d.lda + gk];
            As[kk][mm] = v;
        }
        for (int i = tid; i < FT * FK; i += 256) {
            int kk, nn;
            if (d.b_xc) { nn = i % FT; kk = i / FT; } else { kk = i % FK; nn = i / FK; }
            int gn = n0 + nn, gk = k0 + kk;
            float v = 0.f;
            if (gn < d.N && gk < Ke) v = d.b_xc ? B[(int64_t)gk * d.ldb + gn] : B[(int64_t)gn * d.ldb + gk];
            Bs[kk][nn] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int gm = m0 + ty * 4 + i;
        if (gm >= Me) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn >= d.N) continue;
            int64_t o = (int64_t)gm * d.ldc + gn;
            float v = acc[i][j];
            if (EPI == EPI_GELU) {
                if (d.C2) ((float *)d.C2 + (int64_t)e * d.strideC)[o] = act_grad(v, d.act);
                C[o] = act_fwd(v, d.act);
            } else if (EPI == EPI_DGELU) {
                C[o] = v * ((const float *)d.Zin + (int64_t)e * d.strideC)[o];
            } else {
                C[o] = v;
            }
        }
    }
}

moe_status_t launch_gemm_f32(const GemmDesc &d, hipStream_t s) {
    dim3 grid((d.N + FT - 1) / FT, (d.M + FT - 1) / FT, d.E);
    dim3 block(256);
    switch (d.epi) {
        case EPI_STORE: hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, grid, block, 0, s, d); break;
        case EPI_GELU: hipLaunchKernelGGL(gemm_f32_kernel<EPI_GELU>, grid, block, 0, s, d); break;
        default: hipLaunchKernelGGL(gemm_f32_kernel<EPI_DGELU>, grid, block, 0, s, d); break;
    }
    return check_launch("gemm_f32");
}

}  // namespace moe
