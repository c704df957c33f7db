// HBM-streaming row movers: dispatch, combine and their backward.
// Every kernel moves whole rows with 16-byte accesses; one workgroup handles one row at a time.
#include "moe_common.h"

namespace moe {

template <typename T> struct Vec;    // 16-byte vector of the storage type
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void unpack(const u32x4 &v, float *o) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = __uint_as_float(v[i]);
    }
    __device__ static u32x4 pack(const float *o) {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __float_as_uint(o[i]);
        return v;
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void unpack(const u32x4 &v, float *o) {
        bf16x8 b = __builtin_bit_cast(bf16x8, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = (float)b[i];
    }
    __device__ static u32x4 pack(const float *o) {
        bf16x8 b;
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = (bf16_t)o[i];
        return __builtin_bit_cast(u32x4, b);
    }
};

// buf[r,:] = x[token_of_slot[r],:] for filled slots; empty slots are left alone (no later step reads
// them).  Pure copy: works on 16-byte words of any type.
__global__ __launch_bounds__(256) void dispatch_kernel(const u32x4 *x, const int32_t *token_of_slot, u32x4 *buf,
                                                        int64_t rows, int words) {
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const int tok = token_of_slot[r];
        if (tok < 0) continue;
        u32x4 *dst = buf + r * words;
        const u32x4 *src = x + (int64_t)tok * words;
        for (int i = threadIdx.x; i < words; i += 256) dst[i] = src[i];
    }
}

// ---- duplicate token dropping: rank r of a tensor-parallel group of G keeps rows r, r + G, ... of every
// expert chunk (row s of the chunk is row s / G of share s % G); shares are [E, Cg, words], Cg = ceil(C / G).

// dispatch fused with the drop: share[e, j, :] = x[token_of_slot[e, j G + r], :] for filled slots
__global__ __launch_bounds__(256) void dispatch_dtd_kernel(const u32x4 *x, const int32_t *token_of_slot, u32x4 *share,
                                                            int64_t rows, int64_t C, int64_t Cg, int G, int r, int words) {
    for (int64_t q = blockIdx.x; q < rows; q += gridDim.x) {
        const int64_t e = q / Cg, s = (q - e * Cg) * G + r;
        if (s >= C) continue;
        const int tok = token_of_slot[e * C + s];
        if (tok < 0) continue;
        u32x4 *dst = share + q * words;
        const u32x4 *src = x + (int64_t)tok * words;
        for (int i = threadIdx.x; i < words; i += 256) dst[i] = src[i];
    }
}

// the drop alone: share[e, j, :] = buf[e, j G + r, :] for j G + r < kept[e]
__global__ __launch_bounds__(256) void dtd_drop_kernel(const u32x4 *buf, const int32_t *kept, u32x4 *share, int64_t rows,
                                                        int64_t C, int64_t Cg, int G, int r, int words) {
    for (int64_t q = blockIdx.x; q < rows; q += gridDim.x) {
        const int64_t e = q / Cg, s = (q - e * Cg) * G + r;
        if (s >= kept[e]) continue;
        u32x4 *dst = share + q * words;
        const u32x4 *src = buf + (e * C + s) * words;
        for (int i = threadIdx.x; i < words; i += 256) dst[i] = src[i];
    }
}

// the shares of all G ranks put back in row order: buf[e, s, :] = shares[s % G][e, s / G, :] for s < kept[e]
__global__ __launch_bounds__(256) void dtd_gather_kernel(const u32x4 *shares, const int32_t *kept, u32x4 *buf,
                                                          int64_t rows, int64_t C, int64_t Cg, int G, int E, int words) {
    for (int64_t q = blockIdx.x; q < rows; q += gridDim.x) {
        const int64_t e = q / C, s = q - e * C;
        if (s >= kept[e]) continue;
        u32x4 *dst = buf + q * words;
        const u32x4 *src = shares + (((s % G) * E + e) * Cg + s / G) * words;
        for (int i = threadIdx.x; i < words; i += 256) dst[i] = src[i];
    }
}

// dst[t,:] = src[expert[t], slot[t], :] or 0 (dispatch backward).  G > 1: src holds the G shares
// [G, E, Cg, words] of duplicate token dropping instead of whole chunks (G = 1, Cg = C: the plain layout).
__global__ __launch_bounds__(256) void gather_rows_kernel(const u32x4 *src, const int32_t *expert, const int32_t *slot,
                                                           u32x4 *dst, int64_t T, int64_t Cg, int G, int E, int words) {
    for (int64_t t = blockIdx.x; t < T; t += gridDim.x) {
        const int s = slot[t];
        u32x4 *o = dst + t * words;
        if (s >= 0) {
            const u32x4 *p = src + (((int64_t)(s % G) * E + expert[t]) * Cg + s / G) * words;
            for (int i = threadIdx.x; i < words; i += 256) o[i] = p[i];
        } else {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int i = threadIdx.x; i < words; i += 256) o[i] = z;
        }
    }
}

// out[t,:] = p_t * y[e_t, s_t, :] or 0.
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const u32x4 *y, const int32_t *expert, const int32_t *slot,
                                                       const float *gate_p, u32x4 *out, int64_t Tn, int64_t C,
                                                       int words) {
    constexpr int N = Vec<T>::N;
    for (int64_t t = blockIdx.x; t < Tn; t += gridDim.x) {
        const int s = slot[t];
        u32x4 *o = out + t * words;
        if (s >= 0) {
            const float p = gate_p[t];
            const u32x4 *src = y + ((int64_t)expert[t] * C + s) * words;
            for (int i = threadIdx.x; i < words; i += 256) {
                float v[N];
                Vec<T>::unpack(src[i], v);
#pragma unroll
                for (int j = 0; j < N; ++j) v[j] *= p;
                o[i] = Vec<T>::pack(v);
            }
        } else {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int i = threadIdx.x; i < words; i += 256) o[i] = z;
        }
    }
}

// d_y[r,:] = p * d_out[tok,:];  d_gate_p[tok] = <d_out[tok,:], y[r,:]>;  empty rows are left alone
// (the backward GEMMs read kept rows only); dropped tokens get d_gate_p = 0.
template <typename T>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const u32x4 *d_out, const u32x4 *y,
                                                           const int32_t *token_of_slot, const int32_t *slot,
                                                           const float *gate_p, u32x4 *d_y, float *d_gate_p,
                                                           int64_t rows, int64_t Tn, int words) {
    constexpr int N = Vec<T>::N;
    __shared__ float red[4];
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < Tn; t += (int64_t)gridDim.x * 256)
        if (slot[t] < 0) d_gate_p[t] = 0.f;
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const int tok = token_of_slot[r];
        if (tok < 0) continue;
        u32x4 *o = d_y + r * words;
        const float p = gate_p[tok];
        const u32x4 *g = d_out + (int64_t)tok * words;
        const u32x4 *yy = y + r * words;
        float dot = 0.f;
        for (int i = threadIdx.x; i < words; i += 256) {
            float gv[N], yv[N];
            Vec<T>::unpack(g[i], gv);
            Vec<T>::unpack(yy[i], yv);
#pragma unroll
            for (int j = 0; j < N; ++j) {
                dot = fmaf(gv[j], yv[j], dot);
                gv[j] *= p;
            }
            o[i] = Vec<T>::pack(gv);
        }
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = dot;
        __syncthreads();
        if (threadIdx.x == 0) d_gate_p[tok] = (red[0] + red[1]) + (red[2] + red[3]);
    }
}

// Preparation of the combine that is folded into the second GEMM's epilogue: the scale of every
// buffer row (gate probability of the token in that slot, 0 for an empty slot), and zero rows of `out`
// for dropped tokens, which no buffer row maps to.  Blocks [0, scale_blocks) do the first; each of the
// others looks at 16 tokens, 4 per wave, and a wave clears the rows of its dropped ones.
constexpr int PREP_TOKENS = 16;
__global__ __launch_bounds__(256) void combine_prep_kernel(const int32_t *token_of_slot, const int32_t *slot,
                                                            const float *gate_p, float *scale_of_slot, u32x4 *out,
                                                            int64_t rows, int64_t Tn, int words, int scale_blocks) {
    if ((int)blockIdx.x < scale_blocks) {
        const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (r < rows) {
            const int tok = token_of_slot[r];
            scale_of_slot[r] = tok >= 0 ? gate_p[tok] : 0.f;
        }
        return;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t0 = ((int64_t)blockIdx.x - scale_blocks) * PREP_TOKENS + wave * (PREP_TOKENS / 4);
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int i = 0; i < PREP_TOKENS / 4; ++i) {
        const int64_t t = t0 + i;
        if (t >= Tn || slot[t] >= 0) continue;
        u32x4 *o = out + t * words;
        for (int w = lane; w < words; w += 64) o[w] = z;
    }
}

// ------------------------------------------------------------------ host side
static unsigned row_grid(int64_t rows) { return (unsigned)(rows < 1048576 ? rows : 1048576); }

moe_status_t run_dispatch(const moe_shape_t *sh, const void *x, const int32_t *token_of_slot, void *buf,
                          hipStream_t s) {
    const int esz = sh->dtype == MOE_BF16 ? 2 : 4;
    const int words = sh->h * esz / 16;
    const int64_t rows = (int64_t)sh->E * sh->C;
    hipLaunchKernelGGL(dispatch_kernel, dim3(row_grid(rows)), dim3(256), 0, s, (const u32x4 *)x, token_of_slot,
                       (u32x4 *)buf, rows, words);
    return check_launch("dispatch");
}

// tp_size = 1: d_buf is [E, C, h]; tp_size = G > 1: d_buf holds the G shares [G, E, ceil(C/G), h]
moe_status_t run_dispatch_bwd(const moe_shape_t *sh, const void *d_buf, const int32_t *expert, const int32_t *slot,
                              void *d_x, hipStream_t s, int tp_size) {
    const int esz = sh->dtype == MOE_BF16 ? 2 : 4;
    const int words = sh->h * esz / 16;
    const int64_t Cg = (sh->C + tp_size - 1) / tp_size;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(row_grid(sh->T)), dim3(256), 0, s, (const u32x4 *)d_buf, expert, slot,
                       (u32x4 *)d_x, sh->T, Cg, tp_size, sh->E, words);
    return check_launch("dispatch_bwd");
}

moe_status_t run_dispatch_dtd(const moe_shape_t *sh, const void *x, const int32_t *token_of_slot, int tp_rank,
                              int tp_size, void *share, hipStream_t s) {
    const int words = sh->h * (sh->dtype == MOE_BF16 ? 2 : 4) / 16;
    const int64_t Cg = (sh->C + tp_size - 1) / tp_size, rows = (int64_t)sh->E * Cg;
    hipLaunchKernelGGL(dispatch_dtd_kernel, dim3(row_grid(rows)), dim3(256), 0, s, (const u32x4 *)x, token_of_slot,
                       (u32x4 *)share, rows, sh->C, Cg, tp_size, tp_rank, words);
    return check_launch("dispatch_dtd");
}

// width: elements per row (h for buf / d_buf)
moe_status_t run_dtd_drop(const moe_shape_t *sh, const void *buf, const int32_t *kept, int tp_rank, int tp_size,
                          void *share, hipStream_t s) {
    const int words = sh->h * (sh->dtype == MOE_BF16 ? 2 : 4) / 16;
    const int64_t Cg = (sh->C + tp_size - 1) / tp_size, rows = (int64_t)sh->E * Cg;
    hipLaunchKernelGGL(dtd_drop_kernel, dim3(row_grid(rows)), dim3(256), 0, s, (const u32x4 *)buf, kept, (u32x4 *)share,
                       rows, sh->C, Cg, tp_size, tp_rank, words);
    return check_launch("dtd_drop");
}

moe_status_t run_dtd_gather(const moe_shape_t *sh, const void *shares, const int32_t *kept, int tp_size, void *buf,
                            hipStream_t s) {
    const int words = sh->h * (sh->dtype == MOE_BF16 ? 2 : 4) / 16;
    const int64_t Cg = (sh->C + tp_size - 1) / tp_size, rows = (int64_t)sh->E * sh->C;
    hipLaunchKernelGGL(dtd_gather_kernel, dim3(row_grid(rows)), dim3(256), 0, s, (const u32x4 *)shares, kept,
                       (u32x4 *)buf, rows, sh->C, Cg, tp_size, sh->E, words);
    return check_launch("dtd_gather");
}

moe_status_t run_combine(const moe_shape_t *sh, const void *y, const int32_t *expert, const int32_t *slot,
                         const float *gate_p, void *out, hipStream_t s) {
    const int esz = sh->dtype == MOE_BF16 ? 2 : 4;
    const int words = sh->h * esz / 16;
    if (sh->dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(row_grid(sh->T)), dim3(256), 0, s, (const u32x4 *)y, expert,
                           slot, gate_p, (u32x4 *)out, sh->T, sh->C, words);
    else
        hipLaunchKernelGGL(combine_kernel<float>, dim3(row_grid(sh->T)), dim3(256), 0, s, (const u32x4 *)y, expert,
                           slot, gate_p, (u32x4 *)out, sh->T, sh->C, words);
    return check_launch("combine");
}

moe_status_t run_combine_prep(const moe_shape_t *sh, const int32_t *token_of_slot, const int32_t *slot,
                              const float *gate_p, float *scale_of_slot, void *out, hipStream_t s) {
    const int esz = sh->dtype == MOE_BF16 ? 2 : 4;
    const int words = sh->h * esz / 16;
    const int64_t rows = (int64_t)sh->E * sh->C;
    const int scale_blocks = (int)((rows + 255) / 256);
    const int64_t token_blocks = (sh->T + PREP_TOKENS - 1) / PREP_TOKENS;
    hipLaunchKernelGGL(combine_prep_kernel, dim3((unsigned)(scale_blocks + token_blocks)), dim3(256), 0, s, token_of_slot, slot,
                       gate_p, scale_of_slot, (u32x4 *)out, rows, sh->T, words, scale_blocks);
    return check_launch("combine_prep");
}

moe_status_t run_combine_bwd(const moe_shape_t *sh, const void *d_out, const void *y, const int32_t *token_of_slot,
                             const int32_t *slot, const float *gate_p, void *d_y, float *d_gate_p, hipStream_t s) {
    const int esz = sh->dtype == MOE_BF16 ? 2 : 4;
    const int words = sh->h * esz / 16;
    const int64_t rows = (int64_t)sh->E * sh->C;
    if (sh->dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_bwd_kernel<bf16_t>, dim3(row_grid(rows)), dim3(256), 0, s, (const u32x4 *)d_out,
                           (const u32x4 *)y, token_of_slot, slot, gate_p, (u32x4 *)d_y, d_gate_p, rows, sh->T, words);
    else
        hipLaunchKernelGGL(combine_bwd_kernel<float>, dim3(row_grid(rows)), dim3(256), 0, s, (const u32x4 *)d_out,
                           (const u32x4 *)y, token_of_slot, slot, gate_p, (u32x4 *)d_y, d_gate_p, rows, sh->T, words);
    return check_launch("combine_bwd");
}

}  // namespace moe
