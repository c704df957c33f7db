// HBM-streaming row movers: dispatch, combine and their backward, and the gate backward.
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

// buf[r,:] = x[token_of_slot[r],:] or 0.  Pure copy: works on 16-byte words of any type.
__global__ __launch_bounds__(256) void dispatch_kernel(const u32x4 *x, const int32_t *token_of_slot, u32x4 *buf,
                                                        int64_t rows, int words) {
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const int tok = token_of_slot[r];
        u32x4 *dst = buf + r * words;
        if (tok >= 0) {
            const u32x4 *src = x + (int64_t)tok * words;
            for (int i = threadIdx.x; i < words; i += 256) dst[i] = src[i];
        } else {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int i = threadIdx.x; i < words; i += 256) dst[i] = z;
        }
    }
}

// dst[t,:] = src[expert[t], slot[t], :] or 0 (dispatch backward).
__global__ __launch_bounds__(256) void gather_rows_kernel(const u32x4 *src, const int32_t *expert, const int32_t *slot,
                                                           u32x4 *dst, int64_t T, int64_t C, int words) {
    for (int64_t t = blockIdx.x; t < T; t += gridDim.x) {
        const int s = slot[t];
        u32x4 *o = dst + t * words;
        if (s >= 0) {
            const u32x4 *p = src + ((int64_t)expert[t] * C + s) * words;
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

// d_y[r,:] = p * d_out[tok,:];  d_gate_p[tok] = <d_out[tok,:], y[r,:]>;  empty rows -> 0;
// dropped tokens get d_gate_p = 0.
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
        u32x4 *o = d_y + r * words;
        if (tok < 0) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int i = threadIdx.x; i < words; i += 256) o[i] = z;
            continue;
        }
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

// ------------------------------------------------------------------ gate backward
// d_logits[t,j] = d_gate_p[t] * p_t * ([j == e_t] - probs[t,j])
__global__ void gate_dlogits_kernel(const float *d_gate_p, const float *probs, const int32_t *expert, float *d_logits,
                                    int64_t T, int E) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * E) return;
    int64_t t = i / E;
    int j = (int)(i - t * E);
    int e = expert[t];
    float pe = probs[t * E + e];
    d_logits[i] = d_gate_p[t] * pe * ((j == e ? 1.f : 0.f) - probs[i]);
}

// Block = 64 columns of x (k0..k0+63) x 4 token lanes, token chunk [t0, t1).
//   partial[chunk][k][j] = sum_{t in chunk} x[t,k] * d_logits[t,j]
//   d_x[t,k] += sum_j d_logits[t,j] * w_gate[k,j]
template <typename T, int EJ>
__global__ __launch_bounds__(256) void gate_bwd_main_kernel(const T *x, const float *w_gate, const float *d_logits,
                                                             float *partial, T *d_x, int64_t Tn, int h, int E,
                                                             int64_t chunk_len) {
    __shared__ float red[4][64][EJ + 1];
    const int c = threadIdx.x & 63, tq = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + c;
    const bool kin = k < h;
    const int64_t t0 = (int64_t)blockIdx.y * chunk_len;
    const int64_t t1 = t0 + chunk_len < Tn ? t0 + chunk_len : Tn;
    for (int j0 = 0; j0 < E; j0 += EJ) {
        float wg[EJ], acc[EJ];
#pragma unroll
        for (int j = 0; j < EJ; ++j) {
            wg[j] = (kin && j0 + j < E) ? w_gate[(int64_t)k * E + j0 + j] : 0.f;
            acc[j] = 0.f;
        }
        for (int64_t t = t0 + tq; t < t1; t += 4) {
            const float *dl = d_logits + t * E + j0;
            const float xv = kin ? (float)x[t * h + k] : 0.f;
            float dxa = 0.f;
#pragma unroll
            for (int j = 0; j < EJ; ++j) {
                const float g = (j0 + j < E) ? dl[j] : 0.f;
                acc[j] = fmaf(xv, g, acc[j]);
                dxa = fmaf(g, wg[j], dxa);
            }
            if (d_x && kin) d_x[t * h + k] = (T)((float)d_x[t * h + k] + dxa);
        }
#pragma unroll
        for (int j = 0; j < EJ; ++j) red[tq][c][j] = acc[j];
        __syncthreads();
        if (partial) {
            for (int i = threadIdx.x; i < 64 * EJ; i += 256) {
                int cc = i / EJ, j = i - cc * EJ;
                int kk = blockIdx.x * 64 + cc;
                if (kk < h && j0 + j < E)
                    partial[((int64_t)blockIdx.y * h + kk) * E + j0 + j] =
                        (red[0][cc][j] + red[1][cc][j]) + (red[2][cc][j] + red[3][cc][j]);
            }
        }
        __syncthreads();
    }
}

__global__ void gate_dwg_reduce_kernel(const float *partial, float *d_w_gate, int64_t n, int nchunks) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int c = 0; c < nchunks; ++c) s += partial[(int64_t)c * n + i];
    d_w_gate[i] = s;
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

moe_status_t run_dispatch_bwd(const moe_shape_t *sh, const void *d_buf, const int32_t *expert, const int32_t *slot,
                              void *d_x, hipStream_t s) {
    const int esz = sh->dtype == MOE_BF16 ? 2 : 4;
    const int words = sh->h * esz / 16;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(row_grid(sh->T)), dim3(256), 0, s, (const u32x4 *)d_buf, expert, slot,
                       (u32x4 *)d_x, sh->T, sh->C, words);
    return check_launch("dispatch_bwd");
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

int gate_bwd_chunks(const moe_shape_t *sh) {
    int64_t n = (sh->T + 1023) / 1024;
    return (int)(n < 1 ? 1 : (n > 32 ? 32 : n));
}

size_t gate_bwd_ws_bytes(const moe_shape_t *sh) {
    return (size_t)gate_bwd_chunks(sh) * sh->h * sh->E * 4;
}

template <typename T>
static void launch_gate_bwd_main(const moe_shape_t *sh, const void *x, const float *w_gate, const float *d_logits,
                                 float *partial, void *d_x, int nch, int64_t chunk_len, hipStream_t s) {
    dim3 grid((sh->h + 63) / 64, nch), block(256);
    if (sh->E <= 16)
        hipLaunchKernelGGL((gate_bwd_main_kernel<T, 16>), grid, block, 0, s, (const T *)x, w_gate, d_logits, partial,
                           (T *)d_x, sh->T, sh->h, sh->E, chunk_len);
    else if (sh->E <= 32)
        hipLaunchKernelGGL((gate_bwd_main_kernel<T, 32>), grid, block, 0, s, (const T *)x, w_gate, d_logits, partial,
                           (T *)d_x, sh->T, sh->h, sh->E, chunk_len);
    else
        hipLaunchKernelGGL((gate_bwd_main_kernel<T, 64>), grid, block, 0, s, (const T *)x, w_gate, d_logits, partial,
                           (T *)d_x, sh->T, sh->h, sh->E, chunk_len);
}

moe_status_t run_gate_bwd(const moe_shape_t *sh, const float *d_gate_p, const float *probs, const int32_t *expert,
                          const void *x, const float *w_gate, float *d_logits, float *d_w_gate, void *d_x_accum,
                          void *ws, hipStream_t s) {
    const int64_t n = sh->T * sh->E;
    hipLaunchKernelGGL(gate_dlogits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_gate_p, probs,
                       expert, d_logits, sh->T, sh->E);
    if (d_w_gate || d_x_accum) {
        const int nch = gate_bwd_chunks(sh);
        const int64_t chunk_len = (sh->T + nch - 1) / nch;
        float *partial = d_w_gate ? (float *)ws : nullptr;
        if (sh->dtype == MOE_BF16)
            launch_gate_bwd_main<bf16_t>(sh, x, w_gate, d_logits, partial, d_x_accum, nch, chunk_len, s);
        else
            launch_gate_bwd_main<float>(sh, x, w_gate, d_logits, partial, d_x_accum, nch, chunk_len, s);
        if (d_w_gate) {
            const int64_t m = (int64_t)sh->h * sh->E;
            hipLaunchKernelGGL(gate_dwg_reduce_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, s, partial,
                               d_w_gate, m, nch);
        }
    }
    return check_launch("gate_bwd");
}

}  // namespace moe
