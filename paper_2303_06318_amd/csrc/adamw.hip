// Tiled mixed-precision AdamW step for a flat parameter group (paper Section 4: the 16-bit
// gradients are up-cast to 32 bit for the update; cutting the group into tiles of ts parameters
// bounds the temporary to 4*ts bytes, reused by every tile.  AdamW: Section 6's set-up).
//
// Two ways to run a step:
//   staged: per tile, `upcast_kernel` writes the tile's fp32 gradients into the caller's staging
//           buffer and `adamw_kernel<.., true>` updates the tile from it -- the paper's procedure;
//   fused:  `adamw_kernel<.., false>` converts the 16-bit gradient in registers, so no temporary
//           exists at all and the whole group is one launch.
// Both produce the same bits: the staged value is exactly the fp32 number the fused path holds in a
// register.  The kernels are plain streaming kernels, bound by HBM: per parameter 14 bytes are read
// (2 gradient + 4 master + 4 + 4 moments) and 14 written (bf16 storage); the staged path adds a 4-byte
// write and a 4-byte read of the staging tile, which the memory counters show going to memory and back
// even for a tile of 7 MB (the L2 caches are per XCD, and the reader is in general on another XCD).
#include "moe_common.h"

namespace moe {

struct AdamwConst {
    float lr, beta1, beta2, omb1, omb2, eps, wd, inv_bc1, inv_bc2, grad_mult;
};

constexpr int OPT_THREADS = 256;
constexpr int OPT_VEC = 4;                         // parameters per thread and group: one 16-byte fp32 access per array,
                                                   // so every wave-wide load or store covers one contiguous KB
constexpr int OPT_UNROLL = 1;                      // groups per thread, OPT_THREADS * OPT_VEC parameters apart
                                                   // (2 and 4 stream no faster and make small tiles slower)
constexpr int64_t OPT_PER_BLOCK = (int64_t)OPT_THREADS * OPT_VEC * OPT_UNROLL;

// Plain loads and stores: non-temporal ones were measured 15-30 % slower for this stream.
template <typename V>
__device__ __forceinline__ V ld_stream(const V *p) { return *p; }
template <typename V>
__device__ __forceinline__ void st_stream(V *p, V v) { *p = v; }

// The update of one parameter.  Contraction is switched off and the fused multiply-adds are written
// out, so that every instantiation and both the vector and the ragged-end code round identically:
// a step gives the same bits whatever the tile size and wherever the up-cast happened.
__device__ __forceinline__ void adamw_one(const AdamwConst &c, float g, float &w, float &m, float &v) {
#pragma clang fp contract(off)
    m = __builtin_fmaf(c.beta1, m, c.omb1 * g);
    v = __builtin_fmaf(c.beta2, v, (c.omb2 * g) * g);
    const float mhat = m * c.inv_bc1;
    const float vhat = v * c.inv_bc2;
    const float u = __builtin_fmaf(c.wd, w, mhat / (sqrtf(vhat) + c.eps));
    w = __builtin_fmaf(-c.lr, u, w);
}

template <bool BF16>
__device__ __forceinline__ float load_grad(const void *grad, int64_t i) {
    if constexpr (BF16) return bf16_to_f32(((const bf16_t *)grad)[i]);
    else return ((const float *)grad)[i];
}
template <bool BF16>
__device__ __forceinline__ void store_param(void *param, int64_t i, float w) {
    if constexpr (BF16) ((bf16_t *)param)[i] = f32_to_bf16(w);
    else ((float *)param)[i] = w;
}

template <bool BF16>
__device__ __forceinline__ void load_grad4(const void *grad, int64_t i, float (&g)[OPT_VEC]) {
    if constexpr (BF16) {
        const bf16x4 gv = ld_stream((const bf16x4 *)((const bf16_t *)grad + i));
#pragma unroll
        for (int k = 0; k < OPT_VEC; ++k) g[k] = bf16_to_f32(gv[k]);
    } else {
        const f32x4 gv = ld_stream((const f32x4 *)((const float *)grad + i));
#pragma unroll
        for (int k = 0; k < OPT_VEC; ++k) g[k] = gv[k];
    }
}

// staging[j] = fp32(grad[j]) * grad_mult for j < len
template <bool BF16>
__global__ __launch_bounds__(OPT_THREADS) void upcast_kernel(int64_t len, const void *__restrict__ grad, float mult,
                                                             float *__restrict__ staging) {
    const int64_t base = (int64_t)blockIdx.x * OPT_PER_BLOCK + (int64_t)threadIdx.x * OPT_VEC;
    float g[OPT_UNROLL][OPT_VEC];
#pragma unroll
    for (int u = 0; u < OPT_UNROLL; ++u) {
        const int64_t i = base + (int64_t)u * OPT_THREADS * OPT_VEC;
        if (i + OPT_VEC <= len) load_grad4<BF16>(grad, i, g[u]);
    }
#pragma unroll
    for (int u = 0; u < OPT_UNROLL; ++u) {
        const int64_t i = base + (int64_t)u * OPT_THREADS * OPT_VEC;
        if (i + OPT_VEC <= len) {
            f32x4 o;
#pragma unroll
            for (int k = 0; k < OPT_VEC; ++k) o[k] = g[u][k] * mult;
            st_stream((f32x4 *)(staging + i), o);
        } else {
            for (int64_t j = i; j < len && j < i + OPT_VEC; ++j) staging[j] = load_grad<BF16>(grad, j) * mult;
        }
    }
}

// One AdamW update of len parameters.  STAGED: the gradient is read from `gsrc` as fp32 (already
// multiplied by grad_mult); otherwise `gsrc` holds the stored gradients (bf16 or fp32).
template <bool BF16, bool STAGED>
__global__ __launch_bounds__(OPT_THREADS) void adamw_kernel(int64_t len, AdamwConst c, const void *__restrict__ gsrc,
                                                            float *__restrict__ master, float *__restrict__ exp_avg,
                                                            float *__restrict__ exp_avg_sq, void *__restrict__ param) {
    const int64_t base = (int64_t)blockIdx.x * OPT_PER_BLOCK + (int64_t)threadIdx.x * OPT_VEC;
    float g[OPT_UNROLL][OPT_VEC];
    f32x4 wv[OPT_UNROLL], mv[OPT_UNROLL], vv[OPT_UNROLL];
    // all loads of the thread first, so that every group's requests are in flight together
#pragma unroll
    for (int u = 0; u < OPT_UNROLL; ++u) {
        const int64_t i = base + (int64_t)u * OPT_THREADS * OPT_VEC;
        if (i + OPT_VEC <= len) {
            load_grad4<(BF16 && !STAGED)>(gsrc, i, g[u]);
            wv[u] = ld_stream((const f32x4 *)(master + i));
            mv[u] = ld_stream((const f32x4 *)(exp_avg + i));
            vv[u] = ld_stream((const f32x4 *)(exp_avg_sq + i));
        }
    }
#pragma unroll
    for (int u = 0; u < OPT_UNROLL; ++u) {
        const int64_t i = base + (int64_t)u * OPT_THREADS * OPT_VEC;
        if (i + OPT_VEC <= len) {
            float w[OPT_VEC], m[OPT_VEC], v[OPT_VEC];
#pragma unroll
            for (int k = 0; k < OPT_VEC; ++k) {
                w[k] = wv[u][k]; m[k] = mv[u][k]; v[k] = vv[u][k];
                const float gk = STAGED ? g[u][k] : g[u][k] * c.grad_mult;
                adamw_one(c, gk, w[k], m[k], v[k]);
            }
            f32x4 wq, mq, vq;
#pragma unroll
            for (int k = 0; k < OPT_VEC; ++k) { wq[k] = w[k]; mq[k] = m[k]; vq[k] = v[k]; }
            st_stream((f32x4 *)(master + i), wq);
            st_stream((f32x4 *)(exp_avg + i), mq);
            st_stream((f32x4 *)(exp_avg_sq + i), vq);
            if constexpr (BF16) {
                bf16x4 pv;
#pragma unroll
                for (int k = 0; k < OPT_VEC; ++k) pv[k] = f32_to_bf16(w[k]);
                st_stream((bf16x4 *)((bf16_t *)param + i), pv);
            } else {
                st_stream((f32x4 *)((float *)param + i), wq);
            }
        } else {
            // ragged end of the tile: at most 3 parameters, one at a time
            for (int64_t j = i; j < len && j < i + OPT_VEC; ++j) {
                float gj = STAGED ? ((const float *)gsrc)[j] : load_grad<BF16>(gsrc, j) * c.grad_mult;
                float wj = master[j], mj = exp_avg[j], vj = exp_avg_sq[j];
                adamw_one(c, gj, wj, mj, vj);
                master[j] = wj; exp_avg[j] = mj; exp_avg_sq[j] = vj;
                store_param<BF16>(param, j, wj);
            }
        }
    }
}

static unsigned blocks_for(int64_t len) { return (unsigned)((len + OPT_PER_BLOCK - 1) / OPT_PER_BLOCK); }

// Arguments are validated by the caller: n >= 1, ts >= 1, and with a staging buffer either ts >= n
// or ts a multiple of 8 (tiles then start on 16-byte boundaries of every array).
moe_status_t run_adamw_tiled(int64_t n, int64_t ts, const AdamwConst &c, const void *grad, float *master,
                             float *exp_avg, float *exp_avg_sq, void *param, float *staging, int dtype,
                             hipStream_t s) {
    const bool bf = dtype == MOE_BF16;
    const size_t gsz = bf ? 2 : 4;
    if (staging == nullptr) {
        if (bf) adamw_kernel<true, false><<<blocks_for(n), OPT_THREADS, 0, s>>>(n, c, grad, master, exp_avg, exp_avg_sq, param);
        else adamw_kernel<false, false><<<blocks_for(n), OPT_THREADS, 0, s>>>(n, c, grad, master, exp_avg, exp_avg_sq, param);
        return check_launch("adamw_kernel");
    }
    for (int64_t i0 = 0; i0 < n; i0 += ts) {
        const int64_t len = n - i0 < ts ? n - i0 : ts;
        const void *g = (const char *)grad + (size_t)i0 * gsz;
        void *p = (char *)param + (size_t)i0 * gsz;
        if (bf) {
            upcast_kernel<true><<<blocks_for(len), OPT_THREADS, 0, s>>>(len, g, c.grad_mult, staging);
            adamw_kernel<true, true><<<blocks_for(len), OPT_THREADS, 0, s>>>(len, c, staging, master + i0, exp_avg + i0,
                                                                            exp_avg_sq + i0, p);
        } else {
            upcast_kernel<false><<<blocks_for(len), OPT_THREADS, 0, s>>>(len, g, c.grad_mult, staging);
            adamw_kernel<false, true><<<blocks_for(len), OPT_THREADS, 0, s>>>(len, c, staging, master + i0, exp_avg + i0,
                                                                             exp_avg_sq + i0, p);
        }
    }
    return check_launch("adamw_kernel (tiled)");
}

}  // namespace moe
