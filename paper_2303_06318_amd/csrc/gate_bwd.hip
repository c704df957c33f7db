// Gate backward: d_logits from the softmax Jacobian, d_w_gate = X^T d_logits, d_x += d_logits w_gate^T.
#include <cstdlib>
#include "moe_common.h"

namespace moe {

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


// ================================================================== bf16 tokens: matrix-core path
// d_w_gate = X^T dL is a contraction over tokens.  It runs on 16x16x32 bf16 MFMAs as
// out^T[E, cols] = dL^T[E, tokens] X[tokens, cols]: dL keeps fp32 accuracy by being split into three
// bf16 planes (hi + mid + lo), stored transposed [3][Epad][Tpad] so a lane's 8 consecutive tokens
// are one 16-byte load; X tiles [32 tokens][256 cols] pass through LDS and are read with the LDS
// transpose load.  Each workgroup owns 256 columns x one token chunk and writes a partial
// [Epad][h] fp32 tile; a second kernel sums the chunks in a fixed order (deterministic).

// d_logits and its three transposed bf16 planes.  One thread per (j, t); t is the fast index.
__global__ void gate_dlogits_planes_kernel(const float *d_gate_p, const float *probs, const int32_t *expert,
                                           float *d_logits, bf16_t *planes, int64_t T, int E, int Epad, int64_t Tpad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)Epad * Tpad) return;
    const int j = (int)(i / Tpad);
    const int64_t t = i - (int64_t)j * Tpad;
    float g = 0.f;
    if (j < E && t < T) {
        const int e = expert[t];
        const float pe = probs[t * E + e];
        g = d_gate_p[t] * pe * ((j == e ? 1.f : 0.f) - probs[t * E + j]);
        d_logits[t * E + j] = g;
    }
    const bf16_t hi = f32_to_bf16(g);
    const float r1 = g - bf16_to_f32(hi);
    const bf16_t mid = f32_to_bf16(r1);
    const bf16_t lo = f32_to_bf16(r1 - bf16_to_f32(mid));
    const int64_t n = (int64_t)Epad * Tpad;
    planes[i] = hi;
    planes[n + i] = mid;
    planes[2 * n + i] = lo;
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4_g;

// partial[chunk][e][col] = sum over the chunk's tokens of dL[t,e] * x[t,col]
// The kernel streams x once and is bound by the bytes each compute unit keeps in flight: a workgroup has
// the x tiles of the next two iterations (2 x 16 KB) and the d_logits fragments of the next iteration
// requested while it multiplies.  Within an iteration the small requests (d_logits planes) are issued
// before the x tile: the memory counter retires in issue order, so waiting for the planes of the next
// iteration leaves the newer x tiles in flight.
template <int NT>
__global__ __launch_bounds__(256) void gate_dwg_mfma_kernel(const bf16_t *x, const bf16_t *planes, float *partial,
                                                             int64_t T, int h, int64_t Tpad, int64_t chunk_len,
                                                             int Epad) {
    __shared__ __attribute__((aligned(16))) char xs[3][32 * 512];    // [32 tokens][256 cols] bf16, swizzled
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c0 = blockIdx.x * 256;
    const int64_t t_begin = (int64_t)blockIdx.y * chunk_len;
    const int64_t t_end = t_begin + chunk_len < Tpad ? t_begin + chunk_len : Tpad;
    const int64_t plane = (int64_t)Epad * Tpad;      // distance between the hi / mid / lo planes

    // loader: thread -> token rows tid/32 + 8q (q = 0..3), granule tid%32 (8 columns); rows past T and
    // columns past h read as zero through the buffer resource (offset marker beyond its size)
    const int lg = tid & 31, lrow = tid >> 5;
    const bool col_ok = c0 + lg * 8 < h;
    constexpr uint32_t OUTSIDE = 0x80000000u;
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(x + t_begin * h), 0, (int)((T - t_begin < chunk_len ? T - t_begin : chunk_len) * h * 2), 0x00020000);
    auto gload = [&](int64_t t0, u32x4(&stg)[4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t tr = t0 - t_begin + lrow + 8 * q;         // row inside the chunk
            const uint32_t off = (col_ok & (t0 + lrow + 8 * q < T)) ? ((uint32_t)tr * (uint32_t)h + c0 + lg * 8) * 2u : OUTSIDE;
            stg[q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(xr, off, 0, 0));
        }
    };
    auto sstore = [&](int buf, const u32x4(&stg)[4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = lrow + 8 * q;
            *(u32x4 *)(xs[buf] + k * 512 + ((lg ^ ((k & 3) << 2)) << 4)) = stg[q];
        }
    };
    // B fragment (16 columns x 32 tokens) of column block nb for this wave: lane j%16 of token group
    // G = lane/16 reads 8 bytes at token-row 8G + j/4 (+4), columns 4*(j%4)
    const int kr = 8 * (lane >> 4) + ((lane & 15) >> 2), sw = (lane >> 2) & 3;
    int boff[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
        const int gran = (wave * 64 + nb * 16) / 8 + ((lane & 3) >> 1);
        boff[nb] = kr * 512 + ((gran ^ (sw << 2)) << 4) + (lane & 1) * 8;
    }
    f32x4 acc[NT][4];
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[et][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    // A fragments (d_logits planes, transposed: a lane's 8 consecutive tokens are 16 bytes), one iteration ahead
    auto aload = [&](int64_t t0, u32x4(&av)[NT][3]) {
        const int64_t ts = t0 < t_end ? t0 : t_begin;               // past the end: any valid tile (never used)
#pragma unroll
        for (int et = 0; et < NT; ++et)
#pragma unroll
            for (int p3 = 0; p3 < 3; ++p3)
                av[et][p3] = *(const u32x4 *)(planes + p3 * plane + (int64_t)(et * 16 + (lane & 15)) * Tpad + ts +
                                              8 * (lane >> 4));
    };
    auto compute = [&](int buf, const u32x4(&av)[NT][3]) {
        bf16x8 bfr[4];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            const char *p = xs[buf] + boff[nb];
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_g *)p);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_g *)(p + 4 * 512));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            bfr[nb] = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
#pragma unroll
        for (int et = 0; et < NT; ++et)
#pragma unroll
            for (int p3 = 0; p3 < 3; ++p3) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, av[et][p3]);
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
                    acc[et][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bfr[nb], acc[et][nb], 0, 0, 0);
            }
    };
    // One iteration: tile i sits in xs[i % 3]; s_cur holds tile i + 1 (requested two iterations ago) and is
    // stored to xs[(i + 1) % 3] after this tile's arithmetic; then tile i + 3 is requested into s_cur.  Two
    // register sets alternate (the loop body is two iterations, so no set is ever copied).
    auto iteration = [&](int64_t t0, int buf, const u32x4(&a_cur)[NT][3], u32x4(&a_nxt)[NT][3], u32x4(&s_cur)[4]) {
        aload(t0 + 32, a_nxt);
        __builtin_amdgcn_sched_barrier(0);
        compute(buf, a_cur);
        sstore(buf == 2 ? 0 : buf + 1, s_cur);
        __builtin_amdgcn_sched_barrier(0);
        gload(t0 + 96, s_cur);                                      // past the chunk: zeros, never used
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };
    u32x4 sA[4], sB[4], aA[NT][3], aB[NT][3];
    if (t_begin < t_end) {
        gload(t_begin, sA);
        sstore(0, sA);
        aload(t_begin, aA);
        gload(t_begin + 32, sA);
        gload(t_begin + 64, sB);
    }
    __syncthreads();
    int buf = 0;
    for (int64_t t0 = t_begin; t0 < t_end; t0 += 64) {
        iteration(t0, buf, aA, aB, sA);
        buf = buf == 2 ? 0 : buf + 1;
        if (t0 + 32 < t_end) iteration(t0 + 32, buf, aB, aA, sB);
        buf = buf == 2 ? 0 : buf + 1;
    }
    // result block: lane holds column lane%16, rows (experts) 4*(lane/16) + v
#pragma unroll
    for (int et = 0; et < NT; ++et)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            const int col = c0 + wave * 64 + nb * 16 + (lane & 15);
            if (col < h) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = et * 16 + 4 * (lane >> 4) + v;
                    partial[((int64_t)blockIdx.y * Epad + e) * h + col] = acc[et][nb][v];
                }
            }
        }
}

// d_w_gate[k][j] = sum_chunks partial[chunk][j][k]
__global__ void gate_dwg_reduce_t_kernel(const float *partial, float *d_w_gate, int h, int E, int Epad, int nchunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)E * h) return;
    const int j = (int)(i / h), k = (int)(i - (int64_t)j * h);
    float s = 0.f;
    int c = 0;
    for (; c + 8 <= nchunks; c += 8) {            // 8 loads in flight, summed in chunk order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[((int64_t)(c + u) * Epad + j) * h + k];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < nchunks; ++c) s += partial[((int64_t)c * Epad + j) * h + k];
    d_w_gate[(int64_t)k * E + j] = s;
}

// d_x[t, k] (+)= sum_j dL[t,j] * w_gate[k,j].  A thread keeps CW columns x EJ experts of w_gate in
// registers and walks the tokens of its chunk; dL rows are broadcast from LDS.
// With d_buf == nullptr the sum is added to d_x in place.  With d_buf given, the dispatch backward
// is fused in: d_x[t,:] = d_buf[expert[t], slot[t], :] (0 for a dropped token) + the sum, so d_x is
// written once instead of written, read and written again.
template <int CW, int EJ>
__global__ __launch_bounds__(256) void gate_dx_kernel(const float *w_gate, const float *d_logits, bf16_t *d_x, int64_t T,
                                                       int h, int E, int j0, int64_t chunk_len, const bf16_t *d_buf,
                                                       const int32_t *expert, const int32_t *slot, int64_t Cg, int G) {
    constexpr int TT = 64;
    __shared__ float dl[TT][EJ];
    __shared__ int32_t srow[TT];      // fused gather: buffer row of each token, -1 if dropped
    const int tid = threadIdx.x;
    const int k0 = (blockIdx.x * 256 + tid) * CW;
    const bool kin = k0 < h;
    float wg[CW][EJ];
#pragma unroll
    for (int c = 0; c < CW; ++c)
#pragma unroll
        for (int j = 0; j < EJ; ++j) wg[c][j] = (kin && j0 + j < E) ? w_gate[(int64_t)(k0 + c) * E + j0 + j] : 0.f;
    const int64_t t_begin = (int64_t)blockIdx.y * chunk_len;
    const int64_t t_end = t_begin + chunk_len < T ? t_begin + chunk_len : T;
    for (int64_t tb = t_begin; tb < t_end; tb += TT) {
        __syncthreads();
        for (int i = tid; i < TT * EJ; i += 256) {
            const int tt = i / EJ, j = i - tt * EJ;
            dl[tt][j] = (tb + tt < t_end && j0 + j < E) ? d_logits[(tb + tt) * E + j0 + j] : 0.f;
        }
        if (d_buf && tid < TT && tb + tid < t_end) {
            const int sl = slot[tb + tid];
            srow[tid] = sl < 0 ? -1 : (int32_t)(((int64_t)(sl % G) * E + expert[tb + tid]) * Cg + sl / G);
        }
        __syncthreads();
        const int nt = (int)(t_end - tb < TT ? t_end - tb : TT);
        if (!kin) continue;
        // groups of 4 tokens: the row loads of the next group are issued before the arithmetic of
        // this one (the kernel runs 2 waves per SIMD, so the loads in flight per wave decide the
        // bandwidth), then the 4 stores
        auto load_row = [&](int tt, float(&v)[CW]) {
            bool zero = tt >= nt;
            const bf16_t *src = d_x + (tb + (zero ? 0 : tt)) * h + k0;
            if (d_buf && !zero) {
                const int r = srow[tt];
                zero = r < 0;
                src = d_buf + (int64_t)(zero ? 0 : r) * h + k0;
            }
            if (zero) {
#pragma unroll
                for (int c = 0; c < CW; ++c) v[c] = 0.f;
            } else {
#pragma unroll
                for (int c = 0; c < CW; ++c) v[c] = (float)src[c];
            }
        };
        auto load_row8 = [&](int tt) {           // CW == 8: the raw 16 bytes, zero for a dropped token
            bool zero = tt >= nt;
            const bf16_t *src = d_x + (tb + (zero ? 0 : tt)) * h + k0;
            if (d_buf && !zero) {
                const int r = srow[tt];
                zero = r < 0;
                src = d_buf + (int64_t)(zero ? 0 : r) * h + k0;
            }
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (!zero) raw = *(const u32x4 *)src;
            return raw;
        };
        u32x4 nxt[4];
        if (CW == 8) {
#pragma unroll
            for (int u = 0; u < 4; ++u) nxt[u] = load_row8(u);
        }
        for (int t4 = 0; t4 < nt; t4 += 4) {
            float v[4][CW];
            if (CW == 8) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bf16x8 b = __builtin_bit_cast(bf16x8, nxt[u]);
#pragma unroll
                    for (int c = 0; c < 8; ++c) v[u][c < CW ? c : 0] = (float)b[c];
                }
                if (t4 + 4 < nt) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) nxt[u] = load_row8(t4 + 4 + u);
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) load_row(t4 + u, v[u]);
            }
#pragma unroll
            for (int j = 0; j < EJ; ++j) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float g = dl[(t4 + u) & (TT - 1)][j];
#pragma unroll
                    for (int c = 0; c < CW; ++c) v[u][c] = fmaf(g, wg[c][j], v[u][c]);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int tt = t4 + u;
                if (tt >= nt) continue;
                bf16_t *row = d_x + (tb + tt) * h + k0;
                if (CW == 8) {
                    bf16x8 b;
#pragma unroll
                    for (int c = 0; c < 8; ++c) b[c] = (bf16_t)v[u][c < CW ? c : 0];
                    *(bf16x8 *)row = b;
                } else {
#pragma unroll
                    for (int c = 0; c < CW; ++c) row[c] = (bf16_t)v[u][c];
                }
            }
        }
    }
}

// The same sum for E <= 64 without a transposition through LDS: every wave owns 128 columns and walks
// its tokens 16 at a time with v_mfma_f32_16x16x32_bf16, result block [16 tokens x 16 column slots].
// The column a slot stands for is free to choose (it only decides which row of Wg feeds the B operand),
// so block b (0..7) takes slot n <-> column 8 n + b: after the 8 blocks lane l holds, for each of its 4
// token rows, the 8 CONSECUTIVE columns 8 (l % 16) .. + 7.  The gathered d_buf row piece (16 bytes) is
// loaded, the sum is added and the result stored with one 16-byte access per lane, 16 lanes covering 256
// contiguous bytes of a row; the Wg^T fragments (hi + lo bf16 pieces, 64 registers per 32 experts) stay
// in registers for the wave's whole token range.  Both factors are split in two bf16 pieces and the three
// leading products summed in fp32.  LDS only holds the workgroup's small operands (source row of each
// token, d_logits rows), written once before the loop, so that the loop's only vector-memory traffic is
// the row stream.
constexpr int DX_TOKENS = 192;          // tokens per workgroup (4 waves x 128 columns each); a multiple of 48
template <int KS, bool GATHER>          // 32-expert k-steps (E <= 32 KS); rows gathered from d_buf, or d_x in place
__global__ __launch_bounds__(256, KS == 1 ? 2 : 1) void gate_dx_rows_kernel(
    const float *w_gate, const float *d_logits, bf16_t *d_x, int64_t T, int h, int E, const bf16_t *d_buf,
    const int32_t *expert, const int32_t *slot, int64_t Cg, int G) {
    // d_buf is [E, C, h], or (duplicate token dropping, G > 1) the G shares [G, E, Cg, h]: row s of expert e
    // is row s / G of share s % G; G = 1, Cg = C is the plain layout
    // One dynamic LDS region of 512 rows x (E8 + 4) floats (E8 = E rounded up to 8), used twice: first the
    // workgroup's 512 rows of Wg, read from memory with coalesced accesses and then picked apart into MFMA
    // fragments; afterwards the d_logits rows of its tokens.  Behind it, the source row of every token.
    extern __shared__ __attribute__((aligned(16))) float s_f[];
    const int E8 = (E + 7) & ~7, LDE = E8 + 4;
    int32_t *s_row = (int32_t *)(s_f + 512 * LDE);                // DX_TOKENS + 48 entries (-1: no row): requests run ahead
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int64_t t_begin = (int64_t)blockIdx.y * DX_TOKENS;
    const int nt = (int)(T - t_begin < DX_TOKENS ? T - t_begin : DX_TOKENS);     // tokens of this workgroup
    const int c_first = blockIdx.x * 512;
    const int ncol = h - c_first < 512 ? h - c_first : 512;       // columns of this workgroup inside the matrix
    // Loads are unconditional, from clamped (always valid) addresses, and a select zeroes what lies
    // outside ("&", not "&&": a guarded load becomes a branch around the load plus a full wait).
    if ((E & 3) == 0) {                                           // 16-byte pieces: rows of Wg are contiguous in memory
        const int q4 = E >> 2, e4 = E8 >> 2;
        for (int i = tid; i < 512 * e4; i += 256) {
            const int c = i / e4, k4 = i - c * e4;
            const bool in = (c < ncol) & (k4 < q4);
            const f32x4 v = *(const f32x4 *)(w_gate + (int64_t)(c_first + (c < ncol ? c : 0)) * E + 4 * (k4 < q4 ? k4 : 0));
            *(f32x4 *)&s_f[c * LDE + 4 * k4] = in ? v : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    } else {
        for (int i = tid; i < 512 * E8; i += 256) {
            const int c = i / E8, k = i - c * E8;
            const bool in = (c < ncol) & (k < E);
            const float v = w_gate[(int64_t)(c_first + (c < ncol ? c : 0)) * E + (k < E ? k : 0)];
            s_f[c * LDE + k] = in ? v : 0.f;
        }
    }
    for (int i = tid; i < DX_TOKENS + 48; i += 256) {
        const bool tin = i < nt;
        const int64_t t = t_begin + (tin ? i : 0);
        int32_t r = (int32_t)t;
        if (GATHER) {
            const int sl = slot[t], ex = expert[t];
            r = sl >= 0 ? ((sl % G) * E + ex) * (int32_t)Cg + sl / G : -1;
        }
        s_row[i] = tin ? r : -1;
    }
    __syncthreads();
    const int cw = c_first + wave * 128;                          // first column of the wave
    const int col = cw + 8 * n16;                                 // the lane's 8 columns
    const bool cin = col < h;
    // The lane's 8 experts of k-step ks start at 32 ks + 8 g; at or beyond E8 they do not exist (zeros).
    // B fragments: block b, slot n = lane % 16 <-> column col + b.
    bf16x8 bh[8][KS], bl[8][KS];
#pragma unroll
    for (int b = 0; b < 8; ++b) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int k0 = ks * 32 + 8 * g;
            const bool kin = k0 < E8;
            const float *p = &s_f[(wave * 128 + 8 * n16 + b) * LDE + (kin ? k0 : 0)];
            const f32x4 w0 = *(const f32x4 *)p, w1 = *(const f32x4 *)(p + 4);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float v = kin ? (q < 4 ? w0[q & 3] : w1[q & 3]) : 0.f;
                const bf16_t hq = f32_to_bf16(v);
                bh[b][ks][q] = hq;
                bl[b][ks][q] = f32_to_bf16(v - bf16_to_f32(hq));
            }
        }
    }
    __syncthreads();                                              // the Wg rows have been read: the region is reused
    for (int i = tid; i < (DX_TOKENS + 16) * E8; i += 256) {
        const int tt = i / E8, k = i - tt * E8;
        const bool in = (tt < nt) & (k < E);
        const float v = d_logits[(t_begin + (tt < nt ? tt : 0)) * E + (k < E ? k : 0)];
        s_f[tt * LDE + k] = in ? v : 0.f;
    }
    __syncthreads();
    if (cw >= h) return;                                          // whole wave outside the matrix (no barrier below)
    // Rows move through buffer resources: an offset beyond the resource's size (the marker below, for a
    // dropped token, a token past the end, a column past h) makes a load return zeros and a store do nothing,
    // so the stream has no branches and the compiler's wait counts are exact.
    constexpr uint32_t OUTSIDE = 0x80000000u;                      // the host checks that both arrays are shorter
    const int64_t src_rows = GATHER ? (int64_t)G * E * Cg : T;
    const __amdgpu_buffer_rsrc_t src_r = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(GATHER ? d_buf : d_x), 0, (int)(src_rows * h * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t dst_r = __builtin_amdgcn_make_buffer_rsrc(d_x, 0, (int)(T * h * 2), 0x00020000);
    // the lane's 4 token rows of group tg (tokens tg .. tg + 15 of the workgroup) are tg + 4 g + v
    auto load_rows = [&](int tg, u32x4(&dst)[4]) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int32_t r = s_row[tg + 4 * g + v];
            const uint32_t off = (cin & (r >= 0)) ? ((uint32_t)r * (uint32_t)h + (uint32_t)col) * 2u : OUTSIDE;
            dst[v] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(src_r, off, 0, 0));
        }
    };
    // The kernel is bound by memory latency, i.e. by the bytes each compute unit keeps in flight: row
    // requests run two groups ahead of the arithmetic, in three register sets that rotate (the loop is
    // unrolled, so no set is ever copied: a copy would wait for its load).
    auto step = [&](int tg, const u32x4(&rows_cur)[4], u32x4(&rows_dst)[4]) {
        load_rows(tg + 32, rows_dst);           // past the workgroup's tokens s_row holds -1: zero rows, never stored
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 ah[KS], al[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            // A operand: token tg + lane % 16, experts 32 ks + 8 g .. + 7
            const int k0 = ks * 32 + 8 * g;
            const bool kin = k0 < E8;
            const float *p = &s_f[(tg + n16) * LDE + (kin ? k0 : 0)];
            const f32x4 a0 = *(const f32x4 *)p, a1 = *(const f32x4 *)(p + 4);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float a = kin ? (q < 4 ? a0[q & 3] : a1[q & 3]) : 0.f;
                const bf16_t hq = f32_to_bf16(a);
                ah[ks][q] = hq;
                al[ks][q] = f32_to_bf16(a - bf16_to_f32(hq));
            }
        }
        f32x4 acc[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[ks], bh[b][ks], acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[ks], bl[b][ks], acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[ks], bh[b][ks], acc[b], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // result: lane holds token rows 4 g + v, column slot n16 of block b = column col + b
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tt = tg + 4 * g + v;
            const bf16x8 r = __builtin_bit_cast(bf16x8, rows_cur[v]);
            bf16x8 o;
#pragma unroll
            for (int b = 0; b < 8; ++b) o[b] = f32_to_bf16(bf16_to_f32(r[b]) + acc[b][v]);
            const uint32_t off = (cin & (tt < nt)) ? ((uint32_t)(t_begin + tt) * (uint32_t)h + (uint32_t)col) * 2u : OUTSIDE;
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((ext_vector_type(4))) unsigned int, o), dst_r, off, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    u32x4 r0[4], r1[4], r2[4];
    load_rows(0, r0);
    load_rows(16, r1);
    // step k: rows in r[k % 3], the new requests go to r[(k + 2) % 3].  Every trip runs all three steps, also
    // past the last token (zero rows, nothing stored): no branch, so the waits inside count exact loads.
    static_assert(DX_TOKENS % 48 == 0, "three 16-token steps per trip");
    // Fully unrolled: a loop back-edge makes the register allocator copy the rotating sets, and a copy of a
    // register that a load is still writing is a full wait.
#pragma unroll
    for (int tg = 0; tg < DX_TOKENS; tg += 48) {
        step(tg, r0, r2);
        step(tg + 16, r1, r0);
        step(tg + 32, r2, r1);
    }
}

// ------------------------------------------------------------------ host side
static int simple_chunks(const moe_shape_t *sh) {
    int64_t n = (sh->T + 1023) / 1024;
    return (int)(n < 1 ? 1 : (n > 32 ? 32 : n));
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

static moe_status_t run_gate_bwd_simple(const moe_shape_t *sh, const float *d_gate_p, const float *probs, const int32_t *expert,
                          const void *x, const float *w_gate, float *d_logits, float *d_w_gate, void *d_x_accum,
                          void *ws, hipStream_t s) {
    const int64_t n = sh->T * sh->E;
    hipLaunchKernelGGL(gate_dlogits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_gate_p, probs,
                       expert, d_logits, sh->T, sh->E);
    if (d_w_gate || d_x_accum) {
        const int nch = simple_chunks(sh);
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


// ---- workspace layout of the bf16 path: [planes 3*Epad*Tpad bf16][partial nchunks*Epad*h fp32]
static int epad_of(int E) { return (E + 15) / 16 * 16; }
static int64_t tpad_of(int64_t T) { return (T + 31) / 32 * 32; }
// Token chunks of the d_w_gate kernel: enough workgroups (256-column blocks x chunks) for three per compute
// unit of the 256-CU chip, chunks of at least 128 tokens, at most 64 partial results to sum.
static int dwg_chunks(const moe_shape_t *sh) {
    const int64_t col_blocks = (sh->h + 255) / 256;
    int64_t n = (768 + col_blocks - 1) / col_blocks;
    const int64_t most = (tpad_of(sh->T) + 127) / 128;
    if (n > most) n = most;
    return (int)(n < 1 ? 1 : (n > 64 ? 64 : n));
}
static size_t planes_bytes(const moe_shape_t *sh) {
    return (((size_t)3 * epad_of(sh->E) * tpad_of(sh->T) * 2) + 255) / 256 * 256;
}

size_t gate_bwd_ws_bytes(const moe_shape_t *sh) {
    if (sh->dtype == MOE_BF16)
        return planes_bytes(sh) + (size_t)dwg_chunks(sh) * epad_of(sh->E) * sh->h * 4;
    return (size_t)simple_chunks(sh) * sh->h * sh->E * 4;
}

template <int CW, int EJ>
static void launch_dx(const moe_shape_t *sh, const float *w_gate, const float *d_logits, void *d_x, int j0,
                      hipStream_t s, const void *d_buf = nullptr, const int32_t *expert = nullptr,
                      const int32_t *slot = nullptr, int tp_size = 1) {
    // chunks of 64 tokens, longer ones (a multiple of 64) when there would be more chunks than a grid's second
    // dimension takes
    int64_t chunk_len = 64;
    while ((sh->T + chunk_len - 1) / chunk_len > 65535) chunk_len *= 2;
    dim3 grid((unsigned)((sh->h + 256 * CW - 1) / (256 * CW)), (unsigned)((sh->T + chunk_len - 1) / chunk_len));
    hipLaunchKernelGGL((gate_dx_kernel<CW, EJ>), grid, dim3(256), 0, s, w_gate, d_logits, (bf16_t *)d_x, sh->T, sh->h,
                       sh->E, j0, chunk_len, (const bf16_t *)d_buf, expert, slot, (sh->C + tp_size - 1) / tp_size, tp_size);
}

// the matrix-core kernel keeps buffer row numbers in 32 bits
// (and moves rows through buffer resources whose offsets must stay below 2^31)
static bool dx_rows_ok(const moe_shape_t *sh, int tp_size = 1) {
    const double src_rows = (double)tp_size * sh->E * (double)((sh->C + tp_size - 1) / tp_size);
    return sh->E <= 64 && src_rows * sh->h * 2.0 < 2147483648.0 && (double)sh->T * sh->h * 2.0 < 2147483648.0 &&
           (sh->T + DX_TOKENS - 1) / DX_TOKENS <= 65535;      // one workgroup row per DX_TOKENS tokens in the grid's second dimension
}

static void launch_dx_mfma(const moe_shape_t *sh, const float *w_gate, const float *d_logits, void *d_x, hipStream_t s,
                           const void *d_buf = nullptr, const int32_t *expert = nullptr, const int32_t *slot = nullptr,
                           int tp_size = 1) {
    // a workgroup = 4 waves = 512 columns of one chunk of DX_TOKENS tokens; the chunk amortises the Wg^T
    // fragments (128 columns x E floats per wave) and is short enough to give every compute unit several workgroups
    dim3 grid((unsigned)((sh->h + 511) / 512), (unsigned)((sh->T + DX_TOKENS - 1) / DX_TOKENS));
    const int E8 = (sh->E + 7) & ~7;
    const size_t lds = (size_t)512 * (E8 + 4) * 4 + (DX_TOKENS + 48) * 4;       // 512 >= DX_TOKENS + 16 rows
    static_assert(DX_TOKENS + 16 <= 512, "the d_logits rows reuse the 512-row region");
    // more than 64 KB of dynamic LDS has to be allowed per kernel (E > 32: up to 139 KB)
#define MOE_DX_ROWS(KS, GATHER)                                                                                      \
    do {                                                                                                             \
        if (lds > 65536)                                                                                             \
            (void)hipFuncSetAttribute((const void *)gate_dx_rows_kernel<KS, GATHER>,                                 \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                        \
        hipLaunchKernelGGL((gate_dx_rows_kernel<KS, GATHER>), grid, dim3(256), lds, s, w_gate, d_logits,             \
                           (bf16_t *)d_x, sh->T, sh->h, sh->E, (const bf16_t *)d_buf, expert, slot,                  \
                           (sh->C + tp_size - 1) / tp_size, tp_size);                                                \
    } while (0)
    if (d_buf) {
        if (sh->E <= 32) MOE_DX_ROWS(1, true);
        else MOE_DX_ROWS(2, true);
    } else {
        if (sh->E <= 32) MOE_DX_ROWS(1, false);
        else MOE_DX_ROWS(2, false);
    }
#undef MOE_DX_ROWS
}

moe_status_t run_gate_bwd(const moe_shape_t *sh, const float *d_gate_p, const float *probs, const int32_t *expert,
                          const void *x, const float *w_gate, float *d_logits, float *d_w_gate, void *d_x_accum,
                          void *ws, hipStream_t s) {
    if (sh->dtype != MOE_BF16)
        return run_gate_bwd_simple(sh, d_gate_p, probs, expert, x, w_gate, d_logits, d_w_gate, d_x_accum, ws, s);
    const int E = sh->E, Epad = epad_of(E);
    const int64_t T = sh->T, Tpad = tpad_of(T);
    if (!d_w_gate) {
        const int64_t n = T * E;
        hipLaunchKernelGGL(gate_dlogits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_gate_p, probs,
                           expert, d_logits, T, E);
    } else {
        bf16_t *planes = (bf16_t *)ws;
        float *partial = (float *)((char *)ws + planes_bytes(sh));
        const int64_t n = (int64_t)Epad * Tpad;
        hipLaunchKernelGGL(gate_dlogits_planes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_gate_p,
                           probs, expert, d_logits, planes, T, E, Epad, Tpad);
        const int nch = dwg_chunks(sh);
        int64_t chunk_len = (Tpad + nch - 1) / nch;
        chunk_len = (chunk_len + 31) / 32 * 32;
        dim3 grid((unsigned)((sh->h + 255) / 256), (unsigned)nch);
        const bf16_t *xb = (const bf16_t *)x;
        // up to 64 experts per launch (4 accumulator blocks of 16 experts)
        for (int e0 = 0; e0 < Epad; e0 += 64) {
            const int nt16 = (Epad - e0 < 64 ? Epad - e0 : 64) / 16;
            const bf16_t *pl = planes + (int64_t)e0 * Tpad;
            float *pa = partial + (int64_t)e0 * sh->h;
            switch (nt16) {
                case 1: hipLaunchKernelGGL((gate_dwg_mfma_kernel<1>), grid, dim3(256), 0, s, xb, pl, pa, T, sh->h, Tpad, chunk_len, Epad); break;
                case 2: hipLaunchKernelGGL((gate_dwg_mfma_kernel<2>), grid, dim3(256), 0, s, xb, pl, pa, T, sh->h, Tpad, chunk_len, Epad); break;
                case 3: hipLaunchKernelGGL((gate_dwg_mfma_kernel<3>), grid, dim3(256), 0, s, xb, pl, pa, T, sh->h, Tpad, chunk_len, Epad); break;
                default: hipLaunchKernelGGL((gate_dwg_mfma_kernel<4>), grid, dim3(256), 0, s, xb, pl, pa, T, sh->h, Tpad, chunk_len, Epad); break;
            }
        }
        const int64_t m = (int64_t)E * sh->h;
        hipLaunchKernelGGL(gate_dwg_reduce_t_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, s, partial,
                           d_w_gate, sh->h, E, Epad, nch);
    }
    if (d_x_accum) {
        if (dx_rows_ok(sh)) launch_dx_mfma(sh, w_gate, d_logits, d_x_accum, s);
        else
            for (int j0 = 0; j0 < E; j0 += 64) launch_dx<2, 64>(sh, w_gate, d_logits, d_x_accum, j0, s);
    }
    return check_launch("gate_bwd");
}

// fp32 storage: d_x[t,k] += sum_j d_logits[t,j] * w_gate[k,j], one thread per element (small workloads only)
__global__ void gate_dx_f32_kernel(const float *w_gate, const float *d_logits, float *d_x, int64_t T, int h, int E) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * h) return;
    const int64_t t = i / h;
    const int k = (int)(i - t * h);
    float s = 0.f;
    for (int j = 0; j < E; ++j) s = fmaf(d_logits[t * E + j], w_gate[(int64_t)k * E + j], s);
    d_x[i] += s;
}

moe_status_t run_gate_dx_f32(const moe_shape_t *sh, const float *d_logits, const float *w_gate, void *d_x,
                             hipStream_t s) {
    const int64_t n = sh->T * sh->h;
    hipLaunchKernelGGL(gate_dx_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w_gate, d_logits,
                       (float *)d_x, sh->T, sh->h, sh->E);
    return check_launch("gate_dx_f32");
}

// Dispatch backward with the gate's contribution fused in (bf16 storage):
//   d_x[t,:] = d_buf[expert[t], slot[t], :] (or 0) + d_logits[t,:] w_gate^T
moe_status_t run_dispatch_bwd_fused(const moe_shape_t *sh, const void *d_buf, const int32_t *expert,
                                    const int32_t *slot, void *d_x, const float *d_logits, const float *w_gate,
                                    hipStream_t s, int tp_size) {
    const int E = sh->E;
    if (dx_rows_ok(sh, tp_size)) launch_dx_mfma(sh, w_gate, d_logits, d_x, s, d_buf, expert, slot, tp_size);
    else {
        launch_dx<2, 64>(sh, w_gate, d_logits, d_x, 0, s, d_buf, expert, slot, tp_size);
        for (int j0 = 64; j0 < E; j0 += 64) launch_dx<2, 64>(sh, w_gate, d_logits, d_x, j0, s);
    }
    return check_launch("dispatch_bwd_fused");
}

}  // namespace moe
