// Gate (routing function: linear map, softmax, top-1) and capacity-limited slot assignment.
//
// bf16 tokens: logits = X Wg on the matrix cores in one pass over X.  Wg stays fp32-accurate
// by splitting every weight into three bf16 pieces (hi + mid + lo == w to ~2^-24) and issuing
// three bf16 MFMAs into one fp32 accumulator; bf16 x bf16 products are exact in fp32, so the
// result has fp32 dot-product accuracy while X is streamed once at HBM speed.
// fp32 tokens: plain fp32 FMA dot products (small workloads only).
//
// Routing: per-token-block histograms of the chosen experts (integer LDS atomics: the result does not
// depend on their order), written by the gate kernel itself for bf16 tokens (a block = the 64 or 16
// tokens of a workgroup) and by a small kernel otherwise (blocks of 1024 tokens); then one kernel in
// which every block of 1024 tokens adds up the histograms of the tokens before it (all threads in
// parallel, integer atomics again), ranks its own tokens with wave ballots (token order inside a wave
// = lane order) and writes slot / token_of_slot; the last block writes counts and kept.
#include "moe_common.h"

namespace moe {

// ------------------------------------------------------------------ weight split
// ws layout: 3 planes [Epad][h] bf16 (k contiguous), rows >= E are zero.
__global__ void gate_split_wg_kernel(const float *wg, bf16_t *planes, int h, int E, int Epad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t n = (int64_t)Epad * h;
    if (i >= n) return;
    int e = (int)(i / h), k = (int)(i % h);
    float w = e < E ? wg[(int64_t)k * E + e] : 0.f;
    bf16_t hi = f32_to_bf16(w);
    float r1 = w - bf16_to_f32(hi);
    bf16_t mid = f32_to_bf16(r1);
    float r2 = r1 - bf16_to_f32(mid);
    bf16_t lo = f32_to_bf16(r2);
    planes[i] = hi;
    planes[n + i] = mid;
    planes[2 * n + i] = lo;
}

// ------------------------------------------------------------------ fused gate, bf16 tokens
// Workgroup: NW waves, 16*R tokens.  Wave w takes k-steps w, w+NW, ... (32 k each); the NW partial
// [16R x Epad] tiles are summed through LDS in a fixed order.  The three planes of Wg are read from
// L2 once per workgroup, so R is chosen large enough that this traffic stays below that of X.
template <int NT, int R, int NW, int U>
__global__ __launch_bounds__(64 * NW) void gate_bf16_kernel(const bf16_t *x, const bf16_t *planes, const float *bias,
                                                         float *logits, float *probs, int32_t *expert,
                                                         float *gate_p, int64_t T, int h, int E, int32_t *hist,
                                                         int32_t *token_of_slot, int64_t EC) {
    constexpr int EP = NT * 16;
    constexpr int TM = 16 * R;
    __shared__ float part[NW][TM][EP + 1];
    __shared__ int32_t hist_s[EP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t t0 = (int64_t)blockIdx.x * TM;
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t plane = (int64_t)EP * h;

    f32x4 acc[R][NT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[r][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Buffer resources: rows beyond the last token and k beyond h read as zero, so the loop has no
    // branches and U k-steps of loads are in flight per wave before their MFMAs issue.
    constexpr uint32_t OOB = 0x80000000u;
    const int64_t rows = T - t0 < TM ? T - t0 : TM;
    const __amdgpu_buffer_rsrc_t xr =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x + t0 * h), 0, (int)(rows * h * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t pr =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(planes), 0, (int)(3 * plane * 2), 0x00020000);
    const int nsteps = (h + 31) / 32;
    // A batch = U k-steps of this wave: all its requests (R token fragments and 3 NT plane fragments per
    // k-step) are issued together, and the arithmetic of a batch runs while the requests of the next one
    // are in flight: two register sets alternate.  The scheduling barriers keep the compiler from
    // trickling the loads out between the MFMAs (which it does to save registers, leaving a few KB in
    // flight per wave: the kernel is bound by memory latency).  Batches past the end read zeros.
    auto issue = [&](int s, bf16x8(&a)[U][R], bf16x8(&b)[U][NT][3]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = (s + NW * u) * 32 + g * 8;
            const uint32_t koff = k < h ? (uint32_t)k * 2u : OOB;
#pragma unroll
            for (int r = 0; r < R; ++r)
                a[u][r] = __builtin_bit_cast(
                    bf16x8, __builtin_amdgcn_raw_buffer_load_b128(xr, (uint32_t)(r * 16 + i16) * h * 2u + koff, 0, 0));
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int p = 0; p < 3; ++p)
                    b[u][n][p] = __builtin_bit_cast(
                        bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                                    pr, (uint32_t)(p * plane + (int64_t)(n * 16 + i16) * h) * 2u + koff, 0, 0));
        }
    };
    auto multiply = [&](const bf16x8(&a)[U][R], const bf16x8(&b)[U][NT][3]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        acc[r][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][r], b[u][n][p], acc[r][n], 0, 0, 0);
    };
    // All workgroups read the same Wg planes.  Walking k in the same order, the workgroups of an XCD would ask
    // its L2 for the same few lines at the same time (one or two of its 16 channels serving everybody), so each
    // workgroup starts at a different batch and wraps around.
    constexpr int BS = NW * U;                                   // k-steps per batch of the workgroup
    const int nbatch = (nsteps + BS - 1) / BS;
    const int nbatch2 = (nbatch + 1) & ~1;                       // the loop body holds two batches
    const int rot = (int)((blockIdx.x >> 3) % (unsigned)nbatch2);        // blockIdx / 8: index inside the XCD
    auto first_step = [&](int i) {                               // batch i of this workgroup, rotated; past the end: zeros
        int bi = i + rot;
        bi = bi >= nbatch2 ? bi - nbatch2 : bi;
        return i < nbatch2 ? bi * BS + wave : nsteps;
    };
    constexpr bool TWO_SETS = 2 * U * (R + 3 * NT) * 4 <= 200;   // registers of two batches of fragments
    if constexpr (TWO_SETS) {
        bf16x8 aA[U][R], bA[U][NT][3], aB[U][R], bB[U][NT][3];
        issue(first_step(0), aA, bA);
        for (int i = 0; i < nbatch2; i += 2) {
            issue(first_step(i + 1), aB, bB);
            __builtin_amdgcn_sched_barrier(0);
            multiply(aA, bA);
            __builtin_amdgcn_sched_barrier(0);
            issue(first_step(i + 2), aA, bA);
            __builtin_amdgcn_sched_barrier(0);
            multiply(aB, bB);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {                                                     // many experts: one batch at a time
        bf16x8 aA[U][R], bA[U][NT][3];
        for (int i = 0; i < nbatch2; ++i) {
            issue(first_step(i), aA, bA);
            __builtin_amdgcn_sched_barrier(0);
            multiply(aA, bA);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // 16x16 result: lane holds column (expert) lane%16, rows (tokens) 4*(lane/16) + v
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[wave][r * 16 + g * 4 + v][n * 16 + i16] = acc[r][n][v];
    __syncthreads();
    for (int idx = tid; idx < TM * E; idx += 64 * NW) {
        int tt = idx / E, j = idx - tt * E;
        float v = part[0][tt][j];
#pragma unroll
        for (int w = 1; w < NW; ++w) v += part[w][tt][j];
        if (bias) v += bias[j];
        part[0][tt][j] = v;
        if (t0 + tt < T) logits[(t0 + tt) * E + j] = v;
    }
    if (tid < EP) hist_s[tid] = 0;
    __syncthreads();
    // Softmax and top-1 with TPT adjacent lanes per token: lane `sub` looks at experts sub, sub + TPT, ...;
    // the lanes' candidates are merged by butterfly exchanges (larger logit wins, the lower index among
    // equal ones: the same choice as a left-to-right scan with a strict comparison).
    constexpr int TPT = 64 * NW / TM;
    static_assert(TPT >= 1 && (TPT & (TPT - 1)) == 0 && TPT <= 64, "lanes per token");
    const int tt = tid / TPT, sub = tid % TPT;
    const float *row = &part[0][tt][0];
    float best = -__builtin_inff();
    int bi = 0x7fffffff;
    for (int j = sub; j < E; j += TPT) {
        const float v = row[j];
        if (v > best || bi == 0x7fffffff) { best = v; bi = j; }      // strict: the first of equal values stays
    }
#pragma unroll
    for (int o = 1; o < TPT; o <<= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    float denom = 0.f;
    for (int j = sub; j < E; j += TPT) denom += expf(row[j] - best);
#pragma unroll
    for (int o = 1; o < TPT; o <<= 1) denom += __shfl_xor(denom, o);
    const float inv = 1.0f / denom;
    const int64_t t = t0 + tt;
    if (t < T) {
        if (probs)
            for (int j = sub; j < E; j += TPT) probs[t * E + j] = expf(row[j] - best) * inv;
        if (sub == 0) {
            expert[t] = bi;
            gate_p[t] = inv;
            atomicAdd(&hist_s[bi], 1);
        }
    }
    __syncthreads();
    // the routing kernel's inputs: this block's histogram, and its share of the inverse map cleared
    if (tid < E) hist[(int64_t)blockIdx.x * E + tid] = hist_s[tid];
    const int64_t per = (EC + gridDim.x - 1) / gridDim.x, i0 = (int64_t)blockIdx.x * per;
    for (int64_t i = i0 + tid; i < i0 + per && i < EC; i += 64 * NW) token_of_slot[i] = -1;
}

// ------------------------------------------------------------------ fp32 tokens: logits by fp32 FMA, one wave per token
__global__ __launch_bounds__(256) void gate_logits_f32_kernel(const float *x, const float *wg, const float *bias,
                                                              float *logits, int64_t T, int h, int E) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    for (int j0 = 0; j0 < E; j0 += 16) {
        float acc[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0.f;
        for (int k = lane; k < h; k += 64) {
            float xv = x[t * h + k];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (j0 + j < E) acc[j] = fmaf(xv, wg[(int64_t)k * E + j0 + j], acc[j]);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float v = acc[j];
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
            if (lane == 0 && j0 + j < E) logits[t * E + j0 + j] = v + (bias ? bias[j0 + j] : 0.f);
        }
    }
}

// softmax + top-1 from stored logits: 16 adjacent lanes per token, lane `sub` looks at experts sub, sub + 16, ...
// (consecutive lanes read consecutive logits); candidates merged by butterfly exchanges, lower index among equals
constexpr int SM_TPT = 16;
__global__ __launch_bounds__(256) void gate_softmax_top1_kernel(const float *logits, float *probs, int32_t *expert,
                                                                 float *gate_p, int64_t T, int E) {
    const int64_t t = ((int64_t)blockIdx.x * 256 + threadIdx.x) / SM_TPT;
    const int sub = threadIdx.x % SM_TPT;
    const float *row = logits + (t < T ? t : 0) * E;         // lanes past the end work on row 0 and write nothing
    float best = -__builtin_inff();
    int bi = 0x7fffffff;
    for (int j = sub; j < E; j += SM_TPT) {
        const float v = row[j];
        if (v > best || bi == 0x7fffffff) { best = v; bi = j; }
    }
#pragma unroll
    for (int o = 1; o < SM_TPT; o <<= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    float denom = 0.f;
    for (int j = sub; j < E; j += SM_TPT) denom += expf(row[j] - best);
#pragma unroll
    for (int o = 1; o < SM_TPT; o <<= 1) denom += __shfl_xor(denom, o);
    const float inv = 1.0f / denom;
    if (t >= T) return;
    if (probs)
        for (int j = sub; j < E; j += SM_TPT) probs[t * E + j] = expf(row[j] - best) * inv;
    if (sub == 0) {
        expert[t] = bi;
        gate_p[t] = inv;
    }
}

// ------------------------------------------------------------------ routing
constexpr int RB = 1024;   // tokens per routing block
constexpr unsigned ROUTE_DIRECT_BLOCKS = 64;   // up to this many routing blocks, each sums the histograms in front of it itself

__global__ __launch_bounds__(RB) void route_hist_kernel(const int32_t *expert, int32_t *hist, int32_t *token_of_slot,
                                                         int64_t T, int E, int64_t EC) {
    __shared__ int32_t h[256];
    const int tid = threadIdx.x;
    if (tid < E) h[tid] = 0;
    __syncthreads();
    int64_t t = (int64_t)blockIdx.x * RB + tid;
    if (t < T) atomicAdd(&h[expert[t]], 1);
    __syncthreads();
    if (tid < E) hist[(int64_t)blockIdx.x * E + tid] = h[tid];
    for (int64_t i = (int64_t)blockIdx.x * RB + tid; i < EC; i += (int64_t)gridDim.x * RB) token_of_slot[i] = -1;
}

// Many routing blocks (long token tensors): the tokens in front of every routing block, per expert, by one
// pass over the histogram rows instead of every block summing all rows in front of it.  Workgroup e walks the
// routing blocks 1024 at a time: a thread adds up the rows of one block, the workgroup scans the totals
// (wave shuffles, then the 16 wave totals), and the running sum carries over to the next 1024 blocks.
// block_base[b * E + e] = tokens of expert e in routing blocks 0 .. b-1.
__global__ __launch_bounds__(1024) void route_block_base_kernel(const int32_t *hist, int32_t *block_base, int64_t n_rows,
                                                                 int64_t n_blocks, int E, int rows_per_block) {
    __shared__ int32_t wsum[16];
    __shared__ int32_t carry_s;
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int64_t b0 = 0; b0 < n_blocks; b0 += 1024) {
        const int64_t b = b0 + tid;
        int32_t tot = 0;
        if (b < n_blocks) {
            const int64_t r0 = b * rows_per_block;
            for (int r = 0; r < rows_per_block && r0 + r < n_rows; ++r) tot += hist[(r0 + r) * E + e];
        }
        int32_t inc = tot;                           // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        int32_t before = carry_s;                    // the carry and the waves in front of this one
        for (int w = 0; w < wave; ++w) before += wsum[w];
        if (b < n_blocks) block_base[b * E + e] = before + inc - tot;
        __syncthreads();
        if (tid == 1023) carry_s = before + inc;
        __syncthreads();
    }
}

// hist holds one row of E counts per `hist_block` tokens (RB is a multiple of hist_block).  block_base: the
// result of route_block_base_kernel, or null (few routing blocks: every block sums the rows in front of it).
__global__ __launch_bounds__(RB) void route_slot_kernel(const int32_t *expert, const int32_t *hist, int32_t *slot,
                                                         int32_t *counts, int32_t *kept, int32_t *token_of_slot,
                                                         int64_t T, int E, int64_t C, int hist_block,
                                                         const int32_t *block_base) {
    __shared__ int32_t base[256];
    __shared__ int32_t wcnt[RB / 64][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    for (int i = tid; i < (RB / 64) * 256; i += RB) (&wcnt[0][0])[i] = 0;
    if (tid < 256) base[tid] = 0;
    __syncthreads();
    // tokens before this block: all histogram rows in front of it, summed by all threads at once
    // (consecutive threads read consecutive counts; integer atomics, so the order does not matter)
    if (block_base != nullptr) {
        if (tid < E) base[tid] = block_base[(int64_t)b * E + tid];
    } else {
        const int64_t n_before = (int64_t)b * (RB / hist_block) * E;
        for (int64_t i = tid; i < n_before; i += RB) {
            const int32_t v = hist[i];
            if (v) atomicAdd(&base[(int)(i % E)], v);
        }
    }
    __syncthreads();
    const int64_t t = (int64_t)b * RB + tid;
    const int e = t < T ? expert[t] : -1;
    int rank = 0;
    unsigned long long remaining = __ballot(e >= 0);
    while (remaining) {
        const int leader = __ffsll((long long)remaining) - 1;
        const int e0 = __shfl(e, leader);
        const unsigned long long m = __ballot(e == e0);
        if (e == e0) {
            rank = __popcll(m & ((1ull << lane) - 1ull));
            if (lane == leader) wcnt[wave][e0] = __popcll(m);
        }
        remaining &= ~m;
    }
    __syncthreads();
    if (tid < E) {       // exclusive prefix over the block's waves, in wave order
        int32_t s = base[tid];
        for (int w = 0; w < RB / 64; ++w) {
            int32_t c = wcnt[w][tid];
            wcnt[w][tid] = s;
            s += c;
        }
        if (b == (int)gridDim.x - 1) {
            counts[tid] = s;
            kept[tid] = s < C ? s : (int32_t)C;
        }
    }
    __syncthreads();
    if (e >= 0) {
        const int64_t s = (int64_t)wcnt[wave][e] + rank;
        if (s < C) {
            slot[t] = (int32_t)s;
            token_of_slot[(int64_t)e * C + s] = (int32_t)t;
        } else {
            slot[t] = -1;
        }
    }
}

// ------------------------------------------------------------------ host side
size_t gate_ws_bytes(const moe_shape_t *sh) {
    int NT = 1;
    while (NT * 16 < sh->E) NT *= 2;
    size_t planes = (size_t)3 * NT * 16 * sh->h * 2;
    size_t hist = (size_t)((sh->T + 15) / 16) * sh->E * 4;        // one row per 16 tokens at most (see run_gate)
    size_t bases = (size_t)((sh->T + RB - 1) / RB) * sh->E * 4;   // tokens in front of every routing block
    return ((planes + 255) / 256) * 256 + ((hist + 255) / 256) * 256 + ((bases + 255) / 256) * 256;
}

template <int NT, int R, int NW, int U>
static void launch_gate_bf16(const moe_shape_t *sh, const void *x, const bf16_t *planes, const float *bias,
                             float *logits, float *probs, int32_t *expert, float *gate_p, int32_t *hist,
                             int32_t *token_of_slot, hipStream_t s) {
    const int TM = 16 * R;
    dim3 grid((unsigned)((sh->T + TM - 1) / TM));
    hipLaunchKernelGGL((gate_bf16_kernel<NT, R, NW, U>), grid, dim3(64 * NW), 0, s, (const bf16_t *)x, planes, bias, logits,
                       probs, expert, gate_p, sh->T, sh->h, sh->E, hist, token_of_slot, (int64_t)sh->E * sh->C);
}

moe_status_t run_gate(const moe_shape_t *sh, const void *x, const float *w_gate, const float *bias, float *logits,
                      float *probs, int32_t *expert, float *gate_p, int32_t *slot, int32_t *counts, int32_t *kept,
                      int32_t *token_of_slot, void *ws, hipStream_t s) {
    int NT = 1;
    while (NT * 16 < sh->E) NT *= 2;
    const size_t planes_bytes = (((size_t)3 * NT * 16 * sh->h * 2 + 255) / 256) * 256;
    bf16_t *planes = (bf16_t *)ws;
    int32_t *hist = (int32_t *)((char *)ws + planes_bytes);
    const int64_t T = sh->T;
    if (x == nullptr) {
        hipLaunchKernelGGL(gate_softmax_top1_kernel, dim3((unsigned)((T * SM_TPT + 255) / 256)), dim3(256), 0, s, logits,
                           probs, expert, gate_p, T, sh->E);
    } else if (sh->dtype == MOE_F32) {
        hipLaunchKernelGGL(gate_logits_f32_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, s, (const float *)x,
                           w_gate, bias, logits, T, sh->h, sh->E);
        hipLaunchKernelGGL(gate_softmax_top1_kernel, dim3((unsigned)((T * SM_TPT + 255) / 256)), dim3(256), 0, s, logits,
                           probs, expert, gate_p, T, sh->E);
    } else {
        const int64_t n = (int64_t)NT * 16 * sh->h;
        hipLaunchKernelGGL(gate_split_wg_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w_gate, planes,
                           sh->h, sh->E, NT * 16);
        // template arguments: 16-expert tiles, tokens per workgroup / 16, waves, k-steps per batch (two batches in
        // flight per wave: 2 U (R + 3 NT) fragments of 4 registers)
        switch (NT) {
            case 1: launch_gate_bf16<1, 4, 8, 2>(sh, x, planes, bias, logits, probs, expert, gate_p, hist, token_of_slot, s); break;
            case 2: launch_gate_bf16<2, 4, 8, 2>(sh, x, planes, bias, logits, probs, expert, gate_p, hist, token_of_slot, s); break;
            case 4: launch_gate_bf16<4, 4, 8, 1>(sh, x, planes, bias, logits, probs, expert, gate_p, hist, token_of_slot, s); break;
            case 8: launch_gate_bf16<8, 1, 4, 1>(sh, x, planes, bias, logits, probs, expert, gate_p, hist, token_of_slot, s); break;
            default: launch_gate_bf16<16, 1, 4, 1>(sh, x, planes, bias, logits, probs, expert, gate_p, hist, token_of_slot, s); break;
        }
    }
    moe_status_t st = check_launch("gate");
    if (st != MOE_OK) return st;
    const unsigned nb = (unsigned)((T + RB - 1) / RB);
    int hist_block = RB;
    if (x != nullptr && sh->dtype == MOE_BF16) {
        hist_block = NT >= 8 ? 16 : 64;          // the gate kernel has written a histogram per workgroup (16 R tokens)
    } else {
        hipLaunchKernelGGL(route_hist_kernel, dim3(nb), dim3(RB), 0, s, expert, hist, token_of_slot, T, sh->E,
                           (int64_t)sh->E * sh->C);
    }
    // beyond ROUTE_DIRECT_BLOCKS routing blocks one more small kernel sums the histograms once for all
    int32_t *block_base = nullptr;
    if (nb > ROUTE_DIRECT_BLOCKS) {
        const size_t hist_bytes = (((size_t)((T + 15) / 16) * sh->E * 4 + 255) / 256) * 256;
        block_base = (int32_t *)((char *)hist + hist_bytes);
        hipLaunchKernelGGL(route_block_base_kernel, dim3((unsigned)sh->E), dim3(1024), 0, s, hist, block_base,
                           (T + hist_block - 1) / hist_block, (int64_t)nb, sh->E, RB / hist_block);
    }
    hipLaunchKernelGGL(route_slot_kernel, dim3(nb), dim3(RB), 0, s, expert, hist, slot, counts, kept, token_of_slot,
                       T, sh->E, sh->C, hist_block, block_base);
    return check_launch("route");
}

}  // namespace moe
