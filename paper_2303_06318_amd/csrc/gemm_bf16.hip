// Grouped bf16 GEMM on gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) for the
// expert FFN: forward (Z = D W1 with fused GeLU, Y = H W2), data gradients (dH = dY W2^T with
// fused GeLU', dD = dZ W1^T) and weight gradients (dW = A^T B over the kept rows).
//
// One workgroup of 512 threads (8 waves, 2 x 4) owns a 256 x 256 output tile of one expert and
// walks K in steps of 64 through two LDS stages (global -> registers -> LDS, one barrier per
// step).  Each wave owns 128 x 64 of the tile: 4 x 2 MFMA blocks of 32 x 32.
//
// Operands are taken in the layout the layer stores them in, so no transposed copy is ever made:
//   "KC" operand: the reduction index is contiguous in memory  -> LDS tile [256][64], 16-byte
//                 LDS reads deliver 8 consecutive k to a lane directly;
//   "XC" operand: the output index is contiguous in memory     -> LDS tile [64][256], read with
//                 the LDS transpose load (ds_read_b64_tr_b16), which hands lane i of a 16-lane
//                 group the i-th column of a 4 x 16 block.
// Rows beyond kept[e] are never read (loaded as zero) and never written.
#include "moe_common.h"

namespace moe {

constexpr int BM = 256, BN = 256, BK = 64, GEMM_THREADS = 512;
constexpr int KC_LD = BK + 8;         // 144-byte rows: 16 consecutive rows hit 16 distinct 16-byte bank groups
constexpr int XC_LD = 256 + 32;       // 576-byte k-rows: 4 consecutive k-rows land in 4 distinct 64-byte quarters
constexpr int STAGE_ELEMS = 256 * KC_LD;   // == 64 * XC_LD
static_assert(256 * KC_LD == 64 * XC_LD, "both tile shapes share one stage size");
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// GeLU for the bf16 epilogues: erf by the Abramowitz-Stegun 7.1.26 rational form (absolute error
// 1.5e-7, far below bf16 resolution) with hardware exp and reciprocal; no branches.
__device__ __forceinline__ float erf_exp_fast(float u, float &ex) {   // u >= 0; ex = exp(-u*u)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, u, 1.0f));
    ex = __expf(-u * u);
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    return 1.0f - p * t * ex;
}
__device__ __forceinline__ float tanh_fast(float u) {
    const float e2 = __expf(2.0f * u);
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e2 + 1.0f);
}
__device__ __forceinline__ float gelu_fast(float x, int act) {
    if (act == MOE_GELU_TANH) {
        const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
        return 0.5f * x * (1.0f + tanh_fast(u));
    }
    float ex;
    const float er = erf_exp_fast(fabsf(x) * 0.7071067811865476f, ex);
    return 0.5f * x * (1.0f + copysignf(er, x));
}
__device__ __forceinline__ float gelu_grad_fast(float x, int act) {
    if (act == MOE_GELU_TANH) {
        const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
        const float th = tanh_fast(u);
        const float du = 0.7978845608028654f * (1.0f + 0.134145f * x * x);
        return 0.5f * (1.0f + th) + 0.5f * x * (1.0f - th * th) * du;
    }
    float ex;
    const float er = erf_exp_fast(fabsf(x) * 0.7071067811865476f, ex);
    return 0.5f * (1.0f + copysignf(er, x)) + x * ex * 0.3989422804014327f;
}

struct TileLoader {
    u32x4 r[4];
};

// Buffer resource over one expert's operand: loads beyond `bytes` (and lanes whose offset is forced
// out of range) return zero without a branch.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
constexpr uint32_t OOB = 0x80000000u;

// global -> registers for one operand's k-tile.  xc: tile is [64 k][256 x]; else [256 x][64 k].
// xoff[p] is the byte offset of this thread's p-th 16-byte piece at k = 0 (already out of range
// when its row/column lies outside the operand); the k part is added per tile.
template <bool XC>
__device__ __forceinline__ void loader_init(uint32_t (&xoff)[4], int ld, int x0, int xlim, int tid) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if (XC) {
            const int gx = x0 + (tid & 31) * 8;
            const uint32_t o = ((uint32_t)((tid >> 5) + 16 * p) * ld + gx) * 2u;
            xoff[p] = gx < xlim ? o : OOB;
        } else {
            const int gx = x0 + (tid >> 3) + 64 * p;
            const uint32_t o = ((uint32_t)gx * ld + (tid & 7) * 8) * 2u;
            xoff[p] = gx < xlim ? o : OOB;
        }
    }
}

template <bool XC>
__device__ __forceinline__ void load_tile(TileLoader &t, __amdgpu_buffer_rsrc_t rsrc, const uint32_t (&xoff)[4],
                                          int ld, int k0, int klim, int tid) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        uint32_t off;
        if (XC) {
            const int gk = k0 + (tid >> 5) + 16 * p;
            off = gk < klim ? xoff[p] + (uint32_t)k0 * ld * 2u : OOB;
        } else {
            const int gk = k0 + (tid & 7) * 8;
            off = gk < klim ? xoff[p] + (uint32_t)k0 * 2u : OOB;
        }
        t.r[p] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
    }
}

template <bool XC>
__device__ __forceinline__ void store_tile(const TileLoader &t, bf16_t *stage, int tid) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int off;
        if (XC)
            off = ((tid >> 5) + 16 * p) * XC_LD + (tid & 31) * 8;
        else
            off = ((tid >> 3) + 64 * p) * KC_LD + (tid & 7) * 8;
        *(u32x4 *)(stage + off) = t.r[p];
    }
}

// One 32 x 16 (x by k) MFMA operand fragment for lane `lane`: 8 k values of row/column x = xb + lane%32.
template <bool XC>
__device__ __forceinline__ bf16x8 read_frag(const bf16_t *stage, int xb, int ks, int lane) {
    if (XC) {
        int x = xb + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        int kr = ks * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
        const bf16_t *p0 = stage + kr * XC_LD + x;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p0));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p0 + 4 * XC_LD));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    } else {
        const bf16_t *p = stage + (xb + (lane & 31)) * KC_LD + ks * 16 + (lane >> 5) * 8;
        return *(const bf16x8 *)p;
    }
}

template <bool AXC, bool BXC, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmDesc d, int mt, int nt) {
    // XCD-aware order: consecutive workgroup ids go round-robin over the 8 XCDs, so give every
    // XCD one contiguous range of logical tiles (tiles that share a weight panel share an L2).
    const int nwg = gridDim.x, pid = blockIdx.x;
    const int xcd = pid & 7, per = nwg >> 3, rem = nwg & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (pid >> 3);
    const int e = logical / (mt * nt);
    const int rr = logical - e * (mt * nt);
    const int nti = rr / mt, mti = rr - nti * mt;     // m fastest: the m-tiles of one weight panel run together

    const int kept = d.kept[e];
    const int Me = d.rows_from_kept ? kept : d.M;
    const int Ke = d.rows_from_kept ? d.K : kept;
    const int m0 = mti * BM, n0 = nti * BN;
    if (m0 >= Me) return;

    const bf16_t *Ap = (const bf16_t *)d.A + (int64_t)e * d.strideA;
    const bf16_t *Bp = (const bf16_t *)d.B + (int64_t)e * d.strideB;
    // extent of this expert's operands in bytes (rows x row length)
    const uint32_t a_bytes = (uint32_t)(AXC ? Ke : Me) * (uint32_t)d.lda * 2u;
    const uint32_t b_bytes = (uint32_t)(BXC ? Ke : d.N) * (uint32_t)d.ldb * 2u;
    const __amdgpu_buffer_rsrc_t A = make_rsrc(Ap, a_bytes), B = make_rsrc(Bp, b_bytes);

    __shared__ __attribute__((aligned(16))) bf16_t lds[2][2][STAGE_ELEMS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 2) * 128, wn = (wave & 3) * 64;

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = (Ke + BK - 1) / BK;
    // Software pipeline.  Per k-tile and wave: 4 k-steps of 8 MFMAs.  Fragments are double
    // buffered (F0/F1) so every LDS read is issued one k-step (8 MFMAs) before its use; the next
    // tile's global data sits in registers (ta/tb) for a whole tile before it is written to the
    // other LDS stage.  Loads past K return zero (buffer bounds), so the loop body has no branches.
    bf16x8 a0[4], b0[2], a1[4], b1[2];
    TileLoader ta, tb;
    uint32_t xa[4], xb[4];
    loader_init<AXC>(xa, d.lda, m0, Me, tid);
    loader_init<BXC>(xb, d.ldb, n0, d.N, tid);
    auto rd = [&](bf16x8(&af)[4], bf16x8(&bf)[2], int stage, int ks) {
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = read_frag<AXC>(lds[stage][0], wm + i * 32, ks, lane);
#pragma unroll
        for (int j = 0; j < 2; ++j) bf[j] = read_frag<BXC>(lds[stage][1], wn + j * 32, ks, lane);
    };
    auto mma = [&](const bf16x8(&af)[4], const bf16x8(&bf)[2]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], af[i], acc[i][j], 0, 0, 0);
    };
    if (nk > 0) {
        load_tile<AXC>(ta, A, xa, d.lda, 0, Ke, tid);
        load_tile<BXC>(tb, B, xb, d.ldb, 0, Ke, tid);
        store_tile<AXC>(ta, lds[0][0], tid);
        store_tile<BXC>(tb, lds[0][1], tid);
        load_tile<AXC>(ta, A, xa, d.lda, BK, Ke, tid);
        load_tile<BXC>(tb, B, xb, d.ldb, BK, Ke, tid);
        __syncthreads();
        rd(a0, b0, 0, 0);
    }
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        rd(a1, b1, cur, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        rd(a0, b0, cur, 2);
        __builtin_amdgcn_sched_barrier(0);
        mma(a1, b1);
        __builtin_amdgcn_sched_barrier(0);
        rd(a1, b1, cur, 3);
        store_tile<AXC>(ta, lds[cur ^ 1][0], tid);
        store_tile<BXC>(tb, lds[cur ^ 1][1], tid);
        load_tile<AXC>(ta, A, xa, d.lda, (kt + 2) * BK, Ke, tid);
        load_tile<BXC>(tb, B, xb, d.ldb, (kt + 2) * BK, Ke, tid);
        mma(a0, b0);
        // interleave: one MFMA, one LDS write of the staged tile, one global load of the tile after it
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        rd(a0, b0, cur ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(a1, b1);
        __builtin_amdgcn_sched_barrier(0);
    }

    // Epilogue.  The MFMAs were issued with the operands swapped (B fragment first), so the
    // accumulators hold the transposed block: lane owns output row m = lane%32 and, per group of
    // four registers, four consecutive columns n = (v/4)*8 + (lane/32)*4 + v%4.  The tile is
    // converted to bf16, staged in LDS (the operand stages are free now; reads still in flight
    // from the loop's last prefetch are never used) and written out as full 512-byte rows.
    bf16_t *C = (bf16_t *)d.C + (int64_t)e * d.strideC;
    bf16_t *st = &lds[0][0][0];
    constexpr int CLD = BN + 8;
    static_assert(BM * CLD <= 4 * STAGE_ELEMS, "staging tile fits in the operand stages");
    const int act = d.act;
    auto for_each_quad = [&](auto fn) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    bf16_t *pos = st + (wm + i * 32 + (lane & 31)) * CLD + wn + j * 32 + vq * 8 + (lane >> 5) * 4;
                    f32x4 v = {acc[i][j][vq * 4], acc[i][j][vq * 4 + 1], acc[i][j][vq * 4 + 2], acc[i][j][vq * 4 + 3]};
                    fn(pos, v);
                }
    };
    auto put4 = [](bf16_t *pos, const f32x4 &v) {
        bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
        *(bf16x4 *)pos = o;
    };
    auto flush = [&](bf16_t *out) {
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = (tid >> 5) + 16 * p, gm = m0 + row, gn = n0 + (tid & 31) * 8;
            const u32x4 v = *(const u32x4 *)(st + row * CLD + (tid & 31) * 8);
            if (gm < Me && gn < d.N) *(u32x4 *)(out + (int64_t)gm * d.ldc + gn) = v;
        }
    };
    if (EPI == EPI_STORE) {
        for_each_quad([&](bf16_t *pos, const f32x4 &v) { put4(pos, v); });
        flush(C);
    } else if (EPI == EPI_GELU) {
        if (d.C2) {
            for_each_quad([&](bf16_t *pos, const f32x4 &v) { put4(pos, v); });
            flush((bf16_t *)d.C2 + (int64_t)e * d.strideC);
            __syncthreads();
        }
        for_each_quad([&](bf16_t *pos, const f32x4 &v) {
            f32x4 g = {gelu_fast(v[0], act), gelu_fast(v[1], act), gelu_fast(v[2], act), gelu_fast(v[3], act)};
            put4(pos, g);
        });
        flush(C);
    } else {
        const bf16_t *Zin = (const bf16_t *)d.Zin + (int64_t)e * d.strideC;
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = (tid >> 5) + 16 * p, gm = m0 + row, gn = n0 + (tid & 31) * 8;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (gm < Me && gn < d.N) v = *(const u32x4 *)(Zin + (int64_t)gm * d.ldc + gn);
            *(u32x4 *)(st + row * CLD + (tid & 31) * 8) = v;
        }
        __syncthreads();
        for_each_quad([&](bf16_t *pos, const f32x4 &v) {
            const bf16x4 z = *(const bf16x4 *)pos;
            f32x4 g = {v[0] * gelu_grad_fast((float)z[0], act), v[1] * gelu_grad_fast((float)z[1], act),
                       v[2] * gelu_grad_fast((float)z[2], act), v[3] * gelu_grad_fast((float)z[3], act)};
            put4(pos, g);
        });
        flush(C);
    }
}

template <bool AXC, bool BXC>
static void launch_epi(const GemmDesc &d, int mt, int nt, hipStream_t s) {
    dim3 grid((unsigned)((int64_t)d.E * mt * nt)), block(GEMM_THREADS);
    switch (d.epi) {
        case EPI_STORE:
            hipLaunchKernelGGL((gemm_bf16_kernel<AXC, BXC, EPI_STORE>), grid, block, 0, s, d, mt, nt);
            break;
        case EPI_GELU:
            hipLaunchKernelGGL((gemm_bf16_kernel<AXC, BXC, EPI_GELU>), grid, block, 0, s, d, mt, nt);
            break;
        default:
            hipLaunchKernelGGL((gemm_bf16_kernel<AXC, BXC, EPI_DGELU>), grid, block, 0, s, d, mt, nt);
            break;
    }
}

moe_status_t launch_gemm_bf16(const GemmDesc &d, hipStream_t s) {
    const int mt = (d.M + BM - 1) / BM, nt = (d.N + BN - 1) / BN;
    if (!d.a_xc && d.b_xc)
        launch_epi<false, true>(d, mt, nt, s);      // forward: A [M,K], B [K,N]
    else if (!d.a_xc && !d.b_xc)
        launch_epi<false, false>(d, mt, nt, s);     // data gradient: A [M,K], B [N,K]
    else if (d.a_xc && d.b_xc)
        launch_epi<true, true>(d, mt, nt, s);       // weight gradient: A [K,M], B [K,N]
    else {
        set_error("gemm_bf16: operand layout combination not built");
        return MOE_ERR_UNSUPPORTED;
    }
    return check_launch("gemm_bf16");
}

}  // namespace moe
