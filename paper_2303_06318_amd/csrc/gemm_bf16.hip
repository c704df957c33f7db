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

struct TileLoader {
    u32x4 r[4];
};

// global -> registers for one operand's k-tile.  xc: tile is [64 k][256 x]; else [256 x][64 k].
template <bool XC>
__device__ __forceinline__ void load_tile(TileLoader &t, const bf16_t *base, int ld, int x0, int xlim, int k0,
                                          int klim, int tid) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int gx, gk;
        if (XC) {
            gx = x0 + (tid & 31) * 8;
            gk = k0 + (tid >> 5) + 16 * p;
        } else {
            gx = x0 + (tid >> 3) + 64 * p;
            gk = k0 + (tid & 7) * 8;
        }
        u32x4 v = {0u, 0u, 0u, 0u};
        if (gx < xlim && gk < klim) {
            const bf16_t *ptr = XC ? base + (int64_t)gk * ld + gx : base + (int64_t)gx * ld + gk;
            v = *(const u32x4 *)ptr;
        }
        t.r[p] = v;
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

    const bf16_t *A = (const bf16_t *)d.A + (int64_t)e * d.strideA;
    const bf16_t *B = (const bf16_t *)d.B + (int64_t)e * d.strideB;

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
    TileLoader ta, tb;
    if (nk > 0) {
        load_tile<AXC>(ta, A, d.lda, m0, Me, 0, Ke, tid);
        load_tile<BXC>(tb, B, d.ldb, n0, d.N, 0, Ke, tid);
        store_tile<AXC>(ta, lds[0][0], tid);
        store_tile<BXC>(tb, lds[0][1], tid);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            load_tile<AXC>(ta, A, d.lda, m0, Me, (kt + 1) * BK, Ke, tid);
            load_tile<BXC>(tb, B, d.ldb, n0, d.N, (kt + 1) * BK, Ke, tid);
        }
        const bf16_t *sa = lds[cur][0], *sb = lds[cur][1];
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[4], bfr[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = read_frag<AXC>(sa, wm + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) bfr[j] = read_frag<BXC>(sb, wn + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            store_tile<AXC>(ta, lds[cur ^ 1][0], tid);
            store_tile<BXC>(tb, lds[cur ^ 1][1], tid);
        }
        __syncthreads();
    }

    // Epilogue.  Lane holds column n = lane%32 of each 32x32 block; element v is row
    // (v/4)*8 + (lane/32)*4 + v%4.
    bf16_t *C = (bf16_t *)d.C + (int64_t)e * d.strideC;
    bf16_t *C2 = (EPI == EPI_GELU && d.C2) ? (bf16_t *)d.C2 + (int64_t)e * d.strideC : nullptr;
    const bf16_t *Zin = (EPI == EPI_DGELU) ? (const bf16_t *)d.Zin + (int64_t)e * d.strideC : nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int gn = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int gm = m0 + wm + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (gm < Me && gn < d.N) {
                    const int64_t o = (int64_t)gm * d.ldc + gn;
                    float x = acc[i][j][v];
                    if (EPI == EPI_GELU) {
                        if (C2) C2[o] = f32_to_bf16(x);
                        C[o] = f32_to_bf16(act_fwd(x, d.act));
                    } else if (EPI == EPI_DGELU) {
                        C[o] = f32_to_bf16(x * act_grad(bf16_to_f32(Zin[o]), d.act));
                    } else {
                        C[o] = f32_to_bf16(x);
                    }
                }
            }
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
