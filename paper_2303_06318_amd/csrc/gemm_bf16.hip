// Grouped bf16 GEMM on gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) for the
// expert FFN: forward (Z = D W1 with fused GeLU and GeLU', Y = H W2), data gradients (dH = dY W2^T
// times the saved GeLU', dD = dZ W1^T) and weight gradients (dW = A^T B over the kept rows).
//
// One workgroup of 512 threads (8 waves, 2 x 4) owns a 256 x 256 output tile of one expert and
// walks K in 32-deep tiles through four 32 KB LDS stages (three tiles, 96 KB, in flight).  Each
// wave owns 128 x 64 of the tile: 4 x 2 MFMA blocks of 32 x 32.  Global data goes straight into
// LDS (buffer_load ... lds, 16 bytes per lane, no register staging); out-of-range lanes deliver
// zeros, so ragged row counts and K tails need no branches.  The two waves of a SIMD alternate
// between a memory phase and an MFMA phase, half an iteration apart (see the main loop).
//
// Operands are taken in the layout the layer stores them in, so no transposed copy is ever made:
//   "KC" operand: the reduction index is contiguous in memory  -> LDS tile [256 x][64 k], 16-byte
//                 LDS reads deliver 8 consecutive k to a lane directly;
//   "XC" operand: the output index is contiguous in memory     -> LDS tile [64 k][256 x], read with
//                 the LDS transpose load (ds_read_b64_tr_b16), which hands lane i of a 16-lane
//                 group the i-th column of a 4 x 16 block.
// A direct-to-LDS load writes lane L's 16 bytes at base + 16 L, so tiles cannot be padded; bank
// conflicts are avoided by XOR-swizzling the 16-byte granules inside each row instead:
//   KC: granule g of row r sits at position g ^ ((r >> 1) & 7)   (rows are 128 bytes)
//   XC: granule g of k-row k sits at position g ^ ((k & 3) << 2) (k-rows are 512 bytes)
// Rows beyond kept[e] are never read (loaded as zero) and never written.
#include <type_traits>
#include "moe_common.h"

namespace moe {

constexpr int BM = 256, BN = 256, BK = 32, GEMM_THREADS = 512;
constexpr int KS = BK / 16;                    // MFMA k-steps per k-tile
constexpr int CPW = BK / 16;                   // 1 KB chunks per wave, operand and k-tile
constexpr int KC_ROW = BK * 2;                 // bytes of one KC row in LDS
constexpr int KC_G = BK / 8;                   // 16-byte granules per KC row
constexpr int KC_SWZ_SHIFT = 2;                // rows per 256 bytes
constexpr int LIGHT_BLOCKS = 4;                // an expert with at most this many 32-row blocks is one "light" tile
constexpr int MAXB = 9;                        // 32-row blocks of a tile when A is a KC operand: 8, or 9 in a "tall" tile
constexpr int A_ROWS = MAXB * 32;              // rows of the A stage and of the epilogue staging tile
constexpr int NSTAGE = 4;                      // LDS stages; tiles are requested NSTAGE-1 k-tiles ahead
constexpr int OPER_BYTES = 256 * BK * 2;       // 256 rows or columns of one operand's k-tile (16 KB)
constexpr int OPER_A_BYTES = A_ROWS * BK * 2;  // A's part of a stage: room for the ninth block of a tall tile (18 KB)
constexpr int STAGE_BYTES = OPER_A_BYTES + OPER_BYTES;
constexpr int CLD = BN + 8;                    // epilogue staging row (elements)
constexpr int SMEM_BYTES = A_ROWS * CLD * 2 > NSTAGE * STAGE_BYTES ? A_ROWS * CLD * 2 : NSTAGE * STAGE_BYTES;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;

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
// GeLU and its derivative together (they share the erf / tanh and the exponential).
__device__ __forceinline__ void gelu_both_fast(float x, int act, float &h, float &g) {
    if (act == MOE_GELU_TANH) {
        const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
        const float th = tanh_fast(u);
        const float du = 0.7978845608028654f * (1.0f + 0.134145f * x * x);
        const float phi = 0.5f * (1.0f + th);
        h = x * phi;
        g = phi + 0.5f * x * (1.0f - th * th) * du;
        return;
    }
    float ex;
    const float er = erf_exp_fast(fabsf(x) * 0.7071067811865476f, ex);
    const float phi = 0.5f * (1.0f + copysignf(er, x));
    h = x * phi;
    g = phi + x * ex * 0.3989422804014327f;
}

// Buffer resource (raw, stride 0) over one expert's operand: lanes whose byte offset is not below
// `bytes` -- including offsets forced to OOB -- deliver zero without a branch.
typedef __attribute__((ext_vector_type(4))) int i32x4;
__device__ __forceinline__ i32x4 make_rsrc(const void *p, uint32_t bytes) {
    const uint64_t a = (uint64_t)p;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}
constexpr uint32_t OOB = 0x80000000u;

// One direct global -> LDS load: lane L's 16 bytes land at LDS byte address lds_addr + 16 L.
// Written as inline assembly so that the compiler does not order later LDS reads of the *other*
// stage behind it; completion is awaited explicitly (s_waitcnt vmcnt) before the stage is read.
__device__ __forceinline__ void load_to_lds(const i32x4 &rsrc, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

// Per-thread state of the global -> LDS copy of one operand.  A wave copies CPW consecutive chunks
// of the tile's one-KB chunks; lane L fills granule L of the chunk.
//   KC chunk: 1024 / KC_ROW rows, lane L -> row L / KC_G, position L % KC_G
//   XC chunk: 2 k-rows x 512 bytes, lane L -> k-row L/32, position L%32
struct Loader {
    uint32_t off[CPW];    // byte offset of this lane's granule at k-tile 0 (OOB if outside the operand in x)
    int32_t kthr[CPW];    // the granule is inside K for k-tile origin k0 iff k0 < kthr
};

// Where row gx of a KC operand lives in the array its resource covers, when that is not row gx itself:
// through an index array (negative entry: no such row), or in the row shares of duplicate token dropping
// (share gx % G, row base + gx / G of that share).
struct RowMap {
    const int32_t *index;
    int32_t G, share_rows, base;          // G > 0: shares of share_rows rows each; base = first row of this expert in a share
    __device__ __forceinline__ bool mapped() const { return index != nullptr || G > 0; }
    __device__ __forceinline__ int row(int gx) const {
        return index != nullptr ? index[gx] : (gx % G) * share_rows + base + gx / G;
    }
};

template <bool XC>
__device__ __forceinline__ void loader_init(Loader &L, int ld, int x0, int xlim, int klim, int wave, int lane,
                                            const RowMap &map = RowMap{nullptr, 0, 0, 0}) {
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
        const int chunk = wave * CPW + q;
        if (XC) {
            const int krow = chunk * 2 + (lane >> 5);
            const int g = (lane & 31) ^ ((krow & 3) << 2);
            const int gx = x0 + g * 8;
            L.off[q] = gx < xlim ? ((uint32_t)krow * ld + gx) * 2u : OOB;
            L.kthr[q] = klim - krow;
        } else {
            const int row = chunk * (1024 / KC_ROW) + lane / KC_G;
            const int g = (lane % KC_G) ^ ((row >> KC_SWZ_SHIFT) & (KC_G - 1));
            const int gx = x0 + row;
            if (map.mapped()) {
                const int src = gx < xlim ? map.row(gx) : -1;
                L.off[q] = src >= 0 ? ((uint32_t)src * ld + g * 8) * 2u : OOB;
            } else {
                L.off[q] = gx < xlim ? ((uint32_t)gx * ld + g * 8) * 2u : OOB;
            }
            L.kthr[q] = klim - g * 8;
        }
    }
}

// Byte offsets (inside an operand tile) from which lane `lane` reads its MFMA fragments.
//   KC: one offset per k-step, blocks of 32 rows add 32 * KC_ROW bytes.
//   XC: one offset per 32-column block, k-steps add 16*512 bytes, the second half 4*512.
template <bool XC, int NBLK>
struct FragAddr {
    int32_t a[XC ? NBLK : KS];
    __device__ __forceinline__ void init(int xbase, int lane) {
        if (XC) {
            const int s = (lane >> 2) & 3;
            const int kr = 8 * (lane >> 5) + ((lane & 15) >> 2);
            const int glow = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
            for (int b = 0; b < NBLK; ++b)
                a[b] = kr * 512 + (((((xbase + b * 32) >> 3) ^ (s << 2)) + glow) << 4) + (lane & 1) * 8;
        } else {
            // swizzle term of row = xbase + lane%32 (xbase is a multiple of 32, which the term ignores)
            const int s = ((lane & 31) >> KC_SWZ_SHIFT) & (KC_G - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                a[ks] = (xbase + (lane & 31)) * KC_ROW + (((ks * 2 + (lane >> 5)) ^ s) << 4);
        }
    }
    __device__ __forceinline__ bf16x8 read(const char *tile, int blk, int ks) const {
        if (XC) {
            const char *p = tile + a[blk] + ks * 16 * 512;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * 512));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, both);
        } else {
            return *(const bf16x8 *)(tile + a[ks] + blk * 32 * KC_ROW);
        }
    }
};

// Tile plan.  An expert's rows are cut into 32-row MFMA blocks, and its nb blocks into
// ceil(nb / maxb) m-tiles of nearly equal block counts (maxb = 9 for a KC A operand, else 8): an
// expert with a few rows more than a multiple of 256 gets "tall" tiles of 9 blocks instead of an
// extra tile that would stream a whole weight panel for a handful of rows.  An expert with at most
// LIGHT_BLOCKS blocks is one "light" tile per column of n-tiles.
// The heavy tiles form one list (expert -- in an order that alternates light and heavy experts --, then
// n-tile, then m-tile, so that the m-tiles of one weight panel are neighbours).  The list is cut into 8 contiguous shares of equal work (tile cost x
// k-tiles: experts differ in size), one per XCD, so that tiles which share a weight panel share an
// L2; each share is followed by an eighth of the light tiles.  kept[] lives on the device, so a
// small kernel writes the plan before every GEMM launch:
//   plan[0..7]   per-share fetch counters (zeroed here, advanced by the GEMM workgroups)
//   plan[8..16]  start of each share in the tile array (plan[16] = number of tiles)
//   plan[32 + 4 t ..]  tile t: {expert | blocks << 8 | light << 12, n-tile, first block, kept[expert]}
// The GEMM kernel is persistent: one workgroup per compute unit takes tiles from the share of its
// own XCD (workgroup ids go round-robin over the XCDs) until that share is empty.
constexpr int PLAN_HDR_INTS = 32;
constexpr int PLAN_THREADS = 1024;
constexpr int MAX_PLANS = 4;
constexpr int PLAN_SLICES = 8;                 // blocks per plan: each recomputes the header and fills a slice of the tiles

// Measured cost of a heavy tile by its block count, in half blocks of a full tile's main loop:
// up to 6 blocks run through the loop that skips blocks (slower per block), 7 and 8 through the
// full loop, 9 through the tall loop.
__device__ __forceinline__ int tile_cost(int nblk) { return nblk >= 9 ? 19 : (nblk >= 6 ? 16 : 13); }

struct PlanDesc {
    const int32_t *kept;
    int32_t *plan;
    int E, M, K, nt, rows_from_kept, maxb, cus_per_xcd;
};
struct PlanArgs {
    PlanDesc p[MAX_PLANS];
};

__global__ __launch_bounds__(PLAN_THREADS) void gemm_plan_kernel(PlanArgs args) {
    const PlanDesc &p = args.p[blockIdx.x];
    __shared__ int s_kept[256], s_nb[256], s_hv[256], s_nk[256], s_eid[256];   // by list position, not by expert
    __shared__ int s_preH[257], s_preL[257];      // tiles of the experts before e (heavy, light)
    __shared__ long long s_preW[257], s_w[256];   // work of the heavy tiles of the experts before e, and of expert e
    __shared__ long long s_w0[256];               // work by expert index, for the ordering
    __shared__ int s_ts[9], s_sl[9];              // split points of the heavy and of the light list
    const int tid = threadIdx.x, nt = p.nt;
    int kx = 0, nb = 0, nkf = 1;
    long long w = 0;
    if (tid < p.E) {
        kx = p.kept[tid];
        const int Mx = p.rows_from_kept ? kx : p.M;
        nb = (Mx + 31) >> 5;
        const int nk = p.rows_from_kept ? 1 : (kx + BK - 1) / BK;
        nkf = nk > 0 ? nk : 1;                    // never 0: every heavy tile must fall into some share
        if (nb > LIGHT_BLOCKS) {  // one column of the expert's tiles: bx tiles of bb + 1 blocks, the others of bb
            const int hv = (nb + p.maxb - 1) / p.maxb, bb = nb / hv, bx = nb - bb * hv;
            w = (long long)(bx * tile_cost(bb + 1) + (hv - bx) * tile_cost(bb)) * nkf * nt;
        }
        s_w0[tid] = w;
    }
    __syncthreads();
    if (tid < p.E) {
        // Order of the experts in the list: lightest, heaviest, second lightest, second heaviest, ...  A share
        // mostly holds whole experts (their tiles share weight panels), and with few experts per share the
        // shares of a plain 0, 1, 2, ... order differ by the spread of the experts' sizes; pairing the extremes
        // evens them out.  Any order gives the same results: tiles are independent.
        int r = 0;
        for (int e = 0; e < p.E; ++e) r += (s_w0[e] < w || (s_w0[e] == w && e < tid)) ? 1 : 0;
        const int pos = r < (p.E + 1) / 2 ? 2 * r : 2 * (p.E - 1 - r) + 1;
        s_eid[pos] = tid;
        s_kept[pos] = kx;
        s_nb[pos] = nb;
        s_hv[pos] = nb > LIGHT_BLOCKS ? (nb + p.maxb - 1) / p.maxb : 0;
        s_nk[pos] = nkf;
        s_w[pos] = w;
    }
    __syncthreads();
    if (tid < p.E) {              // exclusive prefix sums, every thread for itself (E <= 256: no dependent chain)
        int h = 0, l = 0;
        long long wp = 0;
        for (int e = 0; e < tid; ++e) {
            h += s_hv[e] * nt;
            l += (s_nb[e] > 0 && s_nb[e] <= LIGHT_BLOCKS) ? nt : 0;
            wp += s_w[e];
        }
        s_preH[tid] = h; s_preL[tid] = l; s_preW[tid] = wp;
        if (tid == p.E - 1) {
            s_preH[p.E] = h + s_hv[tid] * nt;
            s_preL[p.E] = l + ((s_nb[tid] > 0 && s_nb[tid] <= LIGHT_BLOCKS) ? nt : 0);
            s_preW[p.E] = wp + s_w[tid];
        }
    }
    __syncthreads();
    const int nH = s_preH[p.E], nL = s_preL[p.E];
    const long long WH = s_preW[p.E];
    if (tid <= 8) {
        // heavy tiles whose preceding work is below th = tid WH / 8
        const long long th = (tid * WH) >> 3;
        int res = 0;
        if (tid == 8) res = nH;
        else if (th > 0) {
            int e = 0;
            while (s_preW[e + 1] < th) ++e;       // s_preW[e] < th <= s_preW[e + 1], so expert e is heavy
            const int mts = s_hv[e], bb = s_nb[e] / mts, bx = s_nb[e] - bb * mts;
            const int c1 = tile_cost(bb + 1), c0t = tile_cost(bb);
            const long long wc = (long long)(bx * c1 + (mts - bx) * c0t) * s_nk[e];   // work of one column of its tiles
            const long long r = th - s_preW[e];                      // 1 .. wc nt
            const int c0 = (int)((r - 1) / wc);                       // whole columns of n-tiles before
            const int rem = (int)(((r - 1) - c0 * wc) / s_nk[e]);     // cost inside the column, 0 .. wc / nk - 1
            // tiles of the column whose preceding cost is at most rem
            int cm = rem < bx * c1 ? rem / c1 + 1 : bx + (rem - bx * c1) / c0t + 1;
            cm = cm < mts ? cm : mts;
            res = s_preH[e] + c0 * mts + cm;
        }
        // A share is worked off by the cus_per_xcd compute units of one XCD, a tile at a time: a few
        // tiles beyond a multiple of that number cost a whole extra round, so the split points are
        // moved to the nearest multiple (this matters when there are only a few rounds).  With no more
        // tiles than compute units there is one round if no share holds more tiles than its XCD has
        // units: the shares are then equal in tile count, which also uses the memory paths of all XCDs
        // instead of filling two or three of them.
        if (tid > 0 && tid < 8) {
            const int c = p.cus_per_xcd;
            if (nH <= 8 * c) {
                res = (tid * nH) >> 3;
            } else {
                res = (res + c / 2) / c * c;
                res = res < nH ? res : nH;
            }
        }
        s_ts[tid] = res;
        s_sl[tid] = (int)(((long long)tid * nL) >> 3);
    }
    __syncthreads();
    if (blockIdx.y == 0) {
        if (tid < 8) p.plan[tid] = 0;
        if (tid <= 8) p.plan[8 + tid] = s_ts[tid] + s_sl[tid];
    }
    int4 *tiles = (int4 *)(p.plan + PLAN_HDR_INTS);
    for (int t = blockIdx.y * PLAN_THREADS + tid; t < nH + nL; t += PLAN_THREADS * PLAN_SLICES) {
        const bool light = t >= nH;
        const int q = light ? t - nH : t;
        const int *pre = light ? s_preL : s_preH;
        int lo = 0, hi = p.E;                     // largest e with pre[e] <= q (experts without tiles are skipped)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= q) lo = mid; else hi = mid;
        }
        const int e = lo, r = q - pre[e];
        const int *split = light ? s_sl : s_ts;
        int x = 0;
        while (split[x + 1] <= q) ++x;
        int4 ent;
        int pos;
        if (light) {
            ent = make_int4(s_eid[e] | (s_nb[e] << 8) | (1 << 12), r, 0, s_kept[e]);
            pos = s_ts[x + 1] + s_sl[x] + (q - s_sl[x]);
        } else {
            const int mts = s_hv[e];
            // the first nb % mts tiles of a column hold one block more than the others
            const int bb = s_nb[e] / mts, bx = s_nb[e] - bb * mts;
            int nti = r / mts, mti = r - nti * mts;                        // m fastest
            if (bx == 0 && mts > 4) {
                // many equal m-tiles (the weight gradients): n fastest inside groups of 8 n-tiles, so that
                // the 32 tiles an XCD works on together are 4 m-tiles x 8 n-tiles (12 operand panels)
                // rather than 16 x 2 (18 panels)
                const int ng = r / (mts * 8), rr = r - ng * (mts * 8);
                const int gw = nt - ng * 8 < 8 ? nt - ng * 8 : 8;
                mti = rr / gw;
                nti = ng * 8 + (rr - mti * gw);
            }
            const int nblk = bb + (mti < bx ? 1 : 0), blk0 = mti * bb + (mti < bx ? mti : bx);
            ent = make_int4(s_eid[e] | (nblk << 8), nti, blk0, s_kept[e]);
            pos = s_ts[x] + s_sl[x] + (q - s_ts[x]);
        }
        tiles[pos] = ent;
    }
}

template <bool AXC, bool BXC, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmDesc d) {
    __shared__ __attribute__((aligned(1024))) char smem[SMEM_BYTES];
    __shared__ int s_next[8];                    // the tile fetched by thread 0: its plan entry, then its index
    __shared__ int s_ctok[A_ROWS];               // scattered result: target row of each tile row (-1: none) ...
    __shared__ float s_cscl[A_ROWS];             // ... and its scale
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(lds_void *)smem;
    const int tid0 = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
    const int wm = (wave >> 2) * 128, wn = (wave & 3) * 64;
    const int jx = wave >> 2;
    FragAddr<AXC, 4> fa;
    FragAddr<BXC, 2> fb;
    fa.init(wm, tid0 & 63);
    fb.init(wn, tid0 & 63);
    FragAddr<BXC, 1> fbx;                        // B fragment of the wave's block in a tall tile's ninth block row
    fbx.init(wn + jx * 32, tid0 & 63);
    int32_t *plan = (int32_t *)d.plan;
    const int4 *tiles = (const int4 *)(plan + PLAN_HDR_INTS);
    const int myx = blockIdx.x & 7;
    // Tile fetch (thread 0): the workgroup draws tiles from the share of its own XCD until the
    // share's counter passes its size.  (Taking tiles from other shares at the end was tried and
    // lost: such a tile finds nothing of its panels in the local L2 and runs at half speed.)
    int cur_first = 0, cur_cnt = 0;
    auto fetch_blocking = [&]() {
        const int t = atomicAdd(plan + myx, 1);
        return t < cur_cnt ? cur_first + t : -1;
    };
    auto publish = [&](int idx, const int4 &ent) {
        s_next[0] = ent.x; s_next[1] = ent.y; s_next[2] = ent.z; s_next[3] = ent.w; s_next[4] = idx;
    };
    // Fetches run two tiles ahead and only during epilogues: the number of the tile after next is
    // requested and the plan entry of the next tile is loaded while this tile's result is written,
    // so that no such request is outstanding during a main loop (whose explicit vmcnt waits count
    // only the loop's own loads).
    int idx_n = -1;                              // thread 0: the next tile
    if (tid0 == 0) {
        cur_first = plan[8 + myx];
        cur_cnt = plan[9 + myx] - cur_first;
        const int idx = fetch_blocking();
        publish(idx, idx >= 0 ? tiles[idx] : make_int4(0, 0, 0, 0));
        if (idx >= 0) idx_n = fetch_blocking();
    }
    __syncthreads();

  for (;;) {
    // The thread index is made opaque per tile: otherwise the compiler hoists the lane-dependent
    // address arithmetic of the loaders and of the epilogue out of this loop and keeps it in
    // registers through the main loop, which has none to spare.
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int tile_idx = __builtin_amdgcn_readfirstlane(s_next[4]);
    if (tile_idx < 0) break;
    const int ent0 = __builtin_amdgcn_readfirstlane(s_next[0]);
    const int e = ent0 & 255, nblk = (ent0 >> 8) & 15;
    const bool light = (ent0 >> 12) & 1;
    const int nti = __builtin_amdgcn_readfirstlane(s_next[1]);
    const int blk0 = __builtin_amdgcn_readfirstlane(s_next[2]);
    const int kept = __builtin_amdgcn_readfirstlane(s_next[3]);
    const bool tall = !AXC && nblk == MAXB;

    const int Me = d.rows_from_kept ? kept : d.M;
    const int Ke = d.rows_from_kept ? d.K : kept;
    const int m0 = blk0 * 32, n0 = nti * BN;
    const int mlim = Me < m0 + nblk * 32 ? Me : m0 + nblk * 32;     // rows [m0, mlim) are this tile's

    // gathered A (dispatch folded in, or the row shares of duplicate token dropping): one array for all
    // experts, rows through this expert's index slice or the share arithmetic
    RowMap amap = {nullptr, 0, 0, 0};
    if (!AXC && d.a_index != nullptr) amap.index = d.a_index + (int64_t)e * d.M;
    else if (!AXC && d.a_dtd_g > 1) { amap.G = d.a_dtd_g; amap.share_rows = d.E * d.a_dtd_cg; amap.base = e * d.a_dtd_cg; }
    const bool a_index = amap.mapped();
    const bf16_t *Ap = a_index ? (const bf16_t *)d.A : (const bf16_t *)d.A + (int64_t)e * d.strideA;
    const bf16_t *Bp = (const bf16_t *)d.B + (int64_t)e * d.strideB;
    // extent of this expert's operands in bytes (rows x row length)
    const uint32_t a_bytes = a_index ? (uint32_t)d.a_rows * (uint32_t)d.lda * 2u
                                     : (uint32_t)(AXC ? Ke : Me) * (uint32_t)d.lda * 2u;
    // scattered result (combine folded in): target row and scale of each of the tile's rows, through LDS
    const bool scatter = EPI == EPI_STORE && d.c_index != nullptr;
    if (scatter && tid < A_ROWS) {
        const int gm = m0 + tid;
        const bool ok = gm < mlim;
        s_ctok[tid] = ok ? d.c_index[(int64_t)e * d.M + gm] : -1;
        s_cscl[tid] = ok ? d.c_scale[(int64_t)e * d.M + gm] : 0.f;
    }
    const uint32_t b_bytes = (uint32_t)(BXC ? Ke : d.N) * (uint32_t)d.ldb * 2u;
    const i32x4 A = make_rsrc(Ap, a_bytes), B = make_rsrc(Bp, b_bytes);

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // Ninth block row of a tall tile (rows 256..287): its 8 blocks go one to each wave, wave (wm, wn)
    // taking the column block it already holds a B fragment for: 2 (wn / 64) + wm / 128.
    f32x16 accx;
#pragma unroll
    for (int v = 0; v < 16; ++v) accx[v] = 0.f;

    const int nk = (Ke + BK - 1) / BK;
    // Software pipeline.  A k-tile is 32 deep: 2 k-steps of 8 MFMAs per wave.  Tile kt lives in
    // stage kt % NSTAGE and is requested NSTAGE-1 iterations before it is consumed, so up to
    // (NSTAGE-1) x 32 KB are in flight per workgroup.  Each k-step has its own fragment registers
    // (a0/b0, a1/b1), all read in the memory phase that precedes the tile's 16 MFMAs.
    bf16x8 a0[4], b0[2], a1[4], b1[2], ax0, ax1, bx0, bx1;
    Loader la, lb;
    loader_init<AXC>(la, d.lda, m0, mlim, Ke, wave, lane, amap);
    loader_init<BXC>(lb, d.ldb, n0, d.N, Ke, wave, lane);
    // tall tile: the two 1 KB chunks of rows 256..287 are loaded by waves 0 and 5 (one wave of each
    // ping-pong group, on different SIMDs), which therefore have 5 loads per k-tile in flight
    const int xw = wave == 0 ? 0 : (wave == 5 ? 1 : -1);
    const bool has_x = !AXC && tall && xw >= 0;
    uint32_t offx = OOB;
    int32_t kthrx = 0;
    if (has_x) {
        const int row = 256 + 16 * xw + (lane >> 2);
        const int g = (lane & 3) ^ ((row >> KC_SWZ_SHIFT) & (KC_G - 1));
        const int gx = m0 + row;
        if (a_index) {
            const int src = gx < mlim ? amap.row(gx) : -1;
            offx = src >= 0 ? ((uint32_t)src * d.lda + g * 8) * 2u : OOB;
        } else {
            offx = gx < mlim ? ((uint32_t)gx * d.lda + g * 8) * 2u : OOB;
        }
        kthrx = Ke - g * 8;
    }
    // 32-row blocks of this wave that hold valid rows (4 except in a last, partial m-tile)
    const int rv = mlim - m0 - wm;
    const int nvi = __builtin_amdgcn_readfirstlane(rv >= 128 ? 4 : (rv <= 0 ? 0 : (rv + 31) >> 5));
    // Fragment reads and MFMAs of one k-step, in halves: half 0 covers a[0], a[1], b[0], b[1] and
    // block rows 0-1, half 1 a[2], a[3] and block rows 2-3.  In a partial m-tile (full = false)
    // blocks without valid rows are skipped.
    auto rd_half = [&](bf16x8(&af)[4], bf16x8(&bf)[2], int stage, int ks, int half, auto full) {
        const char *ta = smem + stage * STAGE_BYTES, *tb = ta + OPER_A_BYTES;
        if (half == 0 && (decltype(full)::value || nvi > 0)) {
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = fb.read(tb, j, ks);
        }
#pragma unroll
        for (int i = 2 * half; i < 2 * half + 2; ++i)
            if (decltype(full)::value || i < nvi) af[i] = fa.read(ta, i, ks);
    };
    auto mma_half = [&](const bf16x8(&af)[4], const bf16x8(&bf)[2], int half, auto full) {
#pragma unroll
        for (int i = 2 * half; i < 2 * half + 2; ++i)
            if (decltype(full)::value || i < nvi) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], af[i], acc[i][j], 0, 0, 0);
            }
    };
    // one of the 2*CPW one-KB chunk loads this wave contributes to a k-tile (CPW per operand)
    auto request_piece = [&](int kt, int stage, int piece) {
        const int k0 = kt * BK;
        const uint32_t base = smem_addr + stage * STAGE_BYTES;
        if (piece < CPW) {
            const uint32_t kadd = AXC ? (uint32_t)k0 * d.lda * 2u : (uint32_t)k0 * 2u;
            const uint32_t voff = k0 < la.kthr[piece] ? la.off[piece] + kadd : OOB;
            load_to_lds(A, base + (uint32_t)(wave * CPW + piece) * 1024u, voff);
        } else {
            const int q = piece - CPW;
            const uint32_t kadd = BXC ? (uint32_t)k0 * d.ldb * 2u : (uint32_t)k0 * 2u;
            const uint32_t voff = k0 < lb.kthr[q] ? lb.off[q] + kadd : OOB;
            load_to_lds(B, base + OPER_A_BYTES + (uint32_t)(wave * CPW + q) * 1024u, voff);
        }
    };
    auto request_extra = [&](int kt, int stage) {     // tall tiles, waves 0 and 5 only
        static_assert(BK == 32, "16 rows of 64 bytes per chunk");
        const int k0 = kt * BK;
        const uint32_t voff = k0 < kthrx ? offx + (uint32_t)k0 * 2u : OOB;
        load_to_lds(A, smem_addr + stage * STAGE_BYTES + (uint32_t)(256 + 16 * xw) * KC_ROW, voff);
    };
    auto rd_extra = [&](int stage) {
        const char *ta = smem + stage * STAGE_BYTES, *tb = ta + OPER_A_BYTES;
        ax0 = fa.read(ta, 8 - (wm >> 5), 0);
        ax1 = fa.read(ta, 8 - (wm >> 5), 1);
        bx0 = fbx.read(tb, 0, 0);                 // read again rather than picked from b0 / b1: no VALU work
        bx1 = fbx.read(tb, 0, 1);                 // between the MFMAs
    };
    auto mma_extra = [&](const bf16x8 &bx, const bf16x8 &ax) {
        accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx, ax, accx, 0, 0, 0);
    };
    auto mma = [&](const bf16x8(&af)[4], const bf16x8(&bf)[2], auto full) {
        mma_half(af, bf, 0, full);
        mma_half(af, bf, 1, full);
    };
    auto request = [&](int kt, int stage) {
#pragma unroll
        for (int piece = 0; piece < 2 * CPW; ++piece) request_piece(kt, stage, piece);
    };
#pragma unroll
    for (int i = 0; i < 4; ++i) a1[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 2; ++j) b1[j] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    // Main loop, "ping-pong" form.  Waves w and w+4 share a SIMD.  Each wave alternates a memory
    // phase M (request tile kt+3, read all fragments of tile kt from LDS) and a compute phase C
    // (16 MFMAs), every phase ending in a workgroup barrier; waves 4-7 run half an iteration behind
    // waves 0-3 (one extra barrier up front, matched by one extra barrier of waves 0-3 at the end),
    // so on every SIMD one wave feeds the matrix pipe while the other waits on the LDS.
    //  - tile j is complete before any wave reads it: every wave waits for its own loads of tile
    //    kt+1 (at most the two newer tiles outstanding: 8 loads, or 10 in the two waves that load
    //    the ninth block of a tall tile) before each barrier;
    //  - the stage of tile kt-1 is overwritten by requests issued in M(kt), which every wave starts
    //    only after a barrier that follows the last fragment read of tile kt-1 (lgkmcnt(0) before
    //    the barrier that ends each M).
    static_assert(BK == 32 && NSTAGE == 4, "the ping-pong loop is written for 32-deep tiles and 4 stages");
    const bool late_group = wave >= 4;
    auto main_loop = [&](auto full, auto tallc) {
        constexpr bool TALLV = !AXC && decltype(tallc)::value;
        const bool five = TALLV && has_x;   // this wave has 5 loads per k-tile in flight
        // A wave waits until only the loads of the two newest k-tiles are outstanding.  The two waves
        // that load the ninth block issue that fifth load in the MFMA phase (the memory phase is the
        // longer one), so at the end of a memory phase it has not been issued yet for the newest tile.
        auto wait_end_of_M = [&]() {                     // and lgkmcnt(0)
            if (five) __builtin_amdgcn_s_waitcnt(0x0070 | 9);
            else __builtin_amdgcn_s_waitcnt(0x0070 | 8);
        };
        auto wait_end_of_C = [&]() {
            if (five) __builtin_amdgcn_s_waitcnt(0x0F70 | 10);
            else __builtin_amdgcn_s_waitcnt(0x0F70 | 8);
        };
        if (nk > 0) {
#pragma unroll
            for (int t = 0; t < NSTAGE - 1; ++t) {
                request(t, t);
                if (five) request_extra(t, t);
            }
            wait_end_of_C();                             // tile 0 has landed
            __builtin_amdgcn_s_barrier();
            if (late_group) __builtin_amdgcn_s_barrier();
        }
        int stage = 0;                                   // kt % NSTAGE
        for (int kt = 0; kt < nk; ++kt) {
            const int prev = stage == 0 ? NSTAGE - 1 : stage - 1;
            // ---- M: memory phase
            request(kt + NSTAGE - 1, prev);
            rd_half(a0, b0, stage, 0, 0, full);
            rd_half(a0, b0, stage, 0, 1, full);
            rd_half(a1, b1, stage, 1, 0, full);
            rd_half(a1, b1, stage, 1, 1, full);
            if (TALLV) rd_extra(stage);
            __builtin_amdgcn_sched_barrier(0);
            wait_end_of_M();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // ---- C: compute phase
            __builtin_amdgcn_s_setprio(1);
            mma(a0, b0, full);
            if (five) request_extra(kt + NSTAGE - 1, prev);
            if (TALLV) mma_extra(bx0, ax0);
            mma(a1, b1, full);
            if (TALLV) mma_extra(bx1, ax1);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
            wait_end_of_C();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            stage = stage == NSTAGE - 1 ? 0 : stage + 1;
        }
        if (nk > 0 && !late_group) __builtin_amdgcn_s_barrier();
    };
    if (tall)
        main_loop(std::true_type{}, std::true_type{});
    else if (nblk >= 7)        // 7 blocks: one zero block costs less than the per-block branches of the partial loop
        main_loop(std::true_type{}, std::false_type{});
    else
        main_loop(std::false_type{}, std::false_type{});
    __builtin_amdgcn_s_waitcnt(0x0070);              // nothing may still be writing LDS when it is reused
    __syncthreads();
    int4 ent_next = make_int4(0, 0, 0, 0);
    int t_after = 0;
    if (tid == 0) {                                  // both arrive during the epilogue
        if (idx_n >= 0) {
            ent_next = tiles[idx_n];
            t_after = atomicAdd(plan + myx, 1);
        }
    }

    // Epilogue.  The MFMAs were issued with the operands swapped (B fragment first), so the
    // accumulators hold the transposed block: lane owns output row m = lane%32 and, per group of
    // four registers, four consecutive columns n = (v/4)*8 + (lane/32)*4 + v%4.  The tile is
    // converted to bf16, staged in LDS (the operand stages are free now; reads still in flight
    // from the loop's last prefetch are never used) and written out as full 512-byte rows.
    bf16_t *C = (bf16_t *)d.C + (int64_t)e * d.strideC;
    bf16_t *st = (bf16_t *)smem;
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
        if (tall) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                bf16_t *pos = st + (256 + (lane & 31)) * CLD + wn + jx * 32 + vq * 8 + (lane >> 5) * 4;
                f32x4 v = {accx[vq * 4], accx[vq * 4 + 1], accx[vq * 4 + 2], accx[vq * 4 + 3]};
                fn(pos, v);
            }
        }
    };
    auto put4 = [](bf16_t *pos, const f32x4 &v) {
        bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
        *(bf16x4 *)pos = o;
    };
    auto flush = [&](bf16_t *out) {
        __syncthreads();
        auto pass = [&](int p) {
            const int row = (tid >> 5) + 16 * p, gm = m0 + row, gn = n0 + (tid & 31) * 8;
            const u32x4 v = *(const u32x4 *)(st + row * CLD + (tid & 31) * 8);
            if (gm < mlim && gn < d.N) *(u32x4 *)(out + (int64_t)gm * d.ldc + gn) = v;
        };
#pragma unroll
        for (int p = 0; p < 16; ++p) pass(p);
        if (tall) { pass(16); pass(17); }
    };
    if (EPI == EPI_STORE) {
        for_each_quad([&](bf16_t *pos, const f32x4 &v) { put4(pos, v); });
        if (!scatter) {
            flush(C);
        } else {
            // result row (if C is given) and the scaled row at its target: the staged bf16 value times the
            // scale, rounded again -- exactly what a separate combine pass over C would produce
            bf16_t *S = (bf16_t *)d.C_scatter;
            const bool keep = d.C != nullptr;
            __syncthreads();
            auto spass = [&](int p) {
                const int row = (tid >> 5) + 16 * p, gm = m0 + row, gn = n0 + (tid & 31) * 8;
                const u32x4 v = *(const u32x4 *)(st + row * CLD + (tid & 31) * 8);
                const int trg = s_ctok[row];
                const float scl = s_cscl[row];
                if (gm < mlim && gn < d.N) {
                    if (keep) *(u32x4 *)(C + (int64_t)gm * d.ldc + gn) = v;
                    if (trg >= 0) {
                        const bf16x8 b = __builtin_bit_cast(bf16x8, v);
                        bf16x8 o;
#pragma unroll
                        for (int q = 0; q < 8; ++q) o[q] = (bf16_t)((float)b[q] * scl);
                        *(u32x4 *)(S + (int64_t)trg * d.ldc + gn) = __builtin_bit_cast(u32x4, o);
                    }
                }
            };
#pragma unroll
            for (int p = 0; p < 16; ++p) spass(p);
            if (tall) { spass(16); spass(17); }
        }
    } else if (EPI == EPI_GELU) {
        // The activation is a compile-time constant inside (one branch per tile, not per element).
        auto gelu_stage = [&](auto actc) __attribute__((always_inline)) {
            constexpr int ACT = decltype(actc)::value;
            if (d.C2) {
                // Second output act'(z), which is all the backward pass needs of z.  Both values are
                // computed in one go and staged side by side, so the tile goes out in three parts of
                // at most 128 rows (two staging areas of 128 rows fit the LDS): the wave's block rows
                // 0-1, its block rows 2-3, and the ninth block row of a tall tile.
                bf16_t *stG = st, *stH = st + 128 * CLD;
                bf16_t *outG = (bf16_t *)d.C2 + (int64_t)e * d.strideC;
                auto both16 = [&](const f32x16 &a, int srow, int col) __attribute__((always_inline)) {
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        f32x4 g, hv;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float h1, g1;
                            gelu_both_fast(a[vq * 4 + q], ACT, h1, g1);
                            hv[q] = h1;
                            g[q] = g1;
                        }
                        const int off = srow * CLD + col + vq * 8 + (lane >> 5) * 4;
                        put4(stG + off, g);
                        put4(stH + off, hv);
                    }
                };
                // staged row sr of part `part` is tile row trow(sr)
                auto flush_part = [&](int part, int nrows) __attribute__((always_inline)) {
                    __syncthreads();
                    for (int p = 0; p < nrows / 16; ++p) {
                        const int sr = (tid >> 5) + 16 * p;
                        const int trow = part == 2 ? 256 + sr : (sr >> 6) * 128 + part * 64 + (sr & 63);
                        const int gm = m0 + trow, gn = n0 + (tid & 31) * 8;
                        const u32x4 vg = *(const u32x4 *)(stG + sr * CLD + (tid & 31) * 8);
                        const u32x4 vh = *(const u32x4 *)(stH + sr * CLD + (tid & 31) * 8);
                        if (gm < mlim && gn < d.N) {
                            *(u32x4 *)(outG + (int64_t)gm * d.ldc + gn) = vg;
                            *(u32x4 *)(C + (int64_t)gm * d.ldc + gn) = vh;
                        }
                    }
                    __syncthreads();
                };
#pragma unroll
                for (int part = 0; part < 2; ++part) {
#pragma unroll
                    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            both16(acc[2 * part + ii][j], (wm >> 7) * 64 + ii * 32 + (lane & 31), wn + j * 32);
                    flush_part(part, 128);
                }
                if (tall) {
                    both16(accx, lane & 31, wn + jx * 32);
                    flush_part(2, 32);
                }
            } else {
                for_each_quad([&](bf16_t *pos, const f32x4 &v) {
                    f32x4 g = {gelu_fast(v[0], ACT), gelu_fast(v[1], ACT), gelu_fast(v[2], ACT), gelu_fast(v[3], ACT)};
                    put4(pos, g);
                });
            }
        };
        if (act == MOE_GELU_TANH) gelu_stage(std::integral_constant<int, MOE_GELU_TANH>{});
        else gelu_stage(std::integral_constant<int, MOE_GELU_ERF>{});
        if (!d.C2) flush(C);
    } else {
        const bf16_t *Zin = (const bf16_t *)d.Zin + (int64_t)e * d.strideC;
        auto zpass = [&](int p) {
            const int row = (tid >> 5) + 16 * p, gm = m0 + row, gn = n0 + (tid & 31) * 8;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (gm < mlim && gn < d.N) v = *(const u32x4 *)(Zin + (int64_t)gm * d.ldc + gn);
            *(u32x4 *)(st + row * CLD + (tid & 31) * 8) = v;
        };
#pragma unroll
        for (int p = 0; p < 16; ++p) zpass(p);
        if (tall) { zpass(16); zpass(17); }
        __syncthreads();
        for_each_quad([&](bf16_t *pos, const f32x4 &v) {     // Zin holds act'(z)
            const bf16x4 z = *(const bf16x4 *)pos;
            f32x4 g = {v[0] * (float)z[0], v[1] * (float)z[1], v[2] * (float)z[2], v[3] * (float)z[3]};
            put4(pos, g);
        });
        flush(C);
    }
    // the staging tile is reused by the next tile; s_next was last read before the main loop
    if (tid == 0) {
        publish(idx_n, ent_next);
        idx_n = (idx_n >= 0 && t_after < cur_cnt) ? cur_first + t_after : -1;
    }
    __syncthreads();
  }
}

static int num_compute_units() {
    static int cus = 0;                          // same value from every thread that races here
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            n <= 0)
            n = 256;
        cus = n;
    }
    return cus;
}

size_t gemm_bf16_plan_bytes(const GemmDesc &d) {
    const int64_t mt = (d.M + BM - 1) / BM, nt = (d.N + BN - 1) / BN;
    return (size_t)(PLAN_HDR_INTS * 4 + 16 * (int64_t)d.E * mt * nt + 255) / 256 * 256;
}

moe_status_t launch_gemm_bf16_plans(const GemmDesc *descs, int n, hipStream_t s) {
    if (n < 1 || n > MAX_PLANS) {
        set_error("gemm_bf16: %d plans in one launch", n);
        return MOE_ERR_INVALID_ARG;
    }
    PlanArgs args = {};
    for (int i = 0; i < n; ++i) {
        const GemmDesc &d = descs[i];
        if (d.plan == nullptr || d.E > 256) {
            set_error("gemm_bf16: no plan buffer, or more than 256 experts");
            return MOE_ERR_INVALID_ARG;
        }
        PlanDesc &p = args.p[i];
        p.kept = d.kept; p.plan = (int32_t *)d.plan;
        p.E = d.E; p.M = d.M; p.K = d.K; p.nt = (d.N + BN - 1) / BN;
        p.rows_from_kept = d.rows_from_kept; p.maxb = d.a_xc ? 8 : MAXB;
        p.cus_per_xcd = num_compute_units() / 8 > 0 ? num_compute_units() / 8 : 1;
    }
    hipLaunchKernelGGL(gemm_plan_kernel, dim3(n, PLAN_SLICES), dim3(PLAN_THREADS), 0, s, args);
    return check_launch("gemm_plan");
}

template <bool AXC, bool BXC>
static void launch_epi(const GemmDesc &d, hipStream_t s) {
    // persistent: one workgroup per compute unit (the LDS footprint allows no second one)
    dim3 grid((unsigned)num_compute_units()), block(GEMM_THREADS);
    switch (d.epi) {
        case EPI_STORE:
            hipLaunchKernelGGL((gemm_bf16_kernel<AXC, BXC, EPI_STORE>), grid, block, 0, s, d);
            break;
        case EPI_GELU:
            hipLaunchKernelGGL((gemm_bf16_kernel<AXC, BXC, EPI_GELU>), grid, block, 0, s, d);
            break;
        default:
            hipLaunchKernelGGL((gemm_bf16_kernel<AXC, BXC, EPI_DGELU>), grid, block, 0, s, d);
            break;
    }
}

// The plan in d.plan must have been written (launch_gemm_bf16_plans) earlier on the same stream,
// for this descriptor's kept, E, M, N, K, rows_from_kept and A layout; a plan serves one launch.
moe_status_t launch_gemm_bf16(const GemmDesc &d, hipStream_t s) {
    if (d.plan == nullptr) {
        set_error("gemm_bf16: no plan");
        return MOE_ERR_INVALID_ARG;
    }
    if (!d.a_xc && d.b_xc)
        launch_epi<false, true>(d, s);      // forward: A [M,K], B [K,N]
    else if (!d.a_xc && !d.b_xc)
        launch_epi<false, false>(d, s);     // data gradient: A [M,K], B [N,K]
    else if (d.a_xc && d.b_xc)
        launch_epi<true, true>(d, s);       // weight gradient: A [K,M], B [K,N]
    else {
        set_error("gemm_bf16: operand layout combination not built");
        return MOE_ERR_UNSUPPORTED;
    }
    return check_launch("gemm_bf16");
}

}  // namespace moe
