// extern "C" entry points: host-side validation, workspace layout, launches.  See include/moe.h
// for the contract of every call.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include "moe_common.h"

namespace moe {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

moe_status_t check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: HIP error %d (%s)", what, (int)e, hipGetErrorString(e));
        return MOE_ERR_HIP;
    }
    return MOE_OK;
}

size_t gate_ws_bytes(const moe_shape_t *sh);
size_t gate_bwd_ws_bytes(const moe_shape_t *sh);
moe_status_t run_gate(const moe_shape_t *, const void *, const float *, const float *, float *, float *, int32_t *,
                      float *, int32_t *, int32_t *, int32_t *, int32_t *, void *, hipStream_t);
moe_status_t run_dispatch(const moe_shape_t *, const void *, const int32_t *, void *, hipStream_t);
moe_status_t run_dispatch_bwd(const moe_shape_t *, const void *, const int32_t *, const int32_t *, void *,
                              hipStream_t, int tp_size = 1);
moe_status_t run_dispatch_dtd(const moe_shape_t *, const void *, const int32_t *, int, int, void *, hipStream_t);
moe_status_t run_dtd_drop(const moe_shape_t *, const void *, const int32_t *, int, int, void *, hipStream_t);
moe_status_t run_dtd_gather(const moe_shape_t *, const void *, const int32_t *, int, void *, hipStream_t);
moe_status_t run_combine(const moe_shape_t *, const void *, const int32_t *, const int32_t *, const float *, void *,
                         hipStream_t);
moe_status_t run_combine_prep(const moe_shape_t *, const int32_t *, const int32_t *, const float *, float *, void *,
                              hipStream_t);
moe_status_t run_combine_bwd(const moe_shape_t *, const void *, const void *, const int32_t *, const int32_t *,
                             const float *, void *, float *, hipStream_t);
moe_status_t run_gate_bwd(const moe_shape_t *, const float *, const float *, const int32_t *, const void *,
                          const float *, float *, float *, void *, void *, hipStream_t);
moe_status_t run_dispatch_bwd_fused(const moe_shape_t *, const void *, const int32_t *, const int32_t *, void *,
                                    const float *, const float *, hipStream_t, int tp_size = 1);
struct AdamwConst {
    float lr, beta1, beta2, omb1, omb2, eps, wd, inv_bc1, inv_bc2, grad_mult;
};
moe_status_t run_adamw_tiled(int64_t, int64_t, const AdamwConst &, const void *, float *, float *, float *, void *,
                             float *, int, hipStream_t);
moe_status_t run_gate_dx_f32(const moe_shape_t *, const float *, const float *, void *, hipStream_t);

static size_t esize(const moe_shape_t *sh) { return sh->dtype == MOE_BF16 ? 2 : 4; }

static moe_status_t check_shape(const moe_shape_t *sh) {
    if (!sh) {
        set_error("shape is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (sh->T <= 0 || sh->h <= 0 || sh->E <= 0 || sh->f <= 0 || sh->C <= 0) {
        set_error("non-positive size: T=%lld h=%d E=%d f=%d C=%lld", (long long)sh->T, sh->h, sh->E, sh->f,
                  (long long)sh->C);
        return MOE_ERR_INVALID_ARG;
    }
    if (sh->dtype != MOE_F32 && sh->dtype != MOE_BF16) {
        set_error("unknown dtype %d", sh->dtype);
        return MOE_ERR_UNSUPPORTED;
    }
    if (sh->act != MOE_GELU_ERF && sh->act != MOE_GELU_TANH) {
        set_error("unknown activation %d", sh->act);
        return MOE_ERR_UNSUPPORTED;
    }
    if (sh->E > 256) {
        set_error("E=%d exceeds the supported maximum of 256", sh->E);
        return MOE_ERR_UNSUPPORTED;
    }
    const int mult = sh->dtype == MOE_BF16 ? 8 : 4;
    if (sh->h % mult || sh->f % mult) {
        set_error("h=%d and f=%d must be multiples of %d for this dtype", sh->h, sh->f, mult);
        return MOE_ERR_UNSUPPORTED;
    }
    const int64_t w = sh->h > sh->f ? sh->h : sh->f;
    // (T*h*esize < 2^37: the gate backward walks x in at most 64 chunks, each through a 2 GiB buffer window;
    // h, f <= 2^20: the gate's three bf16 planes of up to 256 expert rows stay inside such a window as well)
    if (sh->T > (int64_t)0x7fffffff || sh->C > (int64_t)0x7fffffff || w > (1 << 20) ||
        (double)sh->T * (double)sh->h * (double)esize(sh) >= 137438953472.0 ||
        (double)sh->E * (double)sh->C * (double)w >= 1099511627776.0 ||
        (double)sh->C * (double)w * (double)esize(sh) >= 2147483648.0 ||
        (double)sh->h * (double)sh->f * (double)esize(sh) >= 2147483648.0) {
        set_error("shape too large: T=%lld C=%lld E=%d h=%d f=%d", (long long)sh->T, (long long)sh->C, sh->E, sh->h,
                  sh->f);
        return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

static bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

#define REQUIRE_PTR(p)                                                  \
    do {                                                                \
        if ((p) == nullptr) {                                           \
            set_error("%s: argument '%s' is NULL", __func__, #p);       \
            return MOE_ERR_INVALID_ARG;                                 \
        }                                                               \
        if (misaligned(p)) {                                            \
            set_error("%s: argument '%s' is not 16-byte aligned", __func__, #p); \
            return MOE_ERR_INVALID_ARG;                                 \
        }                                                               \
    } while (0)
#define OPTIONAL_PTR(p)                                                 \
    do {                                                                \
        if ((p) != nullptr && misaligned(p)) {                          \
            set_error("%s: argument '%s' is not 16-byte aligned", __func__, #p); \
            return MOE_ERR_INVALID_ARG;                                 \
        }                                                               \
    } while (0)

static size_t round256(size_t v) { return (v + 255) / 256 * 256; }
static size_t dz_bytes(const moe_shape_t *sh) { return round256((size_t)sh->E * sh->C * sh->f * esize(sh)); }

// The six grouped GEMMs of the expert FFN (bf16 path: each needs a tile plan in the workspace).
enum { G_FWD1, G_FWD2, G_DH, G_DW2, G_DW1, G_DD };
static GemmDesc ffn_gemm(const moe_shape_t &s, int which) {
    GemmDesc g = {};
    g.E = s.E; g.act = s.act; g.epi = EPI_STORE;
    const int32_t C = (int32_t)s.C;
    switch (which) {
        case G_FWD1:   // z = buf w1, hact = act(z)        A = buf [M,h], B = w1 [h,f] = [K,N]
            g.strideA = s.C * s.h; g.strideB = (int64_t)s.h * s.f; g.strideC = s.C * s.f;
            g.M = C; g.N = s.f; g.K = s.h; g.lda = s.h; g.ldb = s.f; g.ldc = s.f;
            g.a_xc = 0; g.b_xc = 1; g.rows_from_kept = 1; g.epi = EPI_GELU;
            break;
        case G_FWD2:   // y = hact w2                      A = hact [M,f], B = w2 [f,h] = [K,N]
            g.strideA = s.C * s.f; g.strideB = (int64_t)s.f * s.h; g.strideC = s.C * s.h;
            g.M = C; g.N = s.h; g.K = s.f; g.lda = s.f; g.ldb = s.h; g.ldc = s.h;
            g.a_xc = 0; g.b_xc = 1; g.rows_from_kept = 1;
            break;
        case G_DH:     // d_z = (d_y w2^T) * act'(z)       A = d_y [M,h], B = w2 [f,h] = [N,K]
            g.strideA = s.C * s.h; g.strideB = (int64_t)s.f * s.h; g.strideC = s.C * s.f;
            g.M = C; g.N = s.f; g.K = s.h; g.lda = s.h; g.ldb = s.h; g.ldc = s.f;
            g.a_xc = 0; g.b_xc = 0; g.rows_from_kept = 1; g.epi = EPI_DGELU;
            break;
        case G_DW2:    // d_w2 = hact^T d_y                A = hact [K=rows, M=f], B = d_y [K=rows, N=h]
            g.strideA = s.C * s.f; g.strideB = s.C * s.h; g.strideC = (int64_t)s.f * s.h;
            g.M = s.f; g.N = s.h; g.K = C; g.lda = s.f; g.ldb = s.h; g.ldc = s.h;
            g.a_xc = 1; g.b_xc = 1; g.rows_from_kept = 0;
            break;
        case G_DW1:    // d_w1 = buf^T d_z                 A = buf [K=rows, M=h], B = d_z [K=rows, N=f]
            g.strideA = s.C * s.h; g.strideB = s.C * s.f; g.strideC = (int64_t)s.h * s.f;
            g.M = s.h; g.N = s.f; g.K = C; g.lda = s.h; g.ldb = s.f; g.ldc = s.f;
            g.a_xc = 1; g.b_xc = 1; g.rows_from_kept = 0;
            break;
        default:       // d_buf = d_z w1^T                 A = d_z [M,f], B = w1 [h,f] = [N,K]
            g.strideA = s.C * s.f; g.strideB = (int64_t)s.h * s.f; g.strideC = s.C * s.h;
            g.M = C; g.N = s.h; g.K = s.f; g.lda = s.f; g.ldb = s.f; g.ldc = s.h;
            g.a_xc = 0; g.b_xc = 0; g.rows_from_kept = 1;
            break;
    }
    return g;
}
static size_t ffn_plan_bytes(const moe_shape_t *sh, int first, int last) {
    if (sh->dtype != MOE_BF16) return 0;
    size_t n = 0;
    for (int w = first; w <= last; ++w) n += gemm_bf16_plan_bytes(ffn_gemm(*sh, w));
    return n;
}
// Workspace layouts of the FFN entry points ([E,C,f] arrays first, each rounded to 256 bytes, plans last):
//   forward:   [hact if the caller keeps none][plans of GEMM1, GEMM2]
//   backward:  [d_z][hact, GeLU'(z) if recomputed][plan of GEMM1 if recomputed][plans of the four backward GEMMs]
static size_t slot_scale_bytes(const moe_shape_t *sh) { return round256((size_t)sh->E * sh->C * 4); }
//   fused forward (dispatch and combine folded in):  [hact if the caller keeps none][scale of every slot][plans]
static size_t ffn_fwd_ws_bytes(const moe_shape_t *sh, bool own_hact, bool fused = false) {
    return (own_hact ? dz_bytes(sh) : 0) + (fused ? slot_scale_bytes(sh) : 0) + ffn_plan_bytes(sh, G_FWD1, G_FWD2);
}
static size_t ffn_bwd_ws_bytes(const moe_shape_t *sh, bool recompute) {
    return dz_bytes(sh) * (recompute ? 3 : 1) + (recompute ? ffn_plan_bytes(sh, G_FWD1, G_FWD1) : 0) +
           ffn_plan_bytes(sh, G_DH, G_DD);
}

static size_t ws_bytes_checked(const moe_shape_t *sh, int for_backward) {
    const bool recompute = for_backward == 2;
    size_t need = gate_ws_bytes(sh);
    if (ffn_fwd_ws_bytes(sh, recompute, true) > need) need = ffn_fwd_ws_bytes(sh, recompute, true);
    if (!for_backward) return need;
    if (ffn_bwd_ws_bytes(sh, recompute) > need) need = ffn_bwd_ws_bytes(sh, recompute);
    if (round256(gate_bwd_ws_bytes(sh)) > need) need = round256(gate_bwd_ws_bytes(sh));
    return need;
}

// Side stream of the FFN backward (bf16): the two weight-gradient GEMMs do not depend on the data-gradient
// GEMM that runs next to them, and every GEMM launch ends with compute units idling while the last tiles
// finish; on a second stream the other GEMM's workgroups move into those units as they free up.  The side
// stream starts behind an event of the caller's stream and the caller's stream waits for its last event,
// so for the caller the call is still ordered on `stream` alone.
struct SideStream {
    hipStream_t caller = nullptr, stream = nullptr;
    hipEvent_t fork = nullptr, mid = nullptr, join = nullptr;
    bool ok = false;
};
// One side stream (with its three events) per caller stream and device, created on first use and kept until the
// process ends: layers that run on different streams do not share one, so their weight gradients are not
// serialised against each other.  At most SIDE_SLOTS caller streams per device get one; a call on any further
// stream, and every call when MOE_TED_SERIAL=1, keeps all its GEMMs on the caller's stream.
constexpr int SIDE_SLOTS = 8;
static SideStream *side_stream(hipStream_t caller) {
    static SideStream slots[16][SIDE_SLOTS];
    static int used[16] = {};
    static std::mutex mu;
    static const bool serial = [] {
        const char *e = getenv("MOE_TED_SERIAL");
        return e != nullptr && e[0] == '1';
    }();
    if (serial) return nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used[dev]; ++i)
        if (slots[dev][i].caller == caller) return slots[dev][i].ok ? &slots[dev][i] : nullptr;
    if (used[dev] == SIDE_SLOTS) return nullptr;
    SideStream &ss = slots[dev][used[dev]++];
    ss.caller = caller;
    ss.ok = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ss.mid, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess;
    if (!ss.ok) (void)hipGetLastError();
    return ss.ok ? &ss : nullptr;
}

// Scratch of the entry point that allocates nothing (moe_expert_ffn_fwd_static): the tile plans of its two
// GEMMs (fetch counters, share boundaries, tile queue) live in this array instead of a caller workspace.
// Every GPU the library runs on holds its own copy at its own address until the process ends; in host
// code the array's name is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t STATIC_SCRATCH_BYTES = MOE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// Device address of this GPU's copy of `scratch`, resolved once per device with that device current.
static moe_status_t static_scratch(void **out) {
    static void *per_device[64] = {};
    static std::mutex mu;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64) {
        set_error("moe_expert_ffn_fwd_static: no current device (%s)", hipGetErrorString(e));
        return MOE_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (per_device[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            set_error("moe_expert_ffn_fwd_static: hipGetSymbolAddress(scratch) failed on device %d: %s", dev,
                      hipGetErrorString(e));
            (void)hipGetLastError();
            return MOE_ERR_HIP;
        }
        per_device[dev] = ptr;
    }
    *out = per_device[dev];
    return MOE_OK;
}

static moe_status_t check_ws(const char *fn, const void *ws, size_t have, size_t need) {
    if (need == 0) return MOE_OK;
    if (ws == nullptr || misaligned(ws)) {
        set_error("%s: workspace is NULL or misaligned", fn);
        return MOE_ERR_INVALID_ARG;
    }
    if (have < need) {
        set_error("%s: workspace too small: %zu bytes given, %zu needed", fn, have, need);
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    return MOE_OK;
}

// The two forward GEMMs (arguments already validated; hact is a real array; `plans` holds
// ffn_plan_bytes(G_FWD1..G_FWD2) bytes on the bf16 path and is unused on the fp32 path).
// tp_size > 1: `buf` holds the tp_size row shares of duplicate token dropping, [G, E, ceil(C/G), h] (bf16 only).
static moe_status_t ffn_fwd_launch(const moe_shape_t &s, const void *buf, const void *w1, const void *w2,
                                   const int32_t *kept, void *z_save, void *hact, void *y, char *plans,
                                   hipStream_t hs, int tp_size = 1) {
    const bool bf = s.dtype == MOE_BF16;
    moe_status_t st;
    GemmDesc g[2] = {ffn_gemm(s, G_FWD1), ffn_gemm(s, G_FWD2)};
    g[0].A = buf; g[0].B = w1; g[0].C = hact; g[0].C2 = z_save; g[0].kept = kept;
    if (tp_size > 1) {
        g[0].a_dtd_g = tp_size;
        g[0].a_dtd_cg = (int32_t)((s.C + tp_size - 1) / tp_size);
        g[0].a_rows = (int64_t)tp_size * s.E * g[0].a_dtd_cg;
    }
    g[1].A = hact; g[1].B = w2; g[1].C = y; g[1].kept = kept;
    if (bf) {
        char *pl = plans;
        for (int i = 0; i < 2; ++i) { g[i].plan = pl; pl += gemm_bf16_plan_bytes(g[i]); }
        if ((st = launch_gemm_bf16_plans(g, 2, hs)) != MOE_OK) return st;
    }
    for (int i = 0; i < 2; ++i)
        if ((st = bf ? launch_gemm_bf16(g[i], hs) : launch_gemm_f32(g[i], hs)) != MOE_OK) return st;
    return MOE_OK;
}

// Launch-latency floor: a kernel of one wave that does nothing.
__global__ void empty_kernel() {}

}  // namespace moe

using namespace moe;

extern "C" {

int moe_version(void) { return 1; }

int64_t moe_capacity(int64_t T, int32_t E, double capacity_factor) {
    if (T <= 0 || E <= 0 || !(capacity_factor > 0.0)) return 0;
    return (int64_t)std::ceil(capacity_factor * (double)T / (double)E);
}

size_t moe_workspace_bytes(const moe_shape_t *shape, int for_backward) {
    if (check_shape(shape) != MOE_OK || for_backward < 0 || for_backward > 2) return 0;
    return ws_bytes_checked(shape, for_backward);
}

const char *moe_status_string(moe_status_t s) {
    switch (s) {
        case MOE_OK: return "MOE_OK";
        case MOE_ERR_INVALID_ARG: return "MOE_ERR_INVALID_ARG";
        case MOE_ERR_UNSUPPORTED: return "MOE_ERR_UNSUPPORTED";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "MOE_ERR_WORKSPACE_TOO_SMALL";
        case MOE_ERR_HIP: return "MOE_ERR_HIP";
    }
    return "MOE_ERR_UNKNOWN";
}

const char *moe_last_error(void) { return g_err; }

moe_status_t moe_launch_floor(int32_t n, void *stream) {
    if (n < 0 || n > 4096) {
        set_error("moe_launch_floor: n=%d outside 0..4096", n);
        return MOE_ERR_INVALID_ARG;
    }
    for (int i = 0; i < n; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
    return check_launch("moe_launch_floor");
}

moe_status_t moe_gate(const moe_shape_t *shape, const void *x, const float *w_gate, const float *logit_bias,
                      float *logits, float *probs, int32_t *expert, float *gate_p, int32_t *slot, int32_t *counts,
                      int32_t *kept, int32_t *token_of_slot, void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (x != nullptr) {
        REQUIRE_PTR(x);
        REQUIRE_PTR(w_gate);
        OPTIONAL_PTR(logit_bias);
    }
    REQUIRE_PTR(logits);
    OPTIONAL_PTR(probs);
    REQUIRE_PTR(expert);
    REQUIRE_PTR(gate_p);
    REQUIRE_PTR(slot);
    REQUIRE_PTR(counts);
    REQUIRE_PTR(kept);
    REQUIRE_PTR(token_of_slot);
    st = check_ws("moe_gate", ws, ws_bytes, gate_ws_bytes(shape));
    if (st != MOE_OK) return st;
    return run_gate(shape, x, w_gate, logit_bias, logits, probs, expert, gate_p, slot, counts, kept, token_of_slot, ws,
                    (hipStream_t)stream);
}

moe_status_t moe_dispatch(const moe_shape_t *shape, const void *x, const int32_t *token_of_slot, void *buf,
                          void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(x);
    REQUIRE_PTR(token_of_slot);
    REQUIRE_PTR(buf);
    return run_dispatch(shape, x, token_of_slot, buf, (hipStream_t)stream);
}

moe_status_t moe_expert_ffn_fwd(const moe_shape_t *shape, const void *buf, const void *w1, const void *w2,
                                const int32_t *kept, void *z_save, void *hact, void *y, void *ws, size_t ws_bytes,
                                void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(buf);
    REQUIRE_PTR(w1);
    REQUIRE_PTR(w2);
    REQUIRE_PTR(kept);
    OPTIONAL_PTR(z_save);
    OPTIONAL_PTR(hact);
    REQUIRE_PTR(y);
    const bool own_hact = hact == nullptr;
    st = check_ws("moe_expert_ffn_fwd", ws, ws_bytes, ffn_fwd_ws_bytes(shape, own_hact));
    if (st != MOE_OK) return st;
    if (own_hact) hact = ws;                   // not kept for the backward: it will be recomputed there
    return ffn_fwd_launch(*shape, buf, w1, w2, kept, z_save, hact, y,
                          (char *)ws + (own_hact ? dz_bytes(shape) : 0), (hipStream_t)stream);
}

moe_status_t moe_expert_ffn_fwd_static(const moe_shape_t *shape, const void *buf, const void *w1, const void *w2,
                                       const int32_t *kept, void *z_save, void *hact, void *y, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(buf);
    REQUIRE_PTR(w1);
    REQUIRE_PTR(w2);
    REQUIRE_PTR(kept);
    OPTIONAL_PTR(z_save);
    REQUIRE_PTR(hact);
    REQUIRE_PTR(y);
    const size_t need = ffn_plan_bytes(shape, G_FWD1, G_FWD2);
    if (need > STATIC_SCRATCH_BYTES) {
        set_error("moe_expert_ffn_fwd_static: the tile plans of this shape need %zu bytes, the library's static scratch "
                  "holds %zu (E=%d C=%lld h=%d f=%d); use moe_expert_ffn_fwd with a workspace",
                  need, STATIC_SCRATCH_BYTES, shape->E, (long long)shape->C, shape->h, shape->f);
        return MOE_ERR_UNSUPPORTED;
    }
    void *plans = nullptr;
    if (need > 0 && (st = static_scratch(&plans)) != MOE_OK) return st;
    // the plan kernel zeroes the fetch counters and rewrites every word the GEMMs read, so what the previous
    // call left in the array does not matter
    return ffn_fwd_launch(*shape, buf, w1, w2, kept, z_save, hact, y, (char *)plans, (hipStream_t)stream);
}

moe_status_t moe_expert_ffn_fwd_fused(const moe_shape_t *shape, const void *x, const void *buf,
                                      const int32_t *token_of_slot, const int32_t *slot, const float *gate_p,
                                      const void *w1, const void *w2, const int32_t *kept, void *z_save, void *hact,
                                      void *y, void *out, void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (shape->dtype != MOE_BF16) {
        set_error("moe_expert_ffn_fwd_fused: bf16 storage only (use moe_dispatch, moe_expert_ffn_fwd, moe_combine)");
        return MOE_ERR_UNSUPPORTED;
    }
    OPTIONAL_PTR(x);
    OPTIONAL_PTR(buf);
    if ((x == nullptr) == (buf == nullptr)) {
        set_error("moe_expert_ffn_fwd_fused: give either x (rows are gathered) or buf (already dispatched)");
        return MOE_ERR_INVALID_ARG;
    }
    REQUIRE_PTR(token_of_slot);
    REQUIRE_PTR(slot);
    REQUIRE_PTR(gate_p);
    REQUIRE_PTR(w1);
    REQUIRE_PTR(w2);
    REQUIRE_PTR(kept);
    OPTIONAL_PTR(z_save);
    OPTIONAL_PTR(hact);
    OPTIONAL_PTR(y);
    REQUIRE_PTR(out);
    const moe_shape_t &s = *shape;
    if (x != nullptr && (double)s.T * s.h * 2.0 >= 2147483648.0) {
        set_error("moe_expert_ffn_fwd_fused: T*h*2 = %.0f bytes of x exceed the 2 GiB a gathered operand can span",
                  (double)s.T * s.h * 2.0);
        return MOE_ERR_UNSUPPORTED;
    }
    const bool own_hact = hact == nullptr;
    st = check_ws("moe_expert_ffn_fwd_fused", ws, ws_bytes, ffn_fwd_ws_bytes(shape, own_hact, true));
    if (st != MOE_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    char *w = (char *)ws;
    if (own_hact) { hact = w; w += dz_bytes(shape); }
    float *scale_of_slot = (float *)w;
    w += slot_scale_bytes(shape);
    GemmDesc g[2] = {ffn_gemm(s, G_FWD1), ffn_gemm(s, G_FWD2)};
    g[0].B = w1; g[0].C = hact; g[0].C2 = z_save; g[0].kept = kept;
    if (buf != nullptr) {
        g[0].A = buf;
    } else {
        g[0].A = x; g[0].a_index = token_of_slot; g[0].a_rows = s.T;
    }
    g[1].A = hact; g[1].B = w2; g[1].C = y; g[1].kept = kept;
    g[1].c_index = token_of_slot; g[1].c_scale = scale_of_slot; g[1].C_scatter = out;
    for (int i = 0; i < 2; ++i) { g[i].plan = w; w += gemm_bf16_plan_bytes(g[i]); }
    if ((st = launch_gemm_bf16_plans(g, 2, hs)) != MOE_OK) return st;
    if ((st = run_combine_prep(shape, token_of_slot, slot, gate_p, scale_of_slot, out, hs)) != MOE_OK) return st;
    for (int i = 0; i < 2; ++i)
        if ((st = launch_gemm_bf16(g[i], hs)) != MOE_OK) return st;
    return MOE_OK;
}

static moe_status_t check_tp(const char *fn, const moe_shape_t *sh, int32_t tp_rank, int32_t tp_size) {
    if (tp_size < 1 || tp_rank < 0 || tp_rank >= tp_size || (int64_t)tp_size > sh->C) {
        set_error("%s: tp_rank=%d tp_size=%d (need 1 <= tp_size <= C = %lld and 0 <= tp_rank < tp_size)", fn, tp_rank,
                  tp_size, (long long)sh->C);
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

moe_status_t moe_dispatch_dtd(const moe_shape_t *shape, const void *x, const int32_t *token_of_slot, int32_t tp_rank,
                              int32_t tp_size, void *share, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((st = check_tp("moe_dispatch_dtd", shape, tp_rank, tp_size)) != MOE_OK) return st;
    REQUIRE_PTR(x);
    REQUIRE_PTR(token_of_slot);
    REQUIRE_PTR(share);
    return run_dispatch_dtd(shape, x, token_of_slot, tp_rank, tp_size, share, (hipStream_t)stream);
}

moe_status_t moe_dtd_drop(const moe_shape_t *shape, const void *buf, const int32_t *kept, int32_t tp_rank,
                          int32_t tp_size, void *share, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((st = check_tp("moe_dtd_drop", shape, tp_rank, tp_size)) != MOE_OK) return st;
    REQUIRE_PTR(buf);
    REQUIRE_PTR(kept);
    REQUIRE_PTR(share);
    return run_dtd_drop(shape, buf, kept, tp_rank, tp_size, share, (hipStream_t)stream);
}

moe_status_t moe_dtd_gather(const moe_shape_t *shape, const void *shares, const int32_t *kept, int32_t tp_size,
                            void *buf, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((st = check_tp("moe_dtd_gather", shape, 0, tp_size)) != MOE_OK) return st;
    REQUIRE_PTR(shares);
    REQUIRE_PTR(kept);
    REQUIRE_PTR(buf);
    return run_dtd_gather(shape, shares, kept, tp_size, buf, (hipStream_t)stream);
}

moe_status_t moe_expert_ffn_fwd_dtd(const moe_shape_t *shape, const void *shares, int32_t tp_size, const void *w1,
                                    const void *w2, const int32_t *kept, void *z_save, void *hact, void *y, void *ws,
                                    size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((st = check_tp("moe_expert_ffn_fwd_dtd", shape, 0, tp_size)) != MOE_OK) return st;
    if (shape->dtype != MOE_BF16) {
        set_error("moe_expert_ffn_fwd_dtd: bf16 storage only (use moe_dtd_gather, then moe_expert_ffn_fwd)");
        return MOE_ERR_UNSUPPORTED;
    }
    const int64_t Cg = (shape->C + tp_size - 1) / tp_size;
    if ((double)tp_size * shape->E * (double)Cg * shape->h * 2.0 >= 2147483648.0) {
        set_error("moe_expert_ffn_fwd_dtd: the shares span %.0f bytes, beyond the 2 GiB a gathered operand can span",
                  (double)tp_size * shape->E * (double)Cg * shape->h * 2.0);
        return MOE_ERR_UNSUPPORTED;
    }
    REQUIRE_PTR(shares);
    REQUIRE_PTR(w1);
    REQUIRE_PTR(w2);
    REQUIRE_PTR(kept);
    OPTIONAL_PTR(z_save);
    OPTIONAL_PTR(hact);
    REQUIRE_PTR(y);
    const bool own_hact = hact == nullptr;
    st = check_ws("moe_expert_ffn_fwd_dtd", ws, ws_bytes, ffn_fwd_ws_bytes(shape, own_hact));
    if (st != MOE_OK) return st;
    if (own_hact) hact = ws;
    return ffn_fwd_launch(*shape, shares, w1, w2, kept, z_save, hact, y,
                          (char *)ws + (own_hact ? dz_bytes(shape) : 0), (hipStream_t)stream, tp_size);
}

moe_status_t moe_dispatch_bwd_dtd(const moe_shape_t *shape, const void *d_shares, int32_t tp_size,
                                  const int32_t *expert, const int32_t *slot, void *d_x, const float *d_logits,
                                  const float *w_gate, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((st = check_tp("moe_dispatch_bwd_dtd", shape, 0, tp_size)) != MOE_OK) return st;
    REQUIRE_PTR(d_shares);
    REQUIRE_PTR(expert);
    REQUIRE_PTR(slot);
    REQUIRE_PTR(d_x);
    OPTIONAL_PTR(d_logits);
    OPTIONAL_PTR(w_gate);
    if ((d_logits == nullptr) != (w_gate == nullptr)) {
        set_error("moe_dispatch_bwd_dtd: d_logits and w_gate must be given together");
        return MOE_ERR_INVALID_ARG;
    }
    if (d_logits == nullptr) return run_dispatch_bwd(shape, d_shares, expert, slot, d_x, (hipStream_t)stream, tp_size);
    if (shape->dtype == MOE_BF16)
        return run_dispatch_bwd_fused(shape, d_shares, expert, slot, d_x, d_logits, w_gate, (hipStream_t)stream, tp_size);
    st = run_dispatch_bwd(shape, d_shares, expert, slot, d_x, (hipStream_t)stream, tp_size);
    if (st != MOE_OK) return st;
    return run_gate_dx_f32(shape, d_logits, w_gate, d_x, (hipStream_t)stream);
}

moe_status_t moe_combine(const moe_shape_t *shape, const void *y, const int32_t *expert, const int32_t *slot,
                         const float *gate_p, void *out, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(y);
    REQUIRE_PTR(expert);
    REQUIRE_PTR(slot);
    REQUIRE_PTR(gate_p);
    REQUIRE_PTR(out);
    return run_combine(shape, y, expert, slot, gate_p, out, (hipStream_t)stream);
}

moe_status_t moe_combine_bwd(const moe_shape_t *shape, const void *d_out, const void *y, const int32_t *token_of_slot,
                             const int32_t *slot, const float *gate_p, void *d_y, float *d_gate_p, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(d_out);
    REQUIRE_PTR(y);
    REQUIRE_PTR(token_of_slot);
    REQUIRE_PTR(slot);
    REQUIRE_PTR(gate_p);
    REQUIRE_PTR(d_y);
    REQUIRE_PTR(d_gate_p);
    return run_combine_bwd(shape, d_out, y, token_of_slot, slot, gate_p, d_y, d_gate_p, (hipStream_t)stream);
}

moe_status_t moe_expert_ffn_bwd(const moe_shape_t *shape, const void *d_y, const void *buf, const void *z_save,
                                const void *hact, const void *w1, const void *w2, const int32_t *kept, void *d_buf,
                                void *d_w1, void *d_w2, void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(d_y);
    REQUIRE_PTR(buf);
    OPTIONAL_PTR(z_save);
    OPTIONAL_PTR(hact);
    REQUIRE_PTR(w1);
    REQUIRE_PTR(w2);
    REQUIRE_PTR(kept);
    REQUIRE_PTR(d_buf);
    REQUIRE_PTR(d_w1);
    REQUIRE_PTR(d_w2);
    if ((z_save == nullptr) != (hact == nullptr)) {
        set_error("moe_expert_ffn_bwd: z_save and hact must be given together (or both NULL to recompute them)");
        return MOE_ERR_INVALID_ARG;
    }
    const bool recompute = hact == nullptr;
    st = check_ws("moe_expert_ffn_bwd", ws, ws_bytes, ffn_bwd_ws_bytes(shape, recompute));
    if (st != MOE_OK) return st;
    const moe_shape_t &s = *shape;
    const bool bf = s.dtype == MOE_BF16;
    hipStream_t hs = (hipStream_t)stream;
    void *d_z = ws;
    char *after = (char *)ws + dz_bytes(shape);
    if (recompute) {
        // activation recomputation: the forward's first GEMM again, hact and GeLU'(z) into the workspace
        void *hact_r = after, *zs_r = after + dz_bytes(shape);
        after += 2 * dz_bytes(shape);
        GemmDesc r = ffn_gemm(s, G_FWD1);
        r.A = buf; r.B = w1; r.C = hact_r; r.C2 = zs_r; r.kept = kept;
        if (bf) {
            r.plan = after;
            after += gemm_bf16_plan_bytes(r);
            if ((st = launch_gemm_bf16_plans(&r, 1, hs)) != MOE_OK) return st;
        }
        if ((st = bf ? launch_gemm_bf16(r, hs) : launch_gemm_f32(r, hs)) != MOE_OK) return st;
        hact = hact_r;
        z_save = zs_r;
    }
    GemmDesc g[4] = {ffn_gemm(s, G_DH), ffn_gemm(s, G_DW2), ffn_gemm(s, G_DW1), ffn_gemm(s, G_DD)};
    g[0].A = d_y; g[0].B = w2; g[0].C = d_z; g[0].Zin = z_save;
    g[1].A = hact; g[1].B = d_y; g[1].C = d_w2;
    g[2].A = buf; g[2].B = d_z; g[2].C = d_w1;
    g[3].A = d_z; g[3].B = w1; g[3].C = d_buf;
    for (int i = 0; i < 4; ++i) g[i].kept = kept;
    if (bf) {
        char *pl = after;
        for (int i = 0; i < 4; ++i) { g[i].plan = pl; pl += gemm_bf16_plan_bytes(g[i]); }
        if ((st = launch_gemm_bf16_plans(g, 4, hs)) != MOE_OK) return st;
    }
    SideStream *ss = bf ? side_stream(hs) : nullptr;
    if (ss == nullptr) {     // fp32, or no side stream: one after the other
        for (int i = 0; i < 4; ++i)
            if ((st = bf ? launch_gemm_bf16(g[i], hs) : launch_gemm_f32(g[i], hs)) != MOE_OK) return st;
        return MOE_OK;
    }
    // caller's stream: plans, dH, dD;  side stream: dW2 (next to dH), dW1 (needs d_z, next to dD)
    auto hip_ok = [](hipError_t e, const char *what) {
        if (e == hipSuccess) return MOE_OK;
        set_error("moe_expert_ffn_bwd: %s: %s", what, hipGetErrorString(e));
        return MOE_ERR_HIP;
    };
    if ((st = hip_ok(hipEventRecord(ss->fork, hs), "event record")) != MOE_OK) return st;
    if ((st = hip_ok(hipStreamWaitEvent(ss->stream, ss->fork, 0), "stream wait")) != MOE_OK) return st;
    // From here on the side stream is tied to the caller's stream (under stream capture it has joined the
    // capture), so whatever fails below, the join at the end is still enqueued before the call returns.
    moe_status_t main_st = launch_gemm_bf16(g[0], hs);
    moe_status_t side = MOE_OK;
    if (main_st == MOE_OK) {
        side = launch_gemm_bf16(g[1], ss->stream);
        if (side == MOE_OK) side = hip_ok(hipEventRecord(ss->mid, hs), "event record");
        if (side == MOE_OK) side = hip_ok(hipStreamWaitEvent(ss->stream, ss->mid, 0), "stream wait");
        if (side == MOE_OK) side = launch_gemm_bf16(g[2], ss->stream);
        main_st = launch_gemm_bf16(g[3], hs);
    }
    moe_status_t j = hip_ok(hipEventRecord(ss->join, ss->stream), "event record");
    if (j == MOE_OK) j = hip_ok(hipStreamWaitEvent(hs, ss->join, 0), "stream wait");
    return main_st != MOE_OK ? main_st : (side != MOE_OK ? side : j);
}

moe_status_t moe_dispatch_bwd(const moe_shape_t *shape, const void *d_buf, const int32_t *expert, const int32_t *slot,
                              void *d_x, const float *d_logits, const float *w_gate, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(d_buf);
    REQUIRE_PTR(expert);
    REQUIRE_PTR(slot);
    REQUIRE_PTR(d_x);
    OPTIONAL_PTR(d_logits);
    OPTIONAL_PTR(w_gate);
    if ((d_logits == nullptr) != (w_gate == nullptr)) {
        set_error("moe_dispatch_bwd: d_logits and w_gate must be given together");
        return MOE_ERR_INVALID_ARG;
    }
    if (d_logits == nullptr) return run_dispatch_bwd(shape, d_buf, expert, slot, d_x, (hipStream_t)stream);
    if (shape->dtype == MOE_BF16)
        return run_dispatch_bwd_fused(shape, d_buf, expert, slot, d_x, d_logits, w_gate, (hipStream_t)stream);
    // fp32 storage: plain row gather, then the gate part added in place
    st = run_dispatch_bwd(shape, d_buf, expert, slot, d_x, (hipStream_t)stream);
    if (st != MOE_OK) return st;
    return run_gate_dx_f32(shape, d_logits, w_gate, d_x, (hipStream_t)stream);
}

moe_status_t moe_gate_bwd(const moe_shape_t *shape, const float *d_gate_p, const float *probs, const int32_t *expert,
                          const void *x, const float *w_gate, float *d_logits, float *d_w_gate, void *d_x_accum,
                          void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    REQUIRE_PTR(d_gate_p);
    REQUIRE_PTR(probs);
    REQUIRE_PTR(expert);
    REQUIRE_PTR(x);
    REQUIRE_PTR(w_gate);
    REQUIRE_PTR(d_logits);
    OPTIONAL_PTR(d_w_gate);
    OPTIONAL_PTR(d_x_accum);
    st = check_ws("moe_gate_bwd", ws, ws_bytes, d_w_gate ? gate_bwd_ws_bytes(shape) : 0);
    if (st != MOE_OK) return st;
    return run_gate_bwd(shape, d_gate_p, probs, expert, x, w_gate, d_logits, d_w_gate, d_x_accum, ws,
                        (hipStream_t)stream);
}

moe_status_t moe_adamw_tiled(int64_t n, int64_t ts, const moe_adamw_t *hp, const void *grad, float *master,
                             float *exp_avg, float *exp_avg_sq, void *param, float *staging, int32_t dtype,
                             void *stream) {
    if (hp == nullptr) {
        set_error("moe_adamw_tiled: hp is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (n < 0 || ts < 1 || hp->step < 1) {
        set_error("moe_adamw_tiled: n=%lld ts=%lld step=%d (need n >= 0, ts >= 1, step >= 1)", (long long)n,
                  (long long)ts, hp->step);
        return MOE_ERR_INVALID_ARG;
    }
    auto ok_nonneg = [](float v) { return std::isfinite(v) && v >= 0.0f; };
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f) || !ok_nonneg(hp->lr) ||
        !ok_nonneg(hp->eps) || !ok_nonneg(hp->weight_decay) || !std::isfinite(hp->grad_mult)) {
        set_error("moe_adamw_tiled: hyperparameters out of range (lr=%g beta1=%g beta2=%g eps=%g weight_decay=%g "
                  "grad_mult=%g)", hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, hp->grad_mult);
        return MOE_ERR_INVALID_ARG;
    }
    if (dtype != MOE_F32 && dtype != MOE_BF16) {
        set_error("moe_adamw_tiled: unknown dtype %d", dtype);
        return MOE_ERR_UNSUPPORTED;
    }
    if (n >= ((int64_t)1 << 40)) {
        set_error("moe_adamw_tiled: n=%lld is beyond the supported 2^40", (long long)n);
        return MOE_ERR_UNSUPPORTED;
    }
    if (n == 0) return MOE_OK;
    REQUIRE_PTR(grad);
    REQUIRE_PTR(master);
    REQUIRE_PTR(exp_avg);
    REQUIRE_PTR(exp_avg_sq);
    REQUIRE_PTR(param);
    OPTIONAL_PTR(staging);
    if (staging != nullptr && ts < n && ts % 8 != 0) {
        set_error("moe_adamw_tiled: ts=%lld must be a multiple of 8 when the group has more than one tile",
                  (long long)ts);
        return MOE_ERR_UNSUPPORTED;
    }
    // constants in double, rounded once; 1 - beta is exact in fp32 for beta in [0.5, 1)
    const double bc1 = 1.0 - std::pow((double)hp->beta1, (double)hp->step);
    const double bc2 = 1.0 - std::pow((double)hp->beta2, (double)hp->step);
    AdamwConst c;
    c.lr = hp->lr;
    c.beta1 = hp->beta1;
    c.beta2 = hp->beta2;
    c.omb1 = (float)(1.0 - (double)hp->beta1);
    c.omb2 = (float)(1.0 - (double)hp->beta2);
    c.eps = hp->eps;
    c.wd = hp->weight_decay;
    c.inv_bc1 = (float)(1.0 / bc1);
    c.inv_bc2 = (float)(1.0 / bc2);
    c.grad_mult = hp->grad_mult;
    return run_adamw_tiled(n, ts, c, grad, master, exp_avg, exp_avg_sq, param, staging, dtype, (hipStream_t)stream);
}

}  // extern "C"
