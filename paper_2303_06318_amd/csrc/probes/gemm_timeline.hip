// Timeline of one launch of the grouped bf16 GEMM: when each tile started and ended (constant
// 100 MHz wall clock) and how many shader cycles it took, which gives the shader clock the chip
// actually ran at, the number of rounds, and the gaps between rounds.  Built together with the
// kernel source, with the timeline stamps and optionally one of the ablation variants switched on:
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -DMOE_GEMM_TL=1 [-DMOE_GEMM_DBG=<1|5|6|7|8>] -o /tmp/gemm_timeline \
//         paper_2303_06318_amd/csrc/probes/gemm_timeline.hip paper_2303_06318_amd/csrc/gemm_bf16.hip
//   /tmp/gemm_timeline [mode] [rows_per_expert]
//
// mode 0: [M,K] x [K,N] (forward), 1: [M,K] x [N,K] (data gradient), 2: [K,M] x [K,N] (weight
// gradient); rows_per_expert 0 = 1024 +- 60 as in the layer's workload.  E = 16, h = f = 4096.
// Operands hold random bf16 bits (sign, mantissa, a few exponents): the clock depends on the data.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../moe_common.h"

namespace moe {
void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vfprintf(stderr, fmt, ap);
    va_end(ap);
}
moe_status_t check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        fprintf(stderr, "%s: %s\n", what, hipGetErrorString(e));
        return MOE_ERR_HIP;
    }
    return MOE_OK;
}
}  // namespace moe
using namespace moe;

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));               \
            return 1;                                                             \
        }                                                                         \
    } while (0)

__global__ void fill_random_bf16(unsigned short *p, size_t n, unsigned seed) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    unsigned r = (unsigned)i * 2654435761u + seed;
    r ^= r >> 15; r *= 2246822519u; r ^= r >> 13; r *= 3266489917u; r ^= r >> 16;
    p[i] = (unsigned short)(((r >> 31) << 15) | ((120u + ((r >> 8) & 7u)) << 7) | (r & 0x7fu));
}

int main(int argc, char **argv) {
    const int E = 16, C = 1280, h = 4096, f = 4096;
    const int mode = argc > 1 ? atoi(argv[1]) : 0;
    const int fixed = argc > 2 ? atoi(argv[2]) : 0;
    if (mode < 0 || mode > 2 || fixed < 0 || fixed > C) {
        fprintf(stderr, "usage: gemm_timeline [mode 0..2] [rows_per_expert 0..%d]\n", C);
        return 2;
    }
    const size_t nA = (size_t)E * C * h, nB = (size_t)E * h * f, nC = (size_t)E * C * f;
    void *A, *B, *Cc;
    int32_t *kept;
    CHECK(hipMalloc(&A, nA * 2));
    CHECK(hipMalloc(&B, nB * 2));
    CHECK(hipMalloc(&Cc, (mode == 2 ? nB : nC) * 2));
    CHECK(hipMalloc(&kept, E * 4));
    fill_random_bf16<<<(unsigned)((nA + 255) / 256), 256>>>((unsigned short *)A, nA, 1u);
    fill_random_bf16<<<(unsigned)((nB + 255) / 256), 256>>>((unsigned short *)B, nB, 2u);
    std::vector<int32_t> hk(E);
    long rows = 0;
    srand(1);
    for (int e = 0; e < E; ++e) {
        hk[e] = fixed ? fixed : 1024 + (rand() % 121) - 60;
        rows += hk[e];
    }
    CHECK(hipMemcpy(kept, hk.data(), E * 4, hipMemcpyHostToDevice));
    GemmDesc g = {};
    g.kept = kept; g.E = E; g.epi = EPI_STORE; g.act = 0;
    g.A = A; g.C = Cc;
    if (mode == 0) {
        g.B = B; g.strideA = (int64_t)C * h; g.strideB = (int64_t)h * f; g.strideC = (int64_t)C * f;
        g.M = C; g.N = f; g.K = h; g.lda = h; g.ldb = f; g.ldc = f; g.a_xc = 0; g.b_xc = 1; g.rows_from_kept = 1;
    } else if (mode == 1) {
        g.B = B; g.strideA = (int64_t)C * h; g.strideB = (int64_t)h * f; g.strideC = (int64_t)C * f;
        g.M = C; g.N = f; g.K = h; g.lda = h; g.ldb = h; g.ldc = f; g.a_xc = 0; g.b_xc = 0; g.rows_from_kept = 1;
    } else {
        g.B = A; g.strideA = (int64_t)C * h; g.strideB = (int64_t)C * h; g.strideC = (int64_t)h * f;
        g.M = h; g.N = f; g.K = C; g.lda = h; g.ldb = h; g.ldc = f; g.a_xc = 1; g.b_xc = 1; g.rows_from_kept = 0;
    }
    void *plan;
    CHECK(hipMalloc(&plan, gemm_bf16_plan_bytes(g)));
    g.plan = plan;
    const int max_wg = 8192;                       // more than the tiles of any of these shapes
    const int it = 20;                             // timed launches, each with its own stamp buffer
    long long *stamps_all;
    CHECK(hipMalloc(&stamps_all, (size_t)it * max_wg * 32));
    CHECK(hipMemset(stamps_all, 0, (size_t)it * max_wg * 32));
    long long *stamps = stamps_all + (size_t)(it - 1) * max_wg * 4;
    bool stamped = false;
#if defined(MOE_GEMM_TL) && MOE_GEMM_TL
    stamped = true;
#endif
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int i = 0; i < 3; ++i) {
        launch_gemm_bf16_plans(&g, 1, 0);
        launch_gemm_bf16(g, 0);
    }
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0, 0));
    for (int i = 0; i < it; ++i) {
        if (stamped) g.C2 = stamps_all + (size_t)i * max_wg * 4;
        launch_gemm_bf16_plans(&g, 1, 0);
        launch_gemm_bf16(g, 0);
    }
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    ms /= it;
    const double flops = 2.0 * h * f * rows;       // every mode multiplies rows x 4096 x 4096 per expert
    printf("mode %d rows %ld: %.1f us per launch, %.0f TFLOP/s\n", mode, rows, ms * 1e3, flops / ms / 1e9);

    std::vector<long long> tl((size_t)max_wg * 4);
    CHECK(hipMemcpy(tl.data(), stamps, (size_t)max_wg * 32, hipMemcpyDeviceToHost));
    struct Rec { long long start, end, cycles, id; };
    std::vector<Rec> recs;
    for (int i = 0; i < max_wg; ++i)
        if (tl[4 * i]) recs.push_back({tl[4 * i], tl[4 * i + 1], tl[4 * i + 2], tl[4 * i + 3]});
    if (recs.empty()) {
        printf("no stamps (build with -DMOE_GEMM_TL=1)\n");
        return 0;
    }
    std::sort(recs.begin(), recs.end(), [](const Rec &a, const Rec &b) { return a.start < b.start; });
    const long long t0 = recs[0].start;
    long long tend = 0;
    for (auto &r : recs) tend = std::max(tend, r.end);
    printf("last launch: %zu tiles, span %.1f us\n", recs.size(), (tend - t0) / 100.0);
    {
        std::vector<long long> tp((size_t)it * max_wg * 4);
        CHECK(hipMemcpy(tp.data(), stamps_all, (size_t)it * max_wg * 32, hipMemcpyDeviceToHost));
        long long first = 0, pend = 0;
        printf("launch: first entry, last exit (us since the first launch's first entry), gap to the previous launch\n");
        for (int l = 0; l < it; ++l) {
            long long lo = 1LL << 62, hi = 0;
            for (int i = 0; i < max_wg; ++i) {
                const long long *r = &tp[((size_t)l * max_wg + i) * 4];
                if (r[0]) { lo = std::min(lo, r[0]); hi = std::max(hi, r[1]); }
            }
            if (l == 0) first = lo;
            printf("  %2d: %8.1f %8.1f  %6.1f\n", l, (lo - first) / 100.0, (hi - first) / 100.0, l ? (lo - pend) / 100.0 : 0.0);
            pend = hi;
        }
        std::vector<double> du;
        for (auto &r : recs) du.push_back((r.end - r.start) / 100.0);
        std::sort(du.begin(), du.end());
        printf("tile duration us: min %.1f  p10 %.1f  median %.1f  p90 %.1f  max %.1f\n", du[0], du[du.size() / 10], du[du.size() / 2],
               du[du.size() * 9 / 10], du.back());
    }
    printf("round  start_us  end_us  duration_us  shader_cycles  shader_MHz   (medians over 256 tiles by start time)\n");
    for (size_t q = 0; q < recs.size(); q += 256) {
        const size_t n = std::min<size_t>(256, recs.size() - q);
        std::vector<double> st, en, du, cy, mhz;
        for (size_t i = q; i < q + n; ++i) {
            const Rec &r = recs[i];
            st.push_back((r.start - t0) / 100.0);
            en.push_back((r.end - t0) / 100.0);
            du.push_back((r.end - r.start) / 100.0);
            cy.push_back((double)r.cycles);
            mhz.push_back(r.end > r.start ? 100.0 * r.cycles / (r.end - r.start) : 0.0);
        }
        auto med = [](std::vector<double> &v) { std::sort(v.begin(), v.end()); return v[v.size() / 2]; };
        printf("%5zu  %8.1f  %6.1f  %11.1f  %13.0f  %10.0f   (%zu tiles)\n", q / 256, med(st), med(en), med(du), med(cy),
               med(mhz), n);
    }
    // by blocks per tile, and the time each XCD's last workgroup ended
    for (int nb = 1; nb <= 9; ++nb) {
        std::vector<double> du, cy;
        for (auto &r : recs)
            if ((r.id & 255) == nb) { du.push_back((r.end - r.start) / 100.0); cy.push_back((double)r.cycles); }
        if (du.empty()) continue;
        std::sort(du.begin(), du.end());
        std::sort(cy.begin(), cy.end());
        std::vector<double> sc;
        for (auto &r : recs)
            if ((r.id & 255) == nb) sc.push_back((double)(r.id >> 32));
        std::sort(sc.begin(), sc.end());
        printf("tiles of %d blocks: %zu, duration us median %.1f max %.1f, shader cycles median %.0f (schedule %.0f)\n", nb, du.size(),
               du[du.size() / 2], du.back(), cy[cy.size() / 2], sc[sc.size() / 2]);
    }
    printf("last exit per XCD (us), tiles:");
    for (int x = 0; x < 8; ++x) {
        long long hi = 0; int n = 0;
        for (auto &r : recs)
            if (((r.id >> 20) & 15) == x) { hi = std::max(hi, r.end); ++n; }
        printf(" %.1f (%d)", (hi - t0) / 100.0, n);
    }
    printf("\n");
    // tiles in flight, sampled every 20 us
    printf("in flight:");
    for (long long t = t0; t < tend; t += 2000) {
        int c = 0;
        for (auto &r : recs) c += (r.start <= t && r.end > t);
        printf(" %d", c);
    }
    printf("\n");
    return 0;
}
