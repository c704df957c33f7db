// Streaming ceilings of the chip's HBM path: read-only, write-only, copy, and four arrays read while four
// are written (the access mix of the optimizer update), with one-shot and with persistent grids.
// Stand-alone probe, not part of the library:
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o /tmp/hbm_stream paper_2303_06318_amd/csrc/probes/hbm_stream.hip
//   /tmp/hbm_stream
//
// Arrays of 1 GiB (far beyond the 256 MB last-level cache), 16-byte accesses, 10 timed launches each.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __attribute__((ext_vector_type(4))) float f4;
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

template <int U> __global__ __launch_bounds__(256) void k_read(const f4 *a, size_t n, float *sink) {
    f4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n; i += (size_t)gridDim.x * 256 * U) {
        f4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) if (i + u * 256 < n) v[u] = a[i + u * 256]; else v[u] = acc;
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
    if (acc[0] + acc[1] + acc[2] + acc[3] == 1.2345f) *sink = 1.0f;
}
template <int U> __global__ __launch_bounds__(256) void k_write(f4 *a, size_t n) {
    f4 v = {1, 2, 3, 4};
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n; i += (size_t)gridDim.x * 256 * U) {
#pragma unroll
        for (int u = 0; u < U; ++u) if (i + u * 256 < n) a[i + u * 256] = v;
    }
}
template <int U> __global__ __launch_bounds__(256) void k_copy(const f4 *a, f4 *b, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n; i += (size_t)gridDim.x * 256 * U) {
        f4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) if (i + u * 256 < n) v[u] = a[i + u * 256];
#pragma unroll
        for (int u = 0; u < U; ++u) if (i + u * 256 < n) b[i + u * 256] = v[u];
    }
}
// in-place update of 3 arrays + read of a 4th + write of a 5th (like the optimizer: rw rw rw r w)
__global__ __launch_bounds__(256) void k_mix(f4 *a, f4 *b, f4 *c, const f4 *d, f4 *e, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        f4 x = a[i], y = b[i], z = c[i], w = d[i];
        a[i] = x + w; b[i] = y + w; c[i] = z * w; e[i] = x + y;
    }
}
int main() {
    const size_t bytes = (size_t)1 << 30, n = bytes / 16;
    f4 *p[5];
    for (int i = 0; i < 5; ++i) { CHECK(hipMalloc(&p[i], bytes)); CHECK(hipMemset(p[i], 0, bytes)); }
    float *sink; CHECK(hipMalloc(&sink, 4));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    auto run = [&](const char *name, double moved, auto launch) {
        for (int i = 0; i < 2; ++i) launch();
        (void)hipEventRecord(e0, 0);
        for (int i = 0; i < 10; ++i) launch();
        (void)hipEventRecord(e1, 0);
        (void)hipEventSynchronize(e1);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        ms /= 10;
        printf("%-34s %8.1f us  %7.0f GB/s\n", name, ms * 1e3, moved / ms / 1e6); fflush(stdout);
    };
    const unsigned full = (unsigned)(n / 256);
    run("read  one-shot U=1", bytes, [&] { k_read<1><<<full, 256>>>(p[0], n, sink); });
    run("read  one-shot U=4", bytes, [&] { k_read<4><<<full / 4, 256>>>(p[0], n, sink); });
    run("read  persistent 256x8 U=4", bytes, [&] { k_read<4><<<2048, 256>>>(p[0], n, sink); });
    run("read  persistent 256x16 U=2", bytes, [&] { k_read<2><<<4096, 256>>>(p[0], n, sink); });
    run("write one-shot U=1", bytes, [&] { k_write<1><<<full, 256>>>(p[1], n); });
    run("write persistent 256x8 U=4", bytes, [&] { k_write<4><<<2048, 256>>>(p[1], n); });
    run("copy  one-shot U=1", 2.0 * bytes, [&] { k_copy<1><<<full, 256>>>(p[0], p[1], n); });
    run("copy  one-shot U=4", 2.0 * bytes, [&] { k_copy<4><<<full / 4, 256>>>(p[0], p[1], n); });
    run("copy  persistent 256x8 U=4", 2.0 * bytes, [&] { k_copy<4><<<2048, 256>>>(p[0], p[1], n); });
    run("hipMemcpyAsync d2d", 2.0 * bytes, [&] { (void)hipMemcpyAsync(p[1], p[0], bytes, hipMemcpyDeviceToDevice, 0); });
    run("mix 4r4w one-shot", 8.0 * bytes, [&] { k_mix<<<full, 256>>>(p[0], p[1], p[2], p[3], p[4], n); });
    run("mix 4r4w persistent 256x8", 8.0 * bytes, [&] { k_mix<<<2048, 256>>>(p[0], p[1], p[2], p[3], p[4], n); });
    return 0;
}
