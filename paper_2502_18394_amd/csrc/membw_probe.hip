// Stand-alone probe of the streaming bandwidth this GPU actually delivers (read, write,
// in-place read+write, copy) as a function of working-set size.  It is the yardstick the
// benchmark quotes next to the nominal 8 TB/s: a kernel that moves its algorithmic bytes at
// the probe's copy rate cannot go faster without moving fewer bytes.
//   usage: membw_probe [size_mb ...]      prints one line per size, GB/s
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

__global__ __launch_bounds__(256) void k_read(const float4 *__restrict__ p, size_t n, float *out) {
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float4 v = p[i];
        acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 123.456f) out[0] = acc;   // keeps the loads alive; practically never true
}
__global__ __launch_bounds__(256) void k_write(float4 *__restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        p[i] = make_float4(1.f, 2.f, 3.f, 4.f);
}
__global__ __launch_bounds__(256) void k_rw(float4 *__restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        float4 v = p[i];
        v.x += 1.f;
        p[i] = v;
    }
}
__global__ __launch_bounds__(256) void k_copy(const float4 *__restrict__ a, float4 *__restrict__ b, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) b[i] = a[i];
}

int main(int argc, char **argv) {
    std::vector<size_t> sizes;
    for (int i = 1; i < argc; ++i) {
        const long v = std::atol(argv[i]);
        if (v >= 1 && v <= 8192) sizes.push_back((size_t)v);
    }
    if (sizes.empty()) sizes = {32, 128, 256, 1024, 4096};
    size_t maxmb = 0;
    for (size_t s : sizes) maxmb = s > maxmb ? s : maxmb;
    float4 *a = nullptr, *b = nullptr;
    float *out = nullptr;
    CK(hipMalloc(&a, maxmb << 20));
    CK(hipMalloc(&b, maxmb << 20));
    CK(hipMalloc(&out, 4));
    CK(hipMemset(a, 0, maxmb << 20));
    CK(hipMemset(b, 0, maxmb << 20));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int grid = 256 * 16;
    std::printf("# working set MB, GB/s: read, write, read+write in place (bytes both ways), copy (bytes both ways)\n");
    for (size_t mb : sizes) {
        const size_t bytes = mb << 20, n = bytes / 16;
        int reps = (int)(((size_t)16 << 30) / bytes);
        reps = reps < 4 ? 4 : (reps > 200 ? 200 : reps);
        double r[4];
        for (int which = 0; which < 4; ++which) {
            float ms = 0.f;
            for (int i = -2; i < reps; ++i) {
                if (i == 0) CK(hipEventRecord(e0));
                if (which == 0) k_read<<<grid, 256>>>(a, n, out);
                else if (which == 1) k_write<<<grid, 256>>>(a, n);
                else if (which == 2) k_rw<<<grid, 256>>>(a, n);
                else k_copy<<<grid, 256>>>(a, b, n / 2);
            }
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
            const double moved = (which == 2) ? 2.0 * bytes : (double)bytes;
            r[which] = moved * reps / (ms * 1e-3) / 1e9;
        }
        std::printf("%zu %.0f %.0f %.0f %.0f\n", mb, r[0], r[1], r[2], r[3]);
        std::fflush(stdout);
    }
    CK(hipFree(a));
    CK(hipFree(b));
    CK(hipFree(out));
    return 0;
}
