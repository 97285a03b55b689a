// HBM stream probes with 16-byte accesses: a read-only pass and a copy over
// buffers far larger than the caches.  `copy_kernel` (1 GiB in, 1 GiB out per
// launch) is also the reference dispatch that the FETCH_SIZE / WRITE_SIZE
// counters of other kernels are scaled by.
#include <hip/hip_runtime.h>
#include <cstdio>

#define CK(e) do { hipError_t e_ = (e); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at %s\n", (int)e_, #e); return 1; } } while (0)

__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ p, size_t n, unsigned* out) {
    unsigned s = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const uint4 v = p[i];
        s += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (s == 0x12345678u) out[0] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ p, uint4* __restrict__ q, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) q[i] = p[i];
}

int main() {
    const size_t bytes = (size_t)1 << 30, n = bytes / 16;
    uint4 *a, *b;
    unsigned* out;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMalloc(&out, 4));
    CK(hipMemset(a, 1, bytes));
    CK(hipMemset(b, 2, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int grid = 2048;
    float ms, best_r = 1e9f, best_c = 1e9f;
    for (int rep = 0; rep < 5; ++rep) {
        CK(hipEventRecord(e0));
        hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, 0, a, n, out);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best_r) best_r = ms;
        CK(hipEventRecord(e0));
        hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, 0, a, b, n);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best_c) best_c = ms;
    }
    printf("read  1 GiB: %.3f ms  %.1f GB/s\n", best_r, bytes / best_r / 1e6);
    printf("copy  1 GiB: %.3f ms  %.1f GB/s (read + write)\n", best_c, 2.0 * bytes / best_c / 1e6);
    return 0;
}
