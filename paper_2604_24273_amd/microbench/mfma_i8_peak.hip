// Achievable int8 matrix-core rate on this chip: a loop of independent
// v_mfma_i32_32x32x32_i8 with no memory traffic, on three kinds of operands
// (all zero, random int8 x random int8, random int8 x ternary offset codes).
// The data-dependent rates differ because the chip runs against its power
// limit; the third line is the ceiling that applies to BitLinear.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

#define CK(e) do { hipError_t e_ = (e); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at %s\n", (int)e_, #e); return 1; } } while (0)

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_loop(int iters, const v4i* __restrict__ src, int* out) {
    v4i a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(blockIdx.x * 256 + threadIdx.x) * 8 + i];
        b[i] = src[(blockIdx.x * 256 + threadIdx.x) * 8 + 4 + i];
    }
    v16i acc[16];
    for (int i = 0; i < 16; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 16; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (s == 0x12345678) out[0] = s;
}

int main() {
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int grid = prop.multiProcessorCount, n = grid * 256 * 8, iters = 20000;
    v4i* h = (v4i*)malloc((size_t)n * sizeof(v4i));
    v4i* d;
    int* out;
    CK(hipMalloc(&d, (size_t)n * sizeof(v4i)));
    CK(hipMalloc(&out, 4));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const char* names[3] = {"zeros", "random int8 x random int8", "random int8 x ternary offset codes"};
    printf("device: %s, %d CUs\n", prop.name, grid);
    for (int mode = 0; mode < 3; ++mode) {
        srand(1);
        for (int i = 0; i < n; ++i)
            for (int c = 0; c < 4; ++c) {
                int r = 0;
                if (mode == 1 || (mode == 2 && i % 8 < 4)) r = rand() ^ (rand() << 16);
                if (mode == 2 && i % 8 >= 4)
                    for (int q = 0; q < 4; ++q) r |= (rand() % 3) << (8 * q);
                h[i][c] = r;
            }
        CK(hipMemcpy(d, h, (size_t)n * sizeof(v4i), hipMemcpyHostToDevice));
        double best = 0;
        for (int rep = 0; rep < 4; ++rep) {
            CK(hipEventRecord(e0));
            hipLaunchKernelGGL(mfma_loop, dim3(grid), dim3(256), 0, 0, iters, d, out);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            const double tops = (double)grid * 4 * iters * 16 * 65536.0 / ms / 1e9;
            if (tops > best) best = tops;
        }
        printf("%-36s %8.1f TOP/s\n", names[mode], best);
    }
    return 0;
}
