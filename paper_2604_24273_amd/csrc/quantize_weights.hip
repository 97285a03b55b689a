// Ternary weight quantisation and 2-bit packing (paper Sec. 3.1, Eq. 2).
//
//   gamma = mean |W|  (fp64 accumulation in a fixed order, rounded to fp32 once)
//   beta  = gamma + eps,  tau = beta / 2
//   code  = (w > tau) - (w < -tau)          (|w| == tau -> 0, as Eq. 2's strict >)
//
// Two launches: per-block fp64 partial sums of |W|, then a pack kernel in which
// every block re-reduces the partials in the same fixed order (so all blocks
// see the same beta and the result does not depend on scheduling).
#include "common.hpp"

namespace brl {

namespace {

constexpr int QW_THREADS = 256;

__device__ inline double block_sum_fixed(double v, double* lds) {
    // fixed reduction tree: xor-butterfly inside the wave, then waves in order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < QW_THREADS / 64; ++w) t += lds[w];
    __syncthreads();
    return t;
}

__global__ __launch_bounds__(QW_THREADS) void absum_partials_kernel(const float* __restrict__ W, size_t total,
                                                                      size_t chunk, double* __restrict__ partials) {
    __shared__ double lds[QW_THREADS / 64];
    const size_t begin = (size_t)blockIdx.x * chunk;            // chunk is a multiple of 4
    size_t end = begin + chunk;
    if (end > total) end = total;
    double acc = 0.0;
    if (begin < end) {
        const size_t n4 = (end - begin) / 4;
        const float4* p4 = reinterpret_cast<const float4*>(W + begin);
        for (size_t i = threadIdx.x; i < n4; i += QW_THREADS) {
            float4 v = p4[i];
            acc += (double)fabsf(v.x);
            acc += (double)fabsf(v.y);
            acc += (double)fabsf(v.z);
            acc += (double)fabsf(v.w);
        }
        for (size_t i = begin + n4 * 4 + threadIdx.x; i < end; i += QW_THREADS) acc += (double)fabsf(W[i]);
    }
    double t = block_sum_fixed(acc, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

__global__ __launch_bounds__(QW_THREADS) void ternary_pack_kernel(const float* __restrict__ W, int N, int K, int nsb,
                                                                    size_t n_words, float eps,
                                                                    const double* __restrict__ partials, int n_partials,
                                                                    uint32_t* __restrict__ packed, float* __restrict__ beta_out,
                                                                    int8_t* __restrict__ codes_dbg, int* __restrict__ flag) {
    __shared__ double lds[QW_THREADS / 64];
    double acc = 0.0;
    for (int i = threadIdx.x; i < n_partials; i += QW_THREADS) acc += partials[i];
    const double total = block_sum_fixed(acc, lds);
    const float gamma = (float)(total / ((double)N * (double)K));
    const float beta = gamma + eps;
    const float tau = 0.5f * beta;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *beta_out = beta;
        *flag = isfinite(gamma) ? 0 : 1;
    }
    const size_t w = (size_t)blockIdx.x * QW_THREADS + threadIdx.x;
    if (w >= n_words) return;
    const int dd = (int)(w & 3);
    const int lane = (int)((w >> 2) & 63);
    const size_t blk = w >> 8;
    const int sb = (int)(blk % (size_t)nsb);
    const int nb = (int)(blk / (size_t)nsb);
    const int n = nb * 32 + (lane & 31);
    const int kbase = sb * 128 + dd * 32 + (lane >> 5) * 16;
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int k = kbase + i;
        int code = 0;
        if (n < N && k < K) {
            const float v = W[(size_t)n * K + k];
            code = (int)(v > tau) - (int)(v < -tau);
            if (codes_dbg) codes_dbg[(size_t)n * K + k] = (int8_t)code;
        }
        const int j = i >> 2, b = i & 3;
        word |= (uint32_t)(code + 1) << (2 * j + 8 * b);
    }
    packed[w] = word;
}

__global__ __launch_bounds__(QW_THREADS) void unpack_codes_kernel(const uint32_t* __restrict__ packed, int N, int K, int nsb,
                                                                    size_t n_words, int8_t* __restrict__ codes) {
    const size_t w = (size_t)blockIdx.x * QW_THREADS + threadIdx.x;
    if (w >= n_words) return;
    const int dd = (int)(w & 3);
    const int lane = (int)((w >> 2) & 63);
    const size_t blk = w >> 8;
    const int sb = (int)(blk % (size_t)nsb);
    const int nb = (int)(blk / (size_t)nsb);
    const int n = nb * 32 + (lane & 31);
    const int kbase = sb * 128 + dd * 32 + (lane >> 5) * 16;
    if (n >= N) return;
    const uint32_t word = packed[w];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int k = kbase + i;
        if (k < K) {
            const int j = i >> 2, b = i & 3;
            codes[(size_t)n * K + k] = (int8_t)((int)((word >> (2 * j + 8 * b)) & 3u) - 1);
        }
    }
}

}  // namespace

int quantize_partials_count(int N, int K) {
    const size_t total = (size_t)N * (size_t)K;
    size_t g = (total + 4095) / 4096;
    if (g > 1024) g = 1024;
    if (g < 1) g = 1;
    return (int)g;
}

int launch_quantize_weights(const float* W, int N, int K, float eps, uint32_t* packed, float* beta,
                            int8_t* codes_dbg, double* partials, int* flag, hipStream_t s) {
    const size_t total = (size_t)N * (size_t)K;
    const int g = quantize_partials_count(N, K);
    size_t chunk = (total + g - 1) / g;
    chunk = (chunk + 3) / 4 * 4;
    LaunchTimer tm(BRL_KC_QUANTIZE_WEIGHTS, s);
    hipLaunchKernelGGL(absum_partials_kernel, dim3(g), dim3(QW_THREADS), 0, s, W, total, chunk, partials);
    BRL_LAUNCH_CHECK("absum_partials_kernel");
    const int nsb = round_up(K, SBK) / SBK;
    const size_t n_words = (size_t)(round_up(N, NB) / NB) * nsb * 256;
    const size_t blocks = (n_words + QW_THREADS - 1) / QW_THREADS;
    hipLaunchKernelGGL(ternary_pack_kernel, dim3((unsigned)blocks), dim3(QW_THREADS), 0, s, W, N, K, nsb, n_words, eps,
                       partials, g, packed, beta, codes_dbg, flag);
    BRL_LAUNCH_CHECK("ternary_pack_kernel");
    return BRL_OK;
}

int launch_unpack_codes(const uint32_t* packed, int N, int K, int8_t* codes, hipStream_t s) {
    const int nsb = round_up(K, SBK) / SBK;
    const size_t n_words = (size_t)(round_up(N, NB) / NB) * nsb * 256;
    const size_t blocks = (n_words + QW_THREADS - 1) / QW_THREADS;
    LaunchTimer tm(BRL_KC_QUANTIZE_WEIGHTS, s);
    hipLaunchKernelGGL(unpack_codes_kernel, dim3((unsigned)blocks), dim3(QW_THREADS), 0, s, packed, N, K, nsb, n_words,
                       codes);
    BRL_LAUNCH_CHECK("unpack_codes_kernel");
    return BRL_OK;
}

}  // namespace brl
