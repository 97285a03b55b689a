// Per-tensor absmax int8 weights for the higher-precision critic backbone
// (paper Sec. 5.3, hybrid-precision rows; the quantiser mirrors the per-token
// activation quantiser on the whole matrix):
//
//   a = max(max |W|, eps);  s = qmax / a;  code = clamp(rne(w * s), -qmax, qmax);  scale = a / qmax
//   (qmax = 127: the int8 critic; qmax = 7: the grid of the int4 critic, still one code per byte)
//
// The codes are written in the int8 MFMA fragment layout of the activations
// (32 rows x 128 columns = four 1 KB fragments, lane (n & 31) + 32 ((k >> 4) & 1)
// owning 16 consecutive k), padded with zeros, so the GEMM stages them as they are.
// Two launches: per-block maxima, then a pack kernel in which every block
// reduces the partial maxima again (a maximum does not depend on the order).
#include "common.hpp"

namespace brl {

namespace {

constexpr int W8_THREADS = 256;

__device__ inline float block_max(float v, float* lds) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < W8_THREADS / 64; ++w) t = fmaxf(t, lds[w]);
    __syncthreads();
    return t;
}

// fmaxf drops NaN operands, so non-finite inputs are tracked separately: they come out as +inf
__device__ inline float abs_or_inf(float v) { return isfinite(v) ? fabsf(v) : INFINITY; }

__global__ __launch_bounds__(W8_THREADS) void absmax_partials_kernel(const float* __restrict__ W, size_t total, size_t chunk,
                                                                      float* __restrict__ partials) {
    __shared__ float lds[W8_THREADS / 64];
    const size_t begin = (size_t)blockIdx.x * chunk;            // chunk is a multiple of 4
    size_t end = begin + chunk;
    if (end > total) end = total;
    float m = 0.f;
    if (begin < end) {
        const size_t n4 = (end - begin) / 4;
        const float4* p4 = reinterpret_cast<const float4*>(W + begin);
        for (size_t i = threadIdx.x; i < n4; i += W8_THREADS) {
            const float4 v = p4[i];
            m = fmaxf(m, fmaxf(fmaxf(abs_or_inf(v.x), abs_or_inf(v.y)), fmaxf(abs_or_inf(v.z), abs_or_inf(v.w))));
        }
        for (size_t i = begin + n4 * 4 + threadIdx.x; i < end; i += W8_THREADS) m = fmaxf(m, abs_or_inf(W[i]));
    }
    const float t = block_max(m, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

// one 16-byte lane slot of the tiled layout per thread
__global__ __launch_bounds__(W8_THREADS) void int8_pack_kernel(const float* __restrict__ W, int N, int K, int nsb,
                                                                size_t n_slots, float eps, float qmax, const float* __restrict__ partials,
                                                                int n_partials, uint4* __restrict__ packed,
                                                                float* __restrict__ scale_out, int8_t* __restrict__ codes_dbg,
                                                                int* __restrict__ flag) {
    __shared__ float lds[W8_THREADS / 64];
    float m = 0.f;
    for (int i = threadIdx.x; i < n_partials; i += W8_THREADS) m = fmaxf(m, partials[i]);
    const float a = block_max(m, lds);
    const float ac = fmaxf(a, eps);
    const float s = qmax / ac;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *scale_out = ac / qmax;
        *flag = isfinite(a) ? 0 : 1;
    }
    const size_t u = (size_t)blockIdx.x * W8_THREADS + threadIdx.x;
    if (u >= n_slots) return;
    const int lane = (int)(u & 63);
    const int dd = (int)((u >> 6) & 3);
    const size_t blk = u >> 8;
    const int sb = (int)(blk % (size_t)nsb);
    const int nb = (int)(blk / (size_t)nsb);
    const int n = nb * 32 + (lane & 31);
    const int kbase = sb * 128 + dd * 32 + (lane >> 5) * 16;
    uint32_t word[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int k = kbase + i;
        int code = 0;
        if (n < N && k < K) {
            const float v = W[(size_t)n * K + k];
            code = (int)fminf(fmaxf(rintf(v * s), -qmax), qmax);
            if (codes_dbg) codes_dbg[(size_t)n * K + k] = (int8_t)code;
        }
        word[i >> 2] |= ((uint32_t)code & 0xffu) << (8 * (i & 3));
    }
    packed[u] = make_uint4(word[0], word[1], word[2], word[3]);
}

__global__ __launch_bounds__(W8_THREADS) void int8_unpack_kernel(const uint4* __restrict__ packed, int N, int K, int nsb,
                                                                  size_t n_slots, int8_t* __restrict__ codes) {
    const size_t u = (size_t)blockIdx.x * W8_THREADS + threadIdx.x;
    if (u >= n_slots) return;
    const int lane = (int)(u & 63);
    const int dd = (int)((u >> 6) & 3);
    const size_t blk = u >> 8;
    const int sb = (int)(blk % (size_t)nsb);
    const int nb = (int)(blk / (size_t)nsb);
    const int n = nb * 32 + (lane & 31);
    const int kbase = sb * 128 + dd * 32 + (lane >> 5) * 16;
    if (n >= N) return;
    const uint4 q = packed[u];
    const uint32_t word[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int k = kbase + i;
        if (k < K) codes[(size_t)n * K + k] = (int8_t)((word[i >> 2] >> (8 * (i & 3))) & 0xffu);
    }
}

}  // namespace

int launch_quantize_weights_int8(const float* W, int N, int K, float eps, int qmax, int8_t* packed, float* scale,
                                 int8_t* codes_dbg, float* partials, int* flag, hipStream_t s) {
    const size_t total = (size_t)N * (size_t)K;
    const int g = quantize_partials_count(N, K);
    size_t chunk = (total + g - 1) / g;
    chunk = (chunk + 3) / 4 * 4;
    LaunchTimer tm(BRL_KC_QUANTIZE_WEIGHTS, s);
    hipLaunchKernelGGL(absmax_partials_kernel, dim3(g), dim3(W8_THREADS), 0, s, W, total, chunk, partials);
    BRL_LAUNCH_CHECK("absmax_partials_kernel");
    const int nsb = round_up(K, SBK) / SBK;
    const size_t n_slots = (size_t)(round_up(N, NB) / NB) * nsb * 256;
    const size_t blocks = (n_slots + W8_THREADS - 1) / W8_THREADS;
    hipLaunchKernelGGL(int8_pack_kernel, dim3((unsigned)blocks), dim3(W8_THREADS), 0, s, W, N, K, nsb, n_slots, eps, (float)qmax, partials,
                       g, reinterpret_cast<uint4*>(packed), scale, codes_dbg, flag);
    BRL_LAUNCH_CHECK("int8_pack_kernel");
    return BRL_OK;
}

int launch_unpack_codes_int8(const int8_t* packed, int N, int K, int8_t* codes, hipStream_t s) {
    const int nsb = round_up(K, SBK) / SBK;
    const size_t n_slots = (size_t)(round_up(N, NB) / NB) * nsb * 256;
    const size_t blocks = (n_slots + W8_THREADS - 1) / W8_THREADS;
    LaunchTimer tm(BRL_KC_QUANTIZE_WEIGHTS, s);
    hipLaunchKernelGGL(int8_unpack_kernel, dim3((unsigned)blocks), dim3(W8_THREADS), 0, s,
                       reinterpret_cast<const uint4*>(packed), N, K, nsb, n_slots, codes);
    BRL_LAUNCH_CHECK("int8_unpack_kernel");
    return BRL_OK;
}

}  // namespace brl
