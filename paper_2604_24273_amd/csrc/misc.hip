// Small kernels around the BitLinear core: embedding gather, final RMSNorm +
// mean-pool (paper Sec. 3.1, Eq. 3: h_t), the fp32 MLP heads.
#include "common.hpp"

namespace brl {

namespace {

// x[m, :] = widen(E[clamp(ids[m]), :]); eight bf16 per thread
__global__ void embed_kernel(const uint16_t* __restrict__ table, const int32_t* __restrict__ ids, int M, int d,
                             int vocab, float* __restrict__ x) {
    const int per_row = d / 8;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * per_row) return;
    const int m = (int)(idx / per_row), c = (int)(idx % per_row) * 8;
    int id = ids[m];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const uint4 raw = *reinterpret_cast<const uint4*>(table + (size_t)id * d + c);
    float4 lo, hi;
    lo.x = __uint_as_float(raw.x << 16); lo.y = __uint_as_float(raw.x & 0xffff0000u);
    lo.z = __uint_as_float(raw.y << 16); lo.w = __uint_as_float(raw.y & 0xffff0000u);
    hi.x = __uint_as_float(raw.z << 16); hi.y = __uint_as_float(raw.z & 0xffff0000u);
    hi.z = __uint_as_float(raw.w << 16); hi.w = __uint_as_float(raw.w & 0xffff0000u);
    float* o = x + (size_t)m * d + c;
    *reinterpret_cast<float4*>(o) = lo;
    *reinterpret_cast<float4*>(o + 4) = hi;
}

// rinv[m] = fp32(1 / sqrt(mean_k x[m,k]^2 + eps)), statistic in fp64; one wavefront per row
__global__ __launch_bounds__(256) void row_rinv_kernel(const float* __restrict__ x, int M, int d, float eps,
                                                        float* __restrict__ rinv) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    const float* p = x + (size_t)row * d;
    double ss = 0.0;
    for (int k = 4 * lane; k < d; k += 256) {
        const float4 v = *reinterpret_cast<const float4*>(p + k);
        ss += (double)v.x * (double)v.x;
        ss += (double)v.y * (double)v.y;
        ss += (double)v.z * (double)v.z;
        ss += (double)v.w * (double)v.w;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) rinv[row] = (float)(1.0 / sqrt(ss / (double)d + (double)eps));
}

// h[b, c] = fp32( sum_{s < len_b} fp64((x[b,s,c] * rinv[b,s]) * g[c]) / len_b ), positions in order
__global__ void pool_kernel(const float* __restrict__ x, const float* __restrict__ rinv, const float* __restrict__ gain,
                            int B, int S, int d, const int32_t* __restrict__ lengths, SeqMap sm, float* __restrict__ h) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)B * d) return;
    const int b = (int)(idx / d), c = (int)(idx % d);
    int len = sm.cu ? seq_len(sm, b, S) : (lengths ? lengths[b] : S);
    len = len < 1 ? 1 : (len > S ? S : len);
    const size_t m0 = (size_t)seq_row0(sm, b, S);
    const float g = gain[c];
    double acc = 0.0;
    for (int s = 0; s < len; ++s) {
        const size_t m = m0 + s;
        const float v = (x[m * d + c] * rinv[m]) * g;
        acc += (double)v;
    }
    h[idx] = (float)(acc / (double)len);
}

// out[b, o] = act(sum_i W[o, i] * in[b, i] + bias[o]), fp64 accumulation; one wavefront per output
__global__ __launch_bounds__(256) void mlp_layer_kernel(const double* __restrict__ in64, const float* __restrict__ in32,
                                                         const float* __restrict__ W, const float* __restrict__ bias,
                                                         int B, int in_dim, int out_dim, int act, int last,
                                                         double* __restrict__ out64, float* __restrict__ out32) {
    const size_t wid = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (wid >= (size_t)B * out_dim) return;
    const int b = (int)(wid / out_dim), o = (int)(wid % out_dim);
    const float* w = W + (size_t)o * in_dim;
    double acc = 0.0;
    for (int i = lane; i < in_dim; i += 64) {
        const double v = in64 ? in64[(size_t)b * in_dim + i] : (double)in32[(size_t)b * in_dim + i];
        acc += (double)w[i] * v;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
        double z = acc + (double)bias[o];
        if (!last) z = (act == BRL_ACT_RELU) ? fmax(z, 0.0) : tanh(z);
        if (last) out32[(size_t)b * out_dim + o] = (float)z;
        else out64[(size_t)b * out_dim + o] = z;
    }
}

// The same layer for every member of an ensemble of equally shaped heads in one launch: member e
// reads its own parameters and (after the first layer) its own activations.
__global__ __launch_bounds__(256) void ensemble_layer_kernel(EnsembleLayer a) {
    const size_t wid = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const size_t per_member = (size_t)a.B * a.out_dim;
    if (wid >= per_member * a.n_members) return;
    const int e = (int)(wid / per_member);
    const size_t r = wid % per_member;
    const int b = (int)(r / a.out_dim), o = (int)(r % a.out_dim);
    const float* w = a.W[e] + (size_t)o * a.in_dim;
    const double* in64 = a.in64 ? a.in64 + ((size_t)e * a.B + b) * a.in_dim : nullptr;
    const float* in32 = a.in32 + (size_t)b * a.in_dim;
    double acc = 0.0;
    for (int i = lane; i < a.in_dim; i += 64) {
        const double v = in64 ? in64[i] : (double)in32[i];
        acc += (double)w[i] * v;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
        double z = acc + (double)a.bias[e][o];
        if (!a.last) z = (a.act == BRL_ACT_RELU) ? fmax(z, 0.0) : tanh(z);
        if (a.last) a.out32[(size_t)e * a.B + b] = (float)z;            // out_dim == 1 on the last layer
        else a.out64[((size_t)e * a.B + b) * a.out_dim + o] = z;
    }
}

// mean[b] = (sum over members, in member order, of each[e][b]) / n in fp64, rounded once
__global__ __launch_bounds__(256) void ensemble_mean_kernel(const float* __restrict__ each, int n, int B,
                                                             float* __restrict__ mean) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    double t = 0.0;
    for (int e = 0; e < n; ++e) t += (double)each[(size_t)e * B + b];
    mean[b] = (float)(t / (double)n);
}

}  // namespace

int launch_ensemble_layer(const EnsembleLayer& a, hipStream_t s) {
    const size_t waves = (size_t)a.n_members * a.B * a.out_dim;
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(ensemble_layer_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, a);
    BRL_LAUNCH_CHECK("ensemble_layer_kernel");
    return BRL_OK;
}

int launch_ensemble_mean(const float* each, int n, int B, float* mean, hipStream_t s) {
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(ensemble_mean_kernel, dim3((B + 255) / 256), dim3(256), 0, s, each, n, B, mean);
    BRL_LAUNCH_CHECK("ensemble_mean_kernel");
    return BRL_OK;
}

int launch_embed(const uint16_t* table, const int32_t* ids, int M, int d, int vocab, float* x, hipStream_t s) {
    const size_t n = (size_t)M * (d / 8);
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(embed_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, table, ids, M, d, vocab, x);
    BRL_LAUNCH_CHECK("embed_kernel");
    return BRL_OK;
}

int launch_final_pool(const float* x, const float* gain, int B, int S, int M, int d, const int32_t* lengths,
                      const SeqMap& sm, float eps_norm, float* rinv, float* h, hipStream_t s) {
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(row_rinv_kernel, dim3((M + 3) / 4), dim3(256), 0, s, x, M, d, eps_norm, rinv);
    BRL_LAUNCH_CHECK("row_rinv_kernel");
    const size_t n = (size_t)B * d;
    hipLaunchKernelGGL(pool_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, rinv, gain, B, S, d, lengths, sm, h);
    BRL_LAUNCH_CHECK("pool_kernel");
    return BRL_OK;
}

int launch_mlp_layer(const double* in64, const float* in32, const float* W, const float* b, int B, int in_dim,
                     int out_dim, int act, double* out64, float* out32, hipStream_t s) {
    const size_t waves = (size_t)B * out_dim;
    const int last = out32 != nullptr;
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(mlp_layer_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, in64, in32, W, b, B, in_dim,
                       out_dim, act, last, out64, out32);
    BRL_LAUNCH_CHECK("mlp_layer_kernel");
    return BRL_OK;
}

}  // namespace brl
