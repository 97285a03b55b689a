// Per-token absmax int8 activation quantisation, with the producers that sit in
// front of it in the blocks fused in: RMSNorm / sub-layer norm, and the
// squared-ReLU GLU.  One wavefront owns one token row and keeps it in
// registers, so the row is read from HBM once: statistic, absmax and the
// quantised store all come from the same registers.
//
//   (GLU)   h_k = (max(g_k,0) * max(g_k,0)) * u_k
//   (norm)  r = fp32(1 / sqrt(mean_k x_k^2 + eps_n))  [fp64 statistic];  x_k <- (x_k * r) * gain_k
//   a = max(max_k |x_k|, eps);  s = 127 / a;  q_k = clamp(rne(x_k * s), -127, 127)
//
// Output goes to the tiled int8 layout the MFMA GEMM reads (see common.hpp),
// plus per-token a, a / 127 and sum_k q_k.
#include "common.hpp"

namespace brl {

namespace {

struct QK {
    const void* x;
    const float* gain;
    int x_dtype, glu;
    float eps_norm, eps_act;
    int M, Mp, K, Kp, nsb;
    int8_t* q_tiled;
    float* absmax;
    float* dscale;
    int32_t* sumq;
    int8_t* xq_rowmajor;
    float* absmax_tap;
};

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

template <int MAXV4>
__global__ __launch_bounds__(256) void act_quant_kernel(QK a) {
    // Workgroups with the same (blockIdx & 7) tend to share an XCD and its L2: give
    // the 8 workgroups that fill one 32-token block the same residue so that their
    // 16-byte pieces of each output line meet in one L2.
    const int w = blockIdx.x;
    const int xcd = w & 7, t = w >> 3;
    const int part = t & 7, mb = (t >> 3) * 8 + xcd;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = mb * 32 + part * 4 + wave;
    if (row >= a.Mp) return;
    const int K = a.K;
    const bool live = row < a.M;

    float4 v[MAXV4];
#pragma unroll
    for (int i = 0; i < MAXV4; ++i) {
        const int k = 4 * (lane + 64 * i);
        float4 e = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live && k < K) {
            if (a.glu) {
                const float* base = reinterpret_cast<const float*>(a.x) + (size_t)row * (2 * (size_t)K);
                const float4 g = *reinterpret_cast<const float4*>(base + k);
                const float4 u = *reinterpret_cast<const float4*>(base + K + k);
                float p;
                p = fmaxf(g.x, 0.f); e.x = (p * p) * u.x;
                p = fmaxf(g.y, 0.f); e.y = (p * p) * u.y;
                p = fmaxf(g.z, 0.f); e.z = (p * p) * u.z;
                p = fmaxf(g.w, 0.f); e.w = (p * p) * u.w;
            } else if (a.x_dtype == BRL_BF16) {
                const uint16_t* base = reinterpret_cast<const uint16_t*>(a.x) + (size_t)row * K;
                const uint2 raw = *reinterpret_cast<const uint2*>(base + k);
                e.x = bf16_to_f32((uint16_t)(raw.x & 0xffffu));
                e.y = bf16_to_f32((uint16_t)(raw.x >> 16));
                e.z = bf16_to_f32((uint16_t)(raw.y & 0xffffu));
                e.w = bf16_to_f32((uint16_t)(raw.y >> 16));
            } else {
                const float* base = reinterpret_cast<const float*>(a.x) + (size_t)row * K;
                e = *reinterpret_cast<const float4*>(base + k);
            }
        }
        v[i] = e;
    }

    if (a.gain) {
        double ss = 0.0;
#pragma unroll
        for (int i = 0; i < MAXV4; ++i) {
            ss += (double)v[i].x * (double)v[i].x;
            ss += (double)v[i].y * (double)v[i].y;
            ss += (double)v[i].z * (double)v[i].z;
            ss += (double)v[i].w * (double)v[i].w;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
        const double ms = ss / (double)K;
        const float r = (float)(1.0 / sqrt(ms + (double)a.eps_norm));
#pragma unroll
        for (int i = 0; i < MAXV4; ++i) {
            const int k = 4 * (lane + 64 * i);
            if (k < K) {
                const float4 g = *reinterpret_cast<const float4*>(a.gain + k);
                v[i].x = (v[i].x * r) * g.x;
                v[i].y = (v[i].y * r) * g.y;
                v[i].z = (v[i].z * r) * g.z;
                v[i].w = (v[i].w * r) * g.w;
            }
        }
    }

    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV4; ++i) {
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[i].x), fabsf(v[i].y)), fmaxf(fabsf(v[i].z), fabsf(v[i].w))));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    const float ac = fmaxf(amax, a.eps_act);
    const float s = 127.0f / ac;

    int sum = 0;
#pragma unroll
    for (int i = 0; i < MAXV4; ++i) {
        const int k = 4 * (lane + 64 * i);
        if (k < a.Kp) {
            int q0 = (int)fminf(fmaxf(rintf(v[i].x * s), -127.f), 127.f);
            int q1 = (int)fminf(fmaxf(rintf(v[i].y * s), -127.f), 127.f);
            int q2 = (int)fminf(fmaxf(rintf(v[i].z * s), -127.f), 127.f);
            int q3 = (int)fminf(fmaxf(rintf(v[i].w * s), -127.f), 127.f);
            sum += q0 + q1 + q2 + q3;
            const uint32_t word = (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) | ((uint32_t)(q2 & 0xff) << 16) |
                                  ((uint32_t)(q3 & 0xff) << 24);
            *reinterpret_cast<uint32_t*>(a.q_tiled + tiled_act_offset(row, k, a.nsb)) = word;
            if (a.xq_rowmajor && live && k < K) {
                *reinterpret_cast<uint32_t*>(a.xq_rowmajor + (size_t)row * K + k) = word;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) {
        a.absmax[row] = ac;
        a.dscale[row] = ac / 127.0f;
        a.sumq[row] = sum;
        if (a.absmax_tap && live) a.absmax_tap[row] = ac;
    }
}

}  // namespace

int launch_act_quant(const QuantArgs& in, const ActBuf& out, hipStream_t s) {
    QK a;
    a.x = in.x; a.gain = in.gain; a.x_dtype = in.x_dtype; a.glu = in.glu;
    a.eps_norm = in.eps_norm; a.eps_act = in.eps_act;
    a.M = in.M; a.Mp = round_up(in.M, NB); a.K = in.K; a.Kp = round_up(in.K, SBK); a.nsb = a.Kp / SBK;
    a.q_tiled = out.q; a.absmax = out.absmax; a.dscale = out.dscale; a.sumq = out.sumq;
    a.xq_rowmajor = in.xq_rowmajor; a.absmax_tap = in.absmax_tap;
    const int nmb = a.Mp / NB;
    const int grid = ((nmb + 7) / 8) * 64;
    const int v4 = a.Kp / 256 + ((a.Kp % 256) ? 1 : 0);
    LaunchTimer tm(BRL_KC_ACT_QUANT, s);
    if (v4 <= 4) {
        hipLaunchKernelGGL(act_quant_kernel<4>, dim3(grid), dim3(256), 0, s, a);
    } else if (v4 <= 12) {
        hipLaunchKernelGGL(act_quant_kernel<12>, dim3(grid), dim3(256), 0, s, a);
    } else if (v4 <= 28) {
        hipLaunchKernelGGL(act_quant_kernel<28>, dim3(grid), dim3(256), 0, s, a);
    } else if (v4 <= 36) {
        hipLaunchKernelGGL(act_quant_kernel<36>, dim3(grid), dim3(256), 0, s, a);
    } else {
        set_error("act_quant: K = %d exceeds the supported %d", in.K, MAX_K);
        return BRL_EINVAL;
    }
    BRL_LAUNCH_CHECK("act_quant_kernel");
    return BRL_OK;
}

}  // namespace brl
