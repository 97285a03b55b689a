// Per-token absmax int8 activation quantisation, with the RMSNorm / sub-layer
// norm that sits in front of it in the blocks fused in.  A token row is kept in
// registers, so it is read from HBM once: statistic, absmax and the quantised
// values all come from the same registers.
//
//   (norm)  r = fp32(1 / sqrt(mean_k x_k^2 + eps_n))  [fp64 statistic];  x_k <- (x_k * r) * gain_k
//   a = max(max_k |x_k|, eps);  s = 127 / a;  q_k = clamp(rne(x_k * s), -127, 127)
//
// Output goes to the tiled int8 layout the MFMA GEMM reads (see common.hpp),
// plus per-token a, a / 127 and sum_k q_k.  In that layout 16 consecutive k of
// one token are 16 bytes, and the same 16 k of the next token follow directly:
// a workgroup therefore takes 8 or 16 consecutive tokens at a time, parks their
// int8 rows in LDS and writes the tile out in runs of 128 or 256 bytes.
//
// Three kernels:
//   act_quant_wave_kernel  many tokens, rows up to 8704 wide: one wavefront per token
//   act_quant_kernel       many tokens, wider rows: four wavefronts per token, LDS reductions
//   act_quant_row_kernel   up to 1024 tokens (latency, not bandwidth): one workgroup per token
#include "common.hpp"

namespace brl {

namespace {

// The persistent kernel runs NWV wavefronts per workgroup (8: two workgroups share a compute unit and
// one computes while the other waits on memory or a barrier; 16: one workgroup per unit).

struct QK {
    const void* x;
    const float* gain;
    int x_dtype;
    float eps_norm, eps_act;
    int M, K, Kp, nsb;
    int8_t* q_tiled;
    float* absmax;
    float* dscale;
    int32_t* sumq;
    int8_t* xq_rowmajor;
    float* absmax_tap;
};

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// HV4: float4 chunks per lane; WPT: wavefronts per token.  The wavefronts of a token interleave
// their chunks (chunk c = WPT i + part covers k = 4 (lane + 64 c) .. + 3), so every load stays coalesced.
template <int HV4, int WPT>
__device__ inline void load_rows(const QK& a, int row, int lane, int part, float4 (&v)[HV4]) {
    const int K = a.K;
    const bool live = row < a.M;
#pragma unroll
    for (int i = 0; i < HV4; ++i) {
        const int k = 4 * (lane + 64 * (WPT * i + part));
        float4 e = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live && k < K) {
            if (a.x_dtype == BRL_BF16) {
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
}

// The NWV wavefronts of a workgroup take NWV / WPT tokens per round; GR / (NWV / WPT) rounds fill the
// group of GR tokens that is written out together.  A workgroup walks the groups g = blockIdx.x,
// + gridDim.x, ... and requests the rows of its next round before it works on the current one.
template <int HV4, int WPT, int GR, int NWV>
__global__ __launch_bounds__(NWV * 64) void act_quant_kernel(QK a) {
    constexpr int AQ_THREADS = NWV * 64;
    constexpr int TPR = NWV / WPT;         // tokens per round
    constexpr int RPG = GR / TPR;          // rounds per group of GR tokens that is written out together
    static_assert(GR == 8 || GR == 16 || GR == 32, "a group is 8, 16 or 32 tokens of one 32-token block of the tile");
    static_assert(GR % TPR == 0, "a group is a whole number of rounds");
    extern __shared__ __attribute__((aligned(16))) unsigned char rowbuf[];   // GR x (Kp + 16) bytes, then the gain
    __shared__ double red_ss[TPR][WPT];
    __shared__ float red_max[TPR][WPT];
    __shared__ int red_sum[TPR][WPT];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rl = wave / WPT, part = wave % WPT;
    const int K = a.K;
    const int stride = a.Kp + 16;          // the 16-byte skew keeps neighbouring rows on different LDS banks
    const int ngroups = (a.M + GR - 1) / GR;

    // (group, round) of the rows being worked on, of the next ones (already requested) and of the ones
    // after them (requested at the top of each round): two rounds of loads are in flight, so the memory
    // pipe does not drain while a round's reductions and barriers run
    int grp = blockIdx.x, rnd = 0;
    int grp1 = RPG == 1 ? grp + (int)gridDim.x : grp, rnd1 = RPG == 1 ? 0 : 1;
    float4 v[HV4], v1[HV4];
    load_rows<HV4, WPT>(a, grp * GR + rl, lane, part, v);
    if (grp1 < ngroups) load_rows<HV4, WPT>(a, grp1 * GR + rnd1 * TPR + rl, lane, part, v1);

    // the norm gain is the same for every token: parked in LDS once (read after the first barrier below)
    float* gain_lds = reinterpret_cast<float*>(rowbuf + (size_t)GR * stride);
    if (a.gain) {
        for (int k = 4 * threadIdx.x; k < K; k += 4 * AQ_THREADS)
            *reinterpret_cast<float4*>(gain_lds + k) = *reinterpret_cast<const float4*>(a.gain + k);
    }

    while (true) {
        const bool more = grp1 < ngroups;
        const int rnd2 = (rnd1 + 1) % RPG;
        const int grp2 = rnd2 == 0 ? grp1 + (int)gridDim.x : grp1;
        float4 v2[HV4];
        if (more && grp2 < ngroups) load_rows<HV4, WPT>(a, grp2 * GR + rnd2 * TPR + rl, lane, part, v2);

        const int row0 = grp * GR;
        const int row = row0 + rnd * TPR + rl;
        const bool live = row < a.M;

        if (a.gain) {
            double ss = 0.0;
#pragma unroll
            for (int i = 0; i < HV4; ++i) {
                ss += (double)v[i].x * (double)v[i].x;
                ss += (double)v[i].y * (double)v[i].y;
                ss += (double)v[i].z * (double)v[i].z;
                ss += (double)v[i].w * (double)v[i].w;
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
            if (lane == 0) red_ss[rl][part] = ss;
            __syncthreads();
            double tot = red_ss[rl][0];
#pragma unroll
            for (int w = 1; w < WPT; ++w) tot += red_ss[rl][w];
            const float r = (float)(1.0 / sqrt(tot / (double)K + (double)a.eps_norm));
#pragma unroll
            for (int i = 0; i < HV4; ++i) {
                const int k = 4 * (lane + 64 * (WPT * i + part));
                if (k < K) {
                    const float4 g = *reinterpret_cast<const float4*>(gain_lds + k);
                    v[i].x = (v[i].x * r) * g.x;
                    v[i].y = (v[i].y * r) * g.y;
                    v[i].z = (v[i].z * r) * g.z;
                    v[i].w = (v[i].w * r) * g.w;
                }
            }
        }

        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < HV4; ++i) {
            amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[i].x), fabsf(v[i].y)), fmaxf(fabsf(v[i].z), fabsf(v[i].w))));
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        if (lane == 0) red_max[rl][part] = amax;
        __syncthreads();
        float ac = a.eps_act;
#pragma unroll
        for (int w = 0; w < WPT; ++w) ac = fmaxf(ac, red_max[rl][w]);
        const float s = 127.0f / ac;

        int sum = 0;
        uint32_t* myrow = reinterpret_cast<uint32_t*>(rowbuf + (size_t)(rnd * TPR + rl) * stride);
#pragma unroll
        for (int i = 0; i < HV4; ++i) {
            const int k = 4 * (lane + 64 * (WPT * i + part));
            if (k < a.Kp) {
                int q0 = (int)fminf(fmaxf(rintf(v[i].x * s), -127.f), 127.f);
                int q1 = (int)fminf(fmaxf(rintf(v[i].y * s), -127.f), 127.f);
                int q2 = (int)fminf(fmaxf(rintf(v[i].z * s), -127.f), 127.f);
                int q3 = (int)fminf(fmaxf(rintf(v[i].w * s), -127.f), 127.f);
                sum += q0 + q1 + q2 + q3;
                const uint32_t word = (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) |
                                      ((uint32_t)(q2 & 0xff) << 16) | ((uint32_t)(q3 & 0xff) << 24);
                myrow[k >> 2] = word;
                if (a.xq_rowmajor && live && k < K)
                    *reinterpret_cast<uint32_t*>(a.xq_rowmajor + (size_t)row * K + k) = word;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane == 0) red_sum[rl][part] = sum;
        __syncthreads();
        if (lane == 0 && part == 0 && live) {
            int tot = red_sum[rl][0];
#pragma unroll
            for (int w = 1; w < WPT; ++w) tot += red_sum[rl][w];
            a.absmax[row] = ac;
            a.dscale[row] = ac / 127.0f;
            a.sumq[row] = tot;
            if (a.absmax_tap) a.absmax_tap[row] = ac;
        }

        if (rnd == RPG - 1) {
            // tiled write-out: thread (token t, chunk kc) moves the 16 bytes of k = 16 kc .. 16 kc + 15;
            // the GR tokens of one chunk are GR * 16 contiguous bytes of the tile (with GR = 32 a wavefront
            // writes whole 1 KB fragments and the workgroup one contiguous 32-token block)
            const int t = threadIdx.x % GR;
            const int mb = row0 >> 5, r0 = row0 & 31;
            const int nchunks = a.Kp >> 4;
            for (int kc = threadIdx.x / GR; kc < nchunks; kc += AQ_THREADS / GR) {
                const uint4 val = *reinterpret_cast<const uint4*>(rowbuf + (size_t)t * stride + 16 * kc);
                const int sb = kc >> 3, dd = (kc >> 1) & 3, hh = kc & 1;
                const size_t off = ((((size_t)mb * a.nsb + sb) * 4 + dd) * 64 + (hh * 32 + r0 + t)) * 16;
                *reinterpret_cast<uint4*>(a.q_tiled + off) = val;
            }
        }

        if (!more) break;
        // (the barriers of the next round order its LDS writes after the reads above)
#pragma unroll
        for (int i = 0; i < HV4; ++i) { v[i] = v1[i]; v1[i] = v2[i]; }
        grp = grp1; rnd = rnd1;
        grp1 = grp2; rnd1 = rnd2;
    }
}

// ---------------------------------------------------------------------------
// Many tokens, one wavefront per token.  A wavefront keeps its token's whole row in registers
// (NC float4 per lane), so the statistic, the absolute maximum and the code sum are reduced inside
// the wavefront with lane exchanges: no LDS reductions and no barrier per token, and the wavefronts
// of a workgroup drift apart instead of marching in step.  The int8 rows of a group of GR tokens
// are parked in LDS and written out together as whole pieces of the tiled layout (one barrier
// pair per group).  Loads are unconditional (row and column indices clamped, values masked
// afterwards).  Small workgroups, several per compute unit, no software prefetch: measured at
// 8192 x 2560, eight wavefronts and 16-token groups take 19.4 us against 26.7 us for sixteen
// wavefronts and 32-token groups (which start, load, and write out all over the chip in the same
// phase) and 21 - 24 us with the next row prefetched into registers (fewer resident wavefronts).
// ---------------------------------------------------------------------------
template <int NC, bool BF16>
__device__ inline void load_row_clamped(const QK& a, int row, int lane, float4 (&v)[NC]) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const int K = a.K;
    const int rc = min(row, a.M - 1);
    // The row index is the same for the whole wavefront: a scalar row base and one 32-bit byte offset per
    // chunk.  The offsets are rebuilt for every row from a value the compiler cannot see through; hoisted
    // out of the token loop they would occupy two registers per chunk next to the row itself.
    const __attribute__((address_space(1))) char* base =
        (const __attribute__((address_space(1))) char*)a.x + (size_t)rc * K * (BF16 ? 2 : 4);
    unsigned lane_k;
    asm volatile("v_lshlrev_b32 %0, 2, %1" : "=v"(lane_k) : "v"(lane));
    const unsigned k_last = (unsigned)(K - 4);                  // K % 4 == 0, K >= 4
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const unsigned k = min(lane_k + 256u * c, k_last);
        if constexpr (BF16) {
            const u32x2 raw = *(const __attribute__((address_space(1))) u32x2*)(base + k * 2u);
            v[c] = make_float4(bf16_to_f32((uint16_t)(raw.x & 0xffffu)), bf16_to_f32((uint16_t)(raw.x >> 16)),
                               bf16_to_f32((uint16_t)(raw.y & 0xffffu)), bf16_to_f32((uint16_t)(raw.y >> 16)));
        } else {
            const f32x4 r = *(const __attribute__((address_space(1))) f32x4*)(base + k * 4u);
            v[c] = make_float4(r.x, r.y, r.z, r.w);
        }
    }
}

template <int NC, int GR, int NWV, bool BF16>
__global__ __launch_bounds__(NWV * 64) void act_quant_wave_kernel(QK a) {
    constexpr int NT = NWV * 64;
    constexpr int TPW = GR / NWV;            // tokens of a group per wavefront
    static_assert(GR % NWV == 0 && (GR == 8 || GR == 16 || GR == 32), "a group is 8, 16 or 32 tokens, split evenly");
    extern __shared__ __attribute__((aligned(16))) unsigned char rowbuf[];   // GR x (Kp + 16) bytes, then the gain
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int K = a.K;
    const int stride = a.Kp + 16;
    const int ngroups = (a.M + GR - 1) / GR;
    const bool norm = a.gain != nullptr;

    float* gain_lds = reinterpret_cast<float*>(rowbuf + (size_t)GR * stride);
    if (norm) {
        for (int k = 4 * threadIdx.x; k < NC * 256; k += 4 * NT)
            *reinterpret_cast<float4*>(gain_lds + k) =
                k < K ? *reinterpret_cast<const float4*>(a.gain + k) : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    // flat walk over this wavefront's tokens: token j of the walk is token wave + (j % TPW) * NWV of group
    // blockIdx.x + (j / TPW) * gridDim.x
    int grp = blockIdx.x, tw = 0;
    float4 v[NC];
    if (grp < ngroups) load_row_clamped<NC, BF16>(a, grp * GR + wave, lane, v);
    __syncthreads();                               // the gain is in LDS

    while (grp < ngroups) {
        const int tw_n = tw + 1 == TPW ? 0 : tw + 1;
        const int grp_n = tw + 1 == TPW ? grp + (int)gridDim.x : grp;

        const int t = wave + tw * NWV;             // token inside the group
        const int row = grp * GR + t;
        const bool live = row < a.M;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const bool in = live && 4 * (lane + 64 * c) < K;
            v[c].x = in ? v[c].x : 0.f; v[c].y = in ? v[c].y : 0.f; v[c].z = in ? v[c].z : 0.f; v[c].w = in ? v[c].w : 0.f;
        }
        if (norm) {
            double ss = 0.0;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                ss += (double)v[c].x * (double)v[c].x;
                ss += (double)v[c].y * (double)v[c].y;
                ss += (double)v[c].z * (double)v[c].z;
                ss += (double)v[c].w * (double)v[c].w;
                __builtin_amdgcn_sched_barrier(0);      // one chunk at a time: the row itself fills the registers
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
            const float r = (float)(1.0 / sqrt(ss / (double)K + (double)a.eps_norm));
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 g = *reinterpret_cast<const float4*>(gain_lds + 4 * (lane + 64 * c));
                v[c].x = (v[c].x * r) * g.x;
                v[c].y = (v[c].y * r) * g.y;
                v[c].z = (v[c].z * r) * g.z;
                v[c].w = (v[c].w * r) * g.w;
                if (c % 2 == 1) __builtin_amdgcn_sched_barrier(0);   // two gain reads in flight at a time
            }
        }
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c)
            amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[c].x), fabsf(v[c].y)), fmaxf(fabsf(v[c].z), fabsf(v[c].w))));
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        const float ac = fmaxf(amax, a.eps_act);
        const float sc = 127.0f / ac;

        int sum = 0;
        uint32_t* myrow = reinterpret_cast<uint32_t*>(rowbuf + (size_t)t * stride);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int k = 4 * (lane + 64 * c);
            const int q0 = (int)fminf(fmaxf(rintf(v[c].x * sc), -127.f), 127.f);
            const int q1 = (int)fminf(fmaxf(rintf(v[c].y * sc), -127.f), 127.f);
            const int q2 = (int)fminf(fmaxf(rintf(v[c].z * sc), -127.f), 127.f);
            const int q3 = (int)fminf(fmaxf(rintf(v[c].w * sc), -127.f), 127.f);
            sum += q0 + q1 + q2 + q3;
            const uint32_t word = (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) | ((uint32_t)(q2 & 0xff) << 16) |
                                  ((uint32_t)(q3 & 0xff) << 24);
            if (k < a.Kp) myrow[k >> 2] = word;
            if (a.xq_rowmajor && live && k < K) *reinterpret_cast<uint32_t*>(a.xq_rowmajor + (size_t)row * K + k) = word;
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane == 0 && live) {
            a.absmax[row] = ac;
            a.dscale[row] = ac / 127.0f;
            a.sumq[row] = sum;
            if (a.absmax_tap) a.absmax_tap[row] = ac;
        }

        if (tw + 1 == TPW) {
            // the group is complete once every wavefront has parked its tokens
            __syncthreads();
            const int tt = threadIdx.x % GR;
            const int row0 = grp * GR;
            const int mb = row0 >> 5, r0 = row0 & 31;
            const int nchunks = a.Kp >> 4;
            for (int kc = threadIdx.x / GR; kc < nchunks; kc += NT / GR) {
                const uint4 val = *reinterpret_cast<const uint4*>(rowbuf + (size_t)tt * stride + 16 * kc);
                const int sb = kc >> 3, dd = (kc >> 1) & 3, hh = kc & 1;
                const size_t off = ((((size_t)mb * a.nsb + sb) * 4 + dd) * 64 + (hh * 32 + r0 + tt)) * 16;
                *reinterpret_cast<uint4*>(a.q_tiled + off) = val;
            }
            __syncthreads();                       // before the next group's tokens overwrite the rows
        }
        if (grp_n < ngroups) load_row_clamped<NC, BF16>(a, grp_n * GR + wave + tw_n * NWV, lane, v);
        grp = grp_n;
        tw = tw_n;
    }
}

// Few tokens: one workgroup of NWV wavefronts per token, everything in flight at once (row and
// gain requested together), two barriers on the way to the int8 row, and the 16-byte pieces of the
// tiled layout assembled from four neighbouring lanes: no LDS staging, nothing persistent.  The
// time of such a launch is latency, not bandwidth.
template <int HV4, int NWV>
__global__ __launch_bounds__(NWV * 64) void act_quant_row_kernel(QK a) {
    __shared__ double red_ss[NWV];
    __shared__ float red_max[NWV];
    __shared__ int red_sum[NWV];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x;
    const int K = a.K;
    float4 v[HV4], g[HV4];
    load_rows<HV4, NWV>(a, row, lane, wave, v);
    if (a.gain) {
#pragma unroll
        for (int i = 0; i < HV4; ++i) {
            const int k = 4 * (lane + 64 * (NWV * i + wave));
            g[i] = k < K ? *reinterpret_cast<const float4*>(a.gain + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        double ss = 0.0;
#pragma unroll
        for (int i = 0; i < HV4; ++i) {
            ss += (double)v[i].x * (double)v[i].x;
            ss += (double)v[i].y * (double)v[i].y;
            ss += (double)v[i].z * (double)v[i].z;
            ss += (double)v[i].w * (double)v[i].w;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
        if (lane == 0) red_ss[wave] = ss;
        __syncthreads();
        double tot = red_ss[0];
#pragma unroll
        for (int w = 1; w < NWV; ++w) tot += red_ss[w];
        const float r = (float)(1.0 / sqrt(tot / (double)K + (double)a.eps_norm));
#pragma unroll
        for (int i = 0; i < HV4; ++i) {
            v[i].x = (v[i].x * r) * g[i].x;
            v[i].y = (v[i].y * r) * g[i].y;
            v[i].z = (v[i].z * r) * g[i].z;
            v[i].w = (v[i].w * r) * g[i].w;
        }
    }
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < HV4; ++i)
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[i].x), fabsf(v[i].y)), fmaxf(fabsf(v[i].z), fabsf(v[i].w))));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if (lane == 0) red_max[wave] = amax;
    __syncthreads();
    float ac = a.eps_act;
#pragma unroll
    for (int w = 0; w < NWV; ++w) ac = fmaxf(ac, red_max[w]);
    const float s = 127.0f / ac;

    int sum = 0;
    const int mb = row >> 5, r0 = row & 31;
#pragma unroll
    for (int i = 0; i < HV4; ++i) {
        const int k = 4 * (lane + 64 * (NWV * i + wave));
        const int q0 = (int)fminf(fmaxf(rintf(v[i].x * s), -127.f), 127.f);
        const int q1 = (int)fminf(fmaxf(rintf(v[i].y * s), -127.f), 127.f);
        const int q2 = (int)fminf(fmaxf(rintf(v[i].z * s), -127.f), 127.f);
        const int q3 = (int)fminf(fmaxf(rintf(v[i].w * s), -127.f), 127.f);
        sum += q0 + q1 + q2 + q3;
        const uint32_t word = (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) | ((uint32_t)(q2 & 0xff) << 16) |
                              ((uint32_t)(q3 & 0xff) << 24);
        if (a.xq_rowmajor && k < K) *reinterpret_cast<uint32_t*>(a.xq_rowmajor + (size_t)row * K + k) = word;
        // lanes 4 j .. 4 j + 3 hold 16 consecutive k: lane 4 j writes them as one piece of the tile
        uint4 piece;
        piece.x = word;
        piece.y = __shfl_down(word, 1, 64);
        piece.z = __shfl_down(word, 2, 64);
        piece.w = __shfl_down(word, 3, 64);
        if ((lane & 3) == 0 && k < a.Kp) {
            const int kc = k >> 4;
            const int sb = kc >> 3, dd = (kc >> 1) & 3, hh = kc & 1;
            const size_t off = ((((size_t)mb * a.nsb + sb) * 4 + dd) * 64 + (hh * 32 + r0)) * 16;
            *reinterpret_cast<uint4*>(a.q_tiled + off) = piece;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) red_sum[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = red_sum[0];
#pragma unroll
        for (int w = 1; w < NWV; ++w) tot += red_sum[w];
        a.absmax[row] = ac;
        a.dscale[row] = ac / 127.0f;
        a.sumq[row] = tot;
        if (a.absmax_tap) a.absmax_tap[row] = ac;
    }
}

template <int HV4, int NWV>
int launch_rows(const QK& a, hipStream_t s) {
    hipLaunchKernelGGL((act_quant_row_kernel<HV4, NWV>), dim3(a.M), dim3(NWV * 64), 0, s, a);
    return BRL_OK;
}

template <int HV4, int WPT, int GR, int NWV>
int launch_one(const QK& a, hipStream_t s) {
    constexpr int AQ_THREADS = NWV * 64;
    const int ngroups = (a.M + GR - 1) / GR;
    const size_t lds = (size_t)GR * (a.Kp + 16) + (a.gain ? (size_t)a.Kp * 4 : 0);
    constexpr size_t max_lds = (size_t)GR * (HV4 * WPT * 256 + 16) + (size_t)HV4 * WPT * 256 * 4;
    static_assert(max_lds <= 160 * 1024, "the rows of a group and the gain fit the LDS of a compute unit");
    static const int slots = [] {    // workgroups the device holds at once; initialised once, thread-safe
        int dev = 0, cus = 0, per_cu = 0;
        hipError_t e = hipSuccess;
        if (max_lds > 65536)         // more than the default 64 KB of dynamic LDS
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&act_quant_kernel<HV4, WPT, GR, NWV>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_lds);
        if (e != hipSuccess || hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, act_quant_kernel<HV4, WPT, GR, NWV>, AQ_THREADS, max_lds) !=
                hipSuccess ||
            cus <= 0 || per_cu <= 0) {
            (void)hipGetLastError();
            return -1;
        }
        return cus * per_cu;
    }();
    if (slots <= 0) {
        set_error("act_quant: the device cannot hold a workgroup with %zu bytes of LDS", max_lds);
        return BRL_EHIP;
    }
    const int grid = ngroups < slots ? ngroups : slots;
    hipLaunchKernelGGL((act_quant_kernel<HV4, WPT, GR, NWV>), dim3(grid), dim3(AQ_THREADS), lds, s, a);
    return BRL_OK;
}

template <int NC, int GR, int NWV>
int launch_wave(const QK& a, hipStream_t s) {
    constexpr int NT = NWV * 64;
    constexpr size_t lds = (size_t)GR * (NC * 256 + 16) + (size_t)NC * 256 * 4;      // sized for the widest row of this NC
    static_assert(lds <= 160 * 1024, "the rows of a group and the gain fit the LDS of a compute unit");
    const int ngroups = (a.M + GR - 1) / GR;
    const bool bf16 = a.x_dtype == BRL_BF16;
    static const int slots = [] {        // workgroups the device holds at once (the two input types use the same resources)
        int dev = 0, cus = 0, per_cu = 0;
        hipError_t e = hipSuccess;
        if (lds > 65536) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&act_quant_wave_kernel<NC, GR, NWV, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e == hipSuccess)
                e = hipFuncSetAttribute(reinterpret_cast<const void*>(&act_quant_wave_kernel<NC, GR, NWV, true>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        }
        if (e != hipSuccess || hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, act_quant_wave_kernel<NC, GR, NWV, false>, NT, lds) !=
                hipSuccess ||
            cus <= 0 || per_cu <= 0) {
            (void)hipGetLastError();
            return -1;
        }
        return cus * per_cu;
    }();
    if (slots <= 0) {
        set_error("act_quant: the device cannot hold a workgroup with %zu bytes of LDS", lds);
        return BRL_EHIP;
    }
    const int grid = ngroups < slots ? ngroups : slots;
    if (bf16)
        hipLaunchKernelGGL((act_quant_wave_kernel<NC, GR, NWV, true>), dim3(grid), dim3(NT), lds, s, a);
    else
        hipLaunchKernelGGL((act_quant_wave_kernel<NC, GR, NWV, false>), dim3(grid), dim3(NT), lds, s, a);
    return BRL_OK;
}

}  // namespace

int launch_act_quant(const QuantArgs& in, const ActBuf& out, hipStream_t s) {
    QK a;
    a.x = in.x; a.gain = in.gain; a.x_dtype = in.x_dtype;
    a.eps_norm = in.eps_norm; a.eps_act = in.eps_act;
    a.M = in.M; a.K = in.K; a.Kp = round_up(in.K, SBK); a.nsb = a.Kp / SBK;
    a.q_tiled = out.q; a.absmax = out.absmax; a.dscale = out.dscale; a.sumq = out.sumq;
    a.xq_rowmajor = in.xq_rowmajor; a.absmax_tap = in.absmax_tap;
    // Up to 1024 tokens: one workgroup per token (latency bound).  Beyond: persistent workgroups; their
    // registers hold the current and the next row share of a lane, at most 2 x 9 float4.
    LaunchTimer tm(BRL_KC_ACT_QUANT, s);
    const bool rows = in.M <= 1024;      // measured crossover: about 1500 tokens at both layer widths
    int rc;
    if (a.Kp > MAX_K) {
        set_error("act_quant: K = %d exceeds the supported %d", in.K, MAX_K);
        return BRL_EINVAL;
    }
    // Many tokens: one wavefront per token; NC float4 per lane hold the row (NC * 256 >= Kp), and as many
    // tokens of a 32-token block are written out together as the LDS holds next to the gain.
    // A few thousand tokens make too few 16-token groups to fill the chip: groups of 8 then (measured: 2560 wide,
    // 1536 / 2048 / 6144 tokens 8.3 / 9.1 / 15.9 us against 10.9 / 11.5 / 17.2; 6912 wide, 1536 / 2048 tokens
    // 17.3 / 19.6 us against 21.4 / 22.8, and the other way round from 3072 tokens on).
    const bool few_narrow = in.M <= 6144, few_wide = in.M <= 2048;
    if (a.Kp <= 1024) {
        rc = rows ? launch_rows<1, 4>(a, s) : launch_wave<4, 16, 8>(a, s);
    } else if (a.Kp <= 2560) {
        rc = rows ? launch_rows<3, 4>(a, s) : few_narrow ? launch_wave<10, 8, 8>(a, s) : launch_wave<10, 16, 8>(a, s);
    } else if (a.Kp <= 3328) {
        rc = rows ? launch_rows<4, 4>(a, s) : few_narrow ? launch_wave<13, 8, 8>(a, s) : launch_wave<13, 16, 8>(a, s);
    } else if (a.Kp <= 4608) {
        rc = rows ? launch_rows<3, 6>(a, s) : few_wide ? launch_wave<18, 8, 8>(a, s) : launch_wave<18, 16, 8>(a, s);
    } else if (a.Kp <= 6912) {
        rc = rows ? launch_rows<4, 7>(a, s) : few_wide ? launch_wave<27, 8, 8>(a, s) : launch_wave<27, 16, 8>(a, s);
    } else if (a.Kp <= 8704) {
        rc = rows ? launch_rows<4, 9>(a, s) : launch_wave<34, 8, 8>(a, s);
    } else {
        // the widest rows do not fit one wavefront's registers: four wavefronts per token, LDS reductions
        rc = rows ? launch_rows<4, 9>(a, s) : launch_one<9, 4, 8, 16>(a, s);
    }
    if (rc != BRL_OK) return rc;
    BRL_LAUNCH_CHECK("act_quant_kernel");
    return BRL_OK;
}

}  // namespace brl
