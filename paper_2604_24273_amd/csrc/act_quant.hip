// Per-token absmax int8 activation quantisation, with the RMSNorm / sub-layer
// norm that sits in front of it in the blocks fused in.  A token row is kept in the
// registers of the 2 or 4 wavefronts that share it, so it is read from HBM once:
// statistic, absmax and the quantised values all come from the same registers.
//
//   (norm)  r = fp32(1 / sqrt(mean_k x_k^2 + eps_n))  [fp64 statistic];  x_k <- (x_k * r) * gain_k
//   a = max(max_k |x_k|, eps);  s = 127 / a;  q_k = clamp(rne(x_k * s), -127, 127)
//
// Output goes to the tiled int8 layout the MFMA GEMM reads (see common.hpp),
// plus per-token a, a / 127 and sum_k q_k.  In that layout 16 consecutive k of
// one token are 16 bytes, and the same 16 k of the next token follow directly:
// a workgroup therefore takes 8 consecutive tokens at a time, parks their int8 rows
// in LDS and writes the tile out in full 128-byte runs.  The workgroups are
// persistent and request the rows of their next tokens before working on the
// current ones, so that HBM stays busy through the reductions and the write-out.
// With at most 1024 tokens the time is latency, not bandwidth: act_quant_row_kernel takes one
// token per workgroup instead.
#include "common.hpp"

namespace brl {

namespace {

constexpr int AQ_ROWS = 8;                 // tokens per workgroup
constexpr int AQ_THREADS = AQ_ROWS * 128;  // two wavefronts per token: each keeps half of the row in registers

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

// The 16 wavefronts of a workgroup take 16 / WPT tokens per round; WPT / 2 rounds fill the 8-token
// group that is written out together.  A workgroup walks the groups g = blockIdx.x, + gridDim.x, ...
// and requests the rows of its next round before it works on the current one.
template <int HV4, int WPT, int GR>
__global__ __launch_bounds__(AQ_THREADS) void act_quant_kernel(QK a) {
    constexpr int TPR = 16 / WPT;          // tokens per round
    constexpr int RPG = GR / TPR;          // rounds per group of GR tokens that is written out together
    static_assert(GR == 8, "groups of 8 tokens: 128-byte runs of the tile");
    static_assert(GR % TPR == 0, "a group is a whole number of rounds");
    extern __shared__ __attribute__((aligned(16))) unsigned char rowbuf[];   // AQ_ROWS x (Kp + 16) bytes, then the gain
    __shared__ double red_ss[TPR][WPT];
    __shared__ float red_max[TPR][WPT];
    __shared__ int red_sum[TPR][WPT];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rl = wave / WPT, part = wave % WPT;
    const int K = a.K;
    const int stride = a.Kp + 16;          // the 16-byte skew keeps the 8 rows on different LDS banks
    const int ngroups = (a.M + GR - 1) / GR;

    int grp = blockIdx.x, rnd = 0;
    float4 v[HV4];
    load_rows<HV4, WPT>(a, grp * GR + rl, lane, part, v);

    // the norm gain is the same for every token: parked in LDS once (read after the first barrier below)
    float* gain_lds = reinterpret_cast<float*>(rowbuf + (size_t)GR * stride);
    if (a.gain) {
        for (int k = 4 * threadIdx.x; k < K; k += 4 * AQ_THREADS)
            *reinterpret_cast<float4*>(gain_lds + k) = *reinterpret_cast<const float4*>(a.gain + k);
    }

    while (true) {
        const int next_rnd = (rnd + 1) % RPG;
        const int next_grp = next_rnd == 0 ? grp + (int)gridDim.x : grp;
        const bool more = next_grp < ngroups;
        float4 vn[HV4];
        if (more) load_rows<HV4, WPT>(a, next_grp * GR + next_rnd * TPR + rl, lane, part, vn);

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
            // the GR tokens of one chunk are GR * 16 contiguous bytes of the tile
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
        for (int i = 0; i < HV4; ++i) v[i] = vn[i];
        grp = next_grp;
        rnd = next_rnd;
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

template <int HV4, int WPT, int GR>
int launch_one(const QK& a, hipStream_t s) {
    const int ngroups = (a.M + GR - 1) / GR;
    const size_t lds = (size_t)GR * (a.Kp + 16) + (a.gain ? (size_t)a.Kp * 4 : 0);
    static int slots = 0;            // workgroups the device holds at once
    static bool raised = false;      // more than the default 64 KB of dynamic LDS allowed
    constexpr size_t max_lds = (size_t)GR * (HV4 * WPT * 256 + 16) + (size_t)HV4 * WPT * 256 * 4;
    if (!raised && max_lds > 65536) {
        BRL_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&act_quant_kernel<HV4, WPT, GR>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_lds));
        raised = true;
    }
    if (slots == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, act_quant_kernel<HV4, WPT, GR>, AQ_THREADS, max_lds) !=
                hipSuccess ||
            cus <= 0 || per_cu <= 0) {
            (void)hipGetLastError();
            cus = 256;
            per_cu = 1;
        }
        slots = cus * per_cu;
    }
    const int grid = ngroups < slots ? ngroups : slots;
    hipLaunchKernelGGL((act_quant_kernel<HV4, WPT, GR>), dim3(grid), dim3(AQ_THREADS), lds, s, a);
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
    if (a.Kp <= 1024) {
        rc = rows ? launch_rows<1, 4>(a, s) : launch_one<2, 2, 8>(a, s);
    } else if (a.Kp <= 3072) {
        rc = rows ? launch_rows<3, 4>(a, s) : launch_one<6, 2, 8>(a, s);
    } else if (a.Kp <= 4608) {
        rc = rows ? launch_rows<3, 6>(a, s) : launch_one<9, 2, 8>(a, s);
    } else if (a.Kp <= 7168) {
        rc = rows ? launch_rows<4, 7>(a, s) : launch_one<7, 4, 8>(a, s);
    } else {
        rc = rows ? launch_rows<4, 9>(a, s) : launch_one<9, 4, 8>(a, s);
    }
    if (rc != BRL_OK) return rc;
    BRL_LAUNCH_CHECK("act_quant_kernel");
    return BRL_OK;
}

}  // namespace brl
