// Bandwidth-bound BitLinear for 1..4 tokens: y = dequant(codes . quant(x)).
//
// The packed weights are streamed once with 16-byte-per-lane loads (a wavefront
// reads one contiguous 1 KB block of 32 rows x 128 columns), expanded in
// registers to offset codes c = code + 1 and contracted with v_dot4_i32_i8
// against the int8 activations held in LDS.  A workgroup owns one 32-row block
// and one slice of k; its weight loads are issued before anything else, and the
// activation quantisation (every workgroup redoes the cheap absmax of the few
// token rows, and quantises only its own k-slice) runs while they are in flight.
// Slices of one row block meet through a self-resetting ticket: the workgroup
// that arrives last adds the integer partials (order free, exact) and applies
// the fp32 rescale.
#include "common.hpp"

namespace brl {

namespace {

constexpr int GV_THREADS = 256;
constexpr int GV_MAX_SB = 8;      // super-blocks per workgroup slice (two per wavefront)

struct GemvArgs {
    const void* x;
    int x_dtype;
    int M, K, N, nsb, ksplit, sb_per;
    const uint4* packed;
    const float* beta;
    float eps_act;
    float* y;
    const float* residual;
    int8_t* xq_dbg;
    float* absmax_dbg;
    int32_t* acc_dbg;
    int32_t* partial;
    unsigned* tickets;
};

__device__ inline float4 load_x4(const void* x, int dtype, size_t idx) {
    if (dtype == BRL_BF16) {
        const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(x) + idx);
        return make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                           __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u));
    }
    return *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(x) + idx);
}

template <int MT>
__global__ __launch_bounds__(GV_THREADS) void gemv_kernel(GemvArgs g) {
    __shared__ __attribute__((aligned(16))) int xq[MT][GV_MAX_SB * 128 / 4];       // int8 activations of this k-slice, as dwords
    __shared__ float wmax[MT][GV_THREADS / 64];
    __shared__ int wsum[MT][GV_THREADS / 64];
    __shared__ int red[GV_THREADS / 64][MT][32];
    __shared__ unsigned last_flag;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nb = blockIdx.x / g.ksplit, ks = blockIdx.x % g.ksplit;
    const int sb_lo = ks * g.sb_per;
    const int sb_hi = min(g.nsb, sb_lo + g.sb_per);

    // 1. weight loads first: they do not depend on the activations
    uint4 wreg[2];
    bool have[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int sb = sb_lo + wave + 4 * u;
        have[u] = sb < sb_hi;
        wreg[u] = make_uint4(0x55555555u, 0x55555555u, 0x55555555u, 0x55555555u);   // code 0 everywhere
        if (have[u]) wreg[u] = g.packed[((size_t)nb * g.nsb + sb) * 64 + lane];
    }

    // 2. per-token absmax over the whole row
    const int K = g.K;
    float tmax[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) tmax[t] = 0.f;
    for (int k = 4 * threadIdx.x; k < K; k += 4 * GV_THREADS) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (t < g.M) {
                const float4 v = load_x4(g.x, g.x_dtype, (size_t)t * K + k);
                tmax[t] = fmaxf(tmax[t], fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            }
        }
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) tmax[t] = fmaxf(tmax[t], __shfl_xor(tmax[t], off, 64));
        if (lane == 0) wmax[t][wave] = tmax[t];
    }
    __syncthreads();
    float ac[MT], sc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const float m = fmaxf(fmaxf(wmax[t][0], wmax[t][1]), fmaxf(wmax[t][2], wmax[t][3]));
        ac[t] = fmaxf(m, g.eps_act);
        sc[t] = 127.0f / ac[t];
    }

    // 3. quantise this workgroup's k-slice into LDS (thread -> 4 consecutive k)
    const int k_lo = sb_lo * 128;
    int qsum[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        qsum[t] = 0;
        const int k = k_lo + 4 * threadIdx.x;
        int word = 0;
        if (t < g.M && 4 * (int)threadIdx.x < (sb_hi - sb_lo) * 128 && k < K) {
            const float4 v = load_x4(g.x, g.x_dtype, (size_t)t * K + k);
            const int q0 = (int)fminf(fmaxf(rintf(v.x * sc[t]), -127.f), 127.f);
            const int q1 = (int)fminf(fmaxf(rintf(v.y * sc[t]), -127.f), 127.f);
            const int q2 = (int)fminf(fmaxf(rintf(v.z * sc[t]), -127.f), 127.f);
            const int q3 = (int)fminf(fmaxf(rintf(v.w * sc[t]), -127.f), 127.f);
            qsum[t] = q0 + q1 + q2 + q3;
            word = (q0 & 0xff) | ((q1 & 0xff) << 8) | ((q2 & 0xff) << 16) | ((q3 & 0xff) << 24);
            if (g.xq_dbg && nb == 0) *reinterpret_cast<int*>(g.xq_dbg + (size_t)t * K + k) = word;
        }
        xq[t][threadIdx.x] = word;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) qsum[t] += __shfl_xor(qsum[t], off, 64);
        if (lane == 0) wsum[t][wave] = qsum[t];
    }
    if (g.absmax_dbg && blockIdx.x == 0 && threadIdx.x < MT && (int)threadIdx.x < g.M)
        g.absmax_dbg[threadIdx.x] = fmaxf(fmaxf(fmaxf(wmax[threadIdx.x][0], wmax[threadIdx.x][1]),
                                                fmaxf(wmax[threadIdx.x][2], wmax[threadIdx.x][3])), g.eps_act);
    __syncthreads();

    // 4. contract: lane (r, hh) holds row 32 nb + r, k-half hh of each 32-column step
    int acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = 0;
    const int hh = lane >> 5;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        if (!have[u]) continue;
        const int sbl = wave + 4 * u;                 // super-block index inside the slice
        const uint32_t wd[4] = {wreg[u].x, wreg[u].y, wreg[u].z, wreg[u].w};
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
            const uint32_t p = wd[dd];
            const int c0 = (int)(p & 0x03030303u), c1 = (int)((p >> 2) & 0x03030303u);
            const int c2 = (int)((p >> 4) & 0x03030303u), c3 = (int)((p >> 6) & 0x03030303u);
            const int xoff = (sbl * 128 + dd * 32 + hh * 16) / 4;
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int4 xv = *reinterpret_cast<const int4*>(&xq[t][xoff]);
                acc[t] = __builtin_amdgcn_sdot4(c0, xv.x, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c1, xv.y, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c2, xv.z, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c3, xv.w, acc[t], false);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        acc[t] += __shfl_xor(acc[t], 32, 64);
        if (lane < 32) red[wave][t][lane] = acc[t];
    }
    __syncthreads();

    // 5. workgroup partial for (row block, k-slice), offset-code correction included
    const int t_of = threadIdx.x >> 5, r_of = threadIdx.x & 31;     // threads 0 .. 32*MT-1 finish
    int part = 0;
    if (t_of < MT) {
        part = red[0][t_of][r_of] + red[1][t_of][r_of] + red[2][t_of][r_of] + red[3][t_of][r_of];
        part -= wsum[t_of][0] + wsum[t_of][1] + wsum[t_of][2] + wsum[t_of][3];
    }
    if (g.ksplit > 1) {
        if (t_of < MT) g.partial[((size_t)blockIdx.x * MT + t_of) * 32 + r_of] = part;
        __threadfence();
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned old = atomicInc(&g.tickets[nb], (unsigned)(g.ksplit - 1));   // wraps back to 0
            last_flag = (old == (unsigned)(g.ksplit - 1)) ? 1u : 0u;
        }
        __syncthreads();
        if (!last_flag) return;
        __threadfence();
        if (t_of < MT) {
            part = 0;
            for (int s = 0; s < g.ksplit; ++s)
                part += g.partial[(((size_t)nb * g.ksplit + s) * MT + t_of) * 32 + r_of];
        }
    }

    // 6. rescale
    if (t_of < MT && t_of < g.M) {
        const int n = nb * 32 + r_of;
        if (n < g.N) {
            const float m = fmaxf(fmaxf(fmaxf(wmax[t_of][0], wmax[t_of][1]), fmaxf(wmax[t_of][2], wmax[t_of][3])), g.eps_act);
            const float d = m / 127.0f;
            const size_t o = (size_t)t_of * g.N + n;
            float val = ((float)part * d) * (*g.beta);
            if (g.residual) val = val + g.residual[o];
            g.y[o] = val;
            if (g.acc_dbg) g.acc_dbg[o] = part;
        }
    }
}

}  // namespace

int gemv_ksplit(int N, int K) {
    const int nsb = round_up(K, SBK) / SBK;
    const int nnb = round_up(N, NB) / NB;
    int ks = (nsb + GV_MAX_SB - 1) / GV_MAX_SB;
    const int want = (512 + nnb - 1) / nnb;
    if (want > ks) ks = want;
    if (ks > nsb) ks = nsb;
    if (ks < 1) ks = 1;
    return ks;
}

int launch_gemv(const void* x, int x_dtype, int M, int K, int N, const uint32_t* packed, const float* beta,
                float eps_act, float* y, const float* residual, int8_t* xq_dbg, float* absmax_dbg,
                int32_t* acc_dbg, const GemvWs& ws, hipStream_t s) {
    GemvArgs g;
    g.x = x; g.x_dtype = x_dtype; g.M = M; g.K = K; g.N = N;
    g.nsb = round_up(K, SBK) / SBK;
    g.ksplit = gemv_ksplit(N, K);
    g.sb_per = (g.nsb + g.ksplit - 1) / g.ksplit;
    if (g.sb_per > GV_MAX_SB) {
        set_error("gemv: k-slice of %d super-blocks exceeds %d", g.sb_per, GV_MAX_SB);
        return BRL_EINVAL;
    }
    g.packed = reinterpret_cast<const uint4*>(packed);
    g.beta = beta; g.eps_act = eps_act; g.y = y; g.residual = residual;
    g.xq_dbg = xq_dbg; g.absmax_dbg = absmax_dbg; g.acc_dbg = acc_dbg;
    g.partial = ws.partial; g.tickets = ws.tickets;
    const int nnb = round_up(N, NB) / NB;
    const int grid = nnb * g.ksplit;
    LaunchTimer tm(BRL_KC_GEMV, s);
    switch (M) {
        case 1: hipLaunchKernelGGL(gemv_kernel<1>, dim3(grid), dim3(GV_THREADS), 0, s, g); break;
        case 2: hipLaunchKernelGGL(gemv_kernel<2>, dim3(grid), dim3(GV_THREADS), 0, s, g); break;
        case 3:
        case 4: hipLaunchKernelGGL(gemv_kernel<4>, dim3(grid), dim3(GV_THREADS), 0, s, g); break;
        default: set_error("gemv: M = %d out of range 1..4", M); return BRL_EINVAL;
    }
    BRL_LAUNCH_CHECK("gemv_kernel");
    return BRL_OK;
}

}  // namespace brl
