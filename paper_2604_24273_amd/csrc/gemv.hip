// Bandwidth-bound BitLinear for 1..4 tokens: y = dequant(codes . quant(x)).
//
// One workgroup of 16 wavefronts owns one block of 32 output rows over the whole
// k range, so no partial sums ever cross workgroups (no atomics, no fences).
// The packed weights are streamed once with 16-byte-per-lane loads (a wavefront
// reads contiguous 1 KB blocks of 32 rows x 128 columns), all of them issued
// before anything else: the whole matrix is in flight while the activation
// rows are quantised (every workgroup redoes that cheap step on its own).
// The 2-bit fields are expanded in registers to offset codes c = code + 1 and
// contracted with v_dot4_i32_i8 against the int8 activations held in LDS;
// sum_k q is subtracted at the end.
#include "common.hpp"

namespace brl {

namespace {

constexpr int GV_THREADS = 1024;
constexpr int GV_WAVES = GV_THREADS / 64;
constexpr int GV_MAX_SB = MAX_K / SBK;                                   // 72 super-blocks
constexpr int GV_SB_PER_WAVE = (GV_MAX_SB + GV_WAVES - 1) / GV_WAVES;    // 5
constexpr int GV_X4 = (MAX_K / 4 + GV_THREADS - 1) / GV_THREADS;         // float4 of one row per thread: 3

struct GemvArgs {
    const void* x;
    int x_dtype;
    int M, K, N, nsb;
    const uint4* packed;
    const float* beta;
    float eps_act;
    float* y;
    const float* residual;
    int8_t* xq_dbg;
    float* absmax_dbg;
    int32_t* acc_dbg;
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
    __shared__ __attribute__((aligned(16))) int xq[MT][MAX_K / 4];     // int8 activations as dwords (zero padded)
    __shared__ float wmax[MT][GV_WAVES];
    __shared__ int wsum[MT][GV_WAVES];
    __shared__ int red[GV_WAVES][MT][32];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nb = blockIdx.x;
    const int K = g.K, Kp = g.nsb * SBK;

    // 1. weight loads first: they do not depend on the activations
    uint4 wreg[GV_SB_PER_WAVE];
#pragma unroll
    for (int u = 0; u < GV_SB_PER_WAVE; ++u) {
        const int sb = wave + GV_WAVES * u;
        wreg[u] = make_uint4(0x55555555u, 0x55555555u, 0x55555555u, 0x55555555u);   // code 0 everywhere
        if (sb < g.nsb) wreg[u] = g.packed[((size_t)nb * g.nsb + sb) * 64 + lane];
    }

    // 2. activation rows into registers, per-token absmax
    float4 xv[MT][GV_X4];
    float tmax[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        tmax[t] = 0.f;
#pragma unroll
        for (int u = 0; u < GV_X4; ++u) {
            const int k = 4 * ((int)threadIdx.x + GV_THREADS * u);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (t < g.M && k < K) v = load_x4(g.x, g.x_dtype, (size_t)t * K + k);
            xv[t][u] = v;
            tmax[t] = fmaxf(tmax[t], fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) tmax[t] = fmaxf(tmax[t], __shfl_xor(tmax[t], off, 64));
        if (lane == 0) wmax[t][wave] = tmax[t];
    }
    __syncthreads();

    // 3. quantise into LDS
    float ac[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        float m = wmax[t][0];
#pragma unroll
        for (int w = 1; w < GV_WAVES; ++w) m = fmaxf(m, wmax[t][w]);
        ac[t] = fmaxf(m, g.eps_act);
        const float sc = 127.0f / ac[t];
        int qsum = 0;
#pragma unroll
        for (int u = 0; u < GV_X4; ++u) {
            const int k = 4 * ((int)threadIdx.x + GV_THREADS * u);
            if (k < Kp) {
                const float4 v = xv[t][u];
                const int q0 = (int)fminf(fmaxf(rintf(v.x * sc), -127.f), 127.f);
                const int q1 = (int)fminf(fmaxf(rintf(v.y * sc), -127.f), 127.f);
                const int q2 = (int)fminf(fmaxf(rintf(v.z * sc), -127.f), 127.f);
                const int q3 = (int)fminf(fmaxf(rintf(v.w * sc), -127.f), 127.f);
                qsum += q0 + q1 + q2 + q3;
                const int word = (q0 & 0xff) | ((q1 & 0xff) << 8) | ((q2 & 0xff) << 16) | ((q3 & 0xff) << 24);
                xq[t][k >> 2] = word;
                if (g.xq_dbg && nb == 0 && t < g.M && k < K) *reinterpret_cast<int*>(g.xq_dbg + (size_t)t * K + k) = word;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) qsum += __shfl_xor(qsum, off, 64);
        if (lane == 0) wsum[t][wave] = qsum;
    }
    if (g.absmax_dbg && nb == 0 && threadIdx.x == 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
            if (t < g.M) g.absmax_dbg[t] = ac[t];
    }
    __syncthreads();

    // 4. contract: lane (r, hh) holds row 32 nb + r, k-half hh of each 32-column step
    int acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = 0;
    const int hh = lane >> 5;
#pragma unroll
    for (int u = 0; u < GV_SB_PER_WAVE; ++u) {
        const int sb = wave + GV_WAVES * u;
        if (sb >= g.nsb) continue;
        const uint32_t wd[4] = {wreg[u].x, wreg[u].y, wreg[u].z, wreg[u].w};
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
            const uint32_t p = wd[dd];
            const int c0 = (int)(p & 0x03030303u), c1 = (int)((p >> 2) & 0x03030303u);
            const int c2 = (int)((p >> 4) & 0x03030303u), c3 = (int)((p >> 6) & 0x03030303u);
            const int xoff = (sb * 128 + dd * 32 + hh * 16) / 4;
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int4 xw = *reinterpret_cast<const int4*>(&xq[t][xoff]);
                acc[t] = __builtin_amdgcn_sdot4(c0, xw.x, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c1, xw.y, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c2, xw.z, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c3, xw.w, acc[t], false);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        acc[t] += __shfl_xor(acc[t], 32, 64);
        if (lane < 32) red[wave][t][lane] = acc[t];
    }
    __syncthreads();

    // 5. finish: threads 0 .. 32 MT - 1 each own one (token, row)
    const int t_of = threadIdx.x >> 5, r_of = threadIdx.x & 31;
    if (t_of < MT && t_of < g.M) {
        int part = 0, sq = 0;
#pragma unroll
        for (int w = 0; w < GV_WAVES; ++w) {
            part += red[w][t_of][r_of];
            sq += wsum[t_of][w];
        }
        part -= sq;
        const int n = nb * 32 + r_of;
        if (n < g.N) {
            float m = wmax[t_of][0];
#pragma unroll
            for (int w = 1; w < GV_WAVES; ++w) m = fmaxf(m, wmax[t_of][w]);
            const float d = fmaxf(m, g.eps_act) / 127.0f;
            const size_t o = (size_t)t_of * g.N + n;
            float val = ((float)part * d) * (*g.beta);
            if (g.residual) val = val + g.residual[o];
            g.y[o] = val;
            if (g.acc_dbg) g.acc_dbg[o] = part;
        }
    }
}

// ---------------------------------------------------------------------------
// Many independent problems of one shape in a single launch.  Work item i is row block
// i % nwg of problem i / nwg.  A persistent workgroup takes a contiguous run of items and
// quantises the activations of a problem once (into LDS) for all of that problem's row
// blocks it owns.  Inside a problem every wavefront owns whole row blocks: it streams the
// block's packed weights in chunks of CH super-blocks (CH chosen to divide k evenly where it can), the next chunk (also across
// row blocks) requested before the current one is contracted, and finishes the 32 rows by
// itself - no partial sums cross wavefronts and no barrier is met until the problem changes.
// ---------------------------------------------------------------------------
struct GemvBatchArgs {
    const uint4* const* packed;   // device arrays of device pointers, one entry per problem
    const float* const* beta;
    const void* const* x;
    float* const* y;
    int x_dtype;
    int M, K, N, nsb, nwg, count;
    float eps_act;
};

// CH = super-blocks (1 KB wavefront loads) per chunk: 4, 5 or 6

// Loads are unconditional (super-blocks past the end of k are clamped to the last one and never
// contracted): with straight-line requests the compiler can count the loads still in flight and
// waits only for the chunk it is about to contract, not for the one just requested.  The weight
// pointers come out of a device array, so they are marked as global memory by hand: generic
// (flat) loads would tie the vector-memory and LDS counters together and force full waits.
typedef unsigned int gb_u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) gb_u32x4* gb_wptr;
template <int CH>
__device__ inline void gb_request(gb_wptr blk, int c, int nsb, uint4 (&w)[CH]) {
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        const int sb = min(c * CH + u, nsb - 1);
        const gb_u32x4 v = blk[(size_t)sb * 64];
        w[u] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// No conditions here either: the activations in LDS are zero from the end of k up to a whole number of
// chunks, so the clamped super-blocks of the last chunk contribute nothing.
template <int MT, int CH>
__device__ inline void gb_contract(const uint4 (&w)[CH], int c, int hh, const int (*xq)[MAX_K / 4], int (&acc)[MT]) {
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        const int sb = c * CH + u;
        const uint32_t wd[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
            const uint32_t pw = wd[dd];
            const int c0 = (int)(pw & 0x03030303u), c1 = (int)((pw >> 2) & 0x03030303u);
            const int c2 = (int)((pw >> 4) & 0x03030303u), c3 = (int)((pw >> 6) & 0x03030303u);
            const int xoff = (sb * 128 + dd * 32 + hh * 16) / 4;
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int4 xw = *reinterpret_cast<const int4*>(&xq[t][xoff]);
                acc[t] = __builtin_amdgcn_sdot4(c0, xw.x, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c1, xw.y, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c2, xw.z, acc[t], false);
                acc[t] = __builtin_amdgcn_sdot4(c3, xw.w, acc[t], false);
            }
        }
    }
}

template <int MT, int CH>
__global__ __launch_bounds__(GV_THREADS) void gemv_batch_kernel(GemvBatchArgs g) {
    __shared__ __attribute__((aligned(16))) int xq[MT][MAX_K / 4];   // CH = 5 is only launched where it divides k
    __shared__ float wmax[MT][GV_WAVES];
    __shared__ int wsum[MT][GV_WAVES];
    constexpr int GB_SLOTS = MT == 4 ? 3 : 16 / MT;          // row blocks a wavefront parks before it stores them
    __shared__ float ypark[GV_WAVES][GB_SLOTS][MT][32];

    // the wavefront index as a scalar: everything derived from it (row blocks, cursors, loop bounds) then lives in
    // scalar registers and branches on it are uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int K = g.K;
    const long items = (long)g.count * g.nwg;
    const long i0 = items * blockIdx.x / gridDim.x, i1 = items * (blockIdx.x + 1) / gridDim.x;
    const int hh = lane >> 5;
    const int nchunks = (g.nsb + CH - 1) / CH;
    const int Kc = nchunks * CH * SBK;                       // the xq rows hold a whole number of chunks

    long it = i0;
    while (it < i1) {
        const int p = (int)(it / g.nwg);
        const long p_end = min(i1, (long)(p + 1) * g.nwg);     // this workgroup's items of problem p: [it, p_end)

        // ---- this wavefront's row blocks: it + wave, + 16, ...; a flat walk over (row block, chunk).  The first
        // chunk does not depend on the activations: it is requested ahead of their quantisation.
        const gb_wptr wp = (gb_wptr)g.packed[p];
        const long first = it + wave;
        const int mine = first < p_end ? (int)((p_end - first + GV_WAVES - 1) / GV_WAVES) : 0;
        const int total = mine * nchunks;
        const int nb_first = (int)(first % g.nwg);              // row blocks of one problem are consecutive
        const size_t blk_stride = (size_t)GV_WAVES * g.nsb * 64;
        uint4 wa[CH], wb[CH];
        // request cursor (runs ahead of the contraction cursor over the same sequence)
        gb_wptr rq_blk = wp + (size_t)nb_first * g.nsb * 64 + lane;
        int rq_c = 0, rq_left = total;
        auto request = [&](uint4 (&w)[CH]) {
            gb_request<CH>(rq_blk, rq_c, g.nsb, w);
            if (rq_left > 1) {                 // past the end the last chunk is requested again and dropped
                --rq_left;
                if (++rq_c == nchunks) { rq_c = 0; rq_blk += blk_stride; }
            }
        };
        if (total > 0) request(wa);

        // ---- quantise the activations of problem p into LDS
        __syncthreads();                   // every wavefront is done with the previous problem's xq
        float dsc[MT];                     // a / 127 per token
        int sq[MT];                        // sum_k q per token
        {
            const void* x = (const void*)(const __attribute__((address_space(1))) char*)g.x[p];
            float4 xv[MT][GV_X4];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                float tm = 0.f;
#pragma unroll
                for (int u = 0; u < GV_X4; ++u) {
                    const int k = 4 * ((int)threadIdx.x + GV_THREADS * u);
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (t < g.M && k < K) v = load_x4(x, g.x_dtype, (size_t)t * K + k);
                    xv[t][u] = v;
                    tm = fmaxf(tm, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) tm = fmaxf(tm, __shfl_xor(tm, off, 64));
                if (lane == 0) wmax[t][wave] = tm;
            }
            __syncthreads();
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                float m = wmax[t][0];
#pragma unroll
                for (int w = 1; w < GV_WAVES; ++w) m = fmaxf(m, wmax[t][w]);
                const float ac = fmaxf(m, g.eps_act);
                dsc[t] = ac / 127.0f;
                const float sc = 127.0f / ac;
                int qsum = 0;
#pragma unroll
                for (int u = 0; u < GV_X4; ++u) {
                    const int k = 4 * ((int)threadIdx.x + GV_THREADS * u);
                    if (k < Kc) {          // zeros from K to a whole number of chunks
                        const float4 v = xv[t][u];
                        const int q0 = (int)fminf(fmaxf(rintf(v.x * sc), -127.f), 127.f);
                        const int q1 = (int)fminf(fmaxf(rintf(v.y * sc), -127.f), 127.f);
                        const int q2 = (int)fminf(fmaxf(rintf(v.z * sc), -127.f), 127.f);
                        const int q3 = (int)fminf(fmaxf(rintf(v.w * sc), -127.f), 127.f);
                        qsum += q0 + q1 + q2 + q3;
                        xq[t][k >> 2] = (q0 & 0xff) | ((q1 & 0xff) << 8) | ((q2 & 0xff) << 16) | ((q3 & 0xff) << 24);
                    }
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) qsum += __shfl_xor(qsum, off, 64);
                if (lane == 0) wsum[t][wave] = qsum;
            }
            __syncthreads();
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                int sum = 0;
#pragma unroll
                for (int w = 0; w < GV_WAVES; ++w) sum += wsum[t][w];
                sq[t] = sum;
            }
        }
        const float beta = *(const __attribute__((address_space(1))) float*)g.beta[p];
        __attribute__((address_space(1))) float* yp = (__attribute__((address_space(1))) float*)g.y[p];
        int acc[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[t] = 0;

        if (total > 0) {
            int cc = 0, nb = nb_first;         // chunk and row block being contracted
            int slot = 0, nb_slot0 = nb_first; // results parked in LDS: row blocks nb_slot0, + 16, ... (slot of them)
            // Results go to LDS first and to memory in groups: a store in flight between the weight loads would
            // make every later wait a wait for everything (loads and stores share one counter).
            auto flush = [&]() {
                for (int sl = 0; sl < slot; ++sl) {
                    const int n = (nb_slot0 + sl * GV_WAVES) * 32 + (lane & 31);
#pragma unroll
                    for (int t = 0; t < MT; ++t)
                        if (lane < 32 && t < g.M && n < g.N) yp[(size_t)t * g.N + n] = ypark[wave][sl][t][lane];
                }
                slot = 0;
            };
            auto contract = [&](const uint4 (&w)[CH]) {
                gb_contract<MT, CH>(w, cc, hh, xq, acc);
                if (++cc == nchunks) {
                    // last chunk of a row block: fold the two k-halves, rescale, park 32 rows per token
                    if (slot == 0) nb_slot0 = nb;
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        const int full = acc[t] + __shfl_xor(acc[t], 32, 64);
                        if (lane < 32) ypark[wave][slot][t][lane] = ((float)(full - sq[t]) * dsc[t]) * beta;
                        acc[t] = 0;
                    }
                    cc = 0;
                    nb += GV_WAVES;
                    if (++slot == GB_SLOTS) flush();
                }
            };

            for (int q = 0; q < total; q += 2) {
                request(wb);
                contract(wa);
                request(wa);
                if (q + 1 < total) contract(wb);
            }
            flush();
        }
        it = p_end;
    }
}

template <int MT, int CH>
int launch_batch_ch(const GemvBatchArgs& g, hipStream_t s) {
    static const int slots = [] {        // workgroups the device holds at once
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_batch_kernel<MT, CH>, GV_THREADS, 0) != hipSuccess ||
            cus <= 0 || per_cu <= 0) {
            (void)hipGetLastError();
            cus = 256;
            per_cu = 1;
        }
        return cus * per_cu;
    }();
    const long items = (long)g.count * g.nwg;
    const int grid = (int)(items < slots ? items : slots);
    hipLaunchKernelGGL((gemv_batch_kernel<MT, CH>), dim3(grid), dim3(GV_THREADS), 0, s, g);
    return BRL_OK;
}

// chunk length: one that divides the number of super-blocks (no clamped tail loads), else 4
template <int MT>
int launch_batch_one(const GemvBatchArgs& g, hipStream_t s) {
    if (g.nsb % 4 == 0) return launch_batch_ch<MT, 4>(g, s);
    if (g.nsb % 6 == 0) return launch_batch_ch<MT, 6>(g, s);
    if (g.nsb % 5 == 0) return launch_batch_ch<MT, 5>(g, s);
    return launch_batch_ch<MT, 4>(g, s);
}

}  // namespace

int launch_gemv(const void* x, int x_dtype, int M, int K, int N, const uint32_t* packed, const float* beta,
                float eps_act, float* y, const float* residual, int8_t* xq_dbg, float* absmax_dbg,
                int32_t* acc_dbg, hipStream_t s) {
    GemvArgs g;
    g.x = x; g.x_dtype = x_dtype; g.M = M; g.K = K; g.N = N;
    g.nsb = round_up(K, SBK) / SBK;
    if (g.nsb > GV_MAX_SB) {
        set_error("gemv: K = %d exceeds the supported %d", K, MAX_K);
        return BRL_EINVAL;
    }
    g.packed = reinterpret_cast<const uint4*>(packed);
    g.beta = beta; g.eps_act = eps_act; g.y = y; g.residual = residual;
    g.xq_dbg = xq_dbg; g.absmax_dbg = absmax_dbg; g.acc_dbg = acc_dbg;
    const int grid = round_up(N, NB) / NB;
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

int launch_gemv_batch(const void* const* packed, const float* const* beta, int N, int K, const void* const* x,
                      int x_dtype, int M, float eps_act, float* const* y, int count, hipStream_t s) {
    GemvBatchArgs g;
    g.packed = reinterpret_cast<const uint4* const*>(packed);
    g.beta = beta; g.x = x; g.y = y; g.x_dtype = x_dtype;
    g.M = M; g.K = K; g.N = N;
    g.nsb = round_up(K, SBK) / SBK;
    g.nwg = round_up(N, NB) / NB;
    g.count = count;
    g.eps_act = eps_act;
    if (g.nsb > GV_MAX_SB) {
        set_error("gemv batch: K = %d exceeds the supported %d", K, MAX_K);
        return BRL_EINVAL;
    }
    if (count == 0) return BRL_OK;
    LaunchTimer tm(BRL_KC_GEMV, s);
    switch (M) {
        case 1: launch_batch_one<1>(g, s); break;
        case 2: launch_batch_one<2>(g, s); break;
        case 3:
        case 4: launch_batch_one<4>(g, s); break;
        default: set_error("gemv batch: M = %d out of range 1..4", M); return BRL_EINVAL;
    }
    BRL_LAUNCH_CHECK("gemv_batch_kernel");
    return BRL_OK;
}

}  // namespace brl
