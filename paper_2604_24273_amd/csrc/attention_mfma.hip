// Rotary causal grouped-query attention on the matrix cores: fp16 hi + lo split
// operands, fp32 accumulation and softmax.
//
// Every fp32 operand x is carried as hi = fp16(x), lo = fp16(x - hi); a product is
// taken as hi*hi + hi*lo + lo*hi (three v_mfma_f32_32x32x16_f16 per step), which
// keeps about 21 mantissa bits - the accuracy of fp32 attention at matrix-core speed.
//
// Two kernels:
//  attn_pack_kernel   reads the fp32 k | v rows once, applies the rotary
//                     embedding to k and writes hi / lo fp16 MFMA operand
//                     fragments: 1 KB pieces in lane order, so that every later
//                     load of them is a linear, fully coalesced copy.  (q rows
//                     are used by exactly one wavefront and are rotated and
//                     split by that wavefront itself.)
//  attention_frag_kernel  a wavefront owns 32 queries of one head (lane & 31 =
//                     query, lane >> 5 = k-group).  Per block of 32 keys it
//                     computes the transposed scores S^T = K Q^T, so a lane ends
//                     up with 16 scores of ITS query: the softmax is lane-local
//                     apart from one exchange with lane ^ 32.  The probabilities
//                     stay in registers and become the B operand of
//                     O^T = V^T P^T, which again keeps one query per lane.  The
//                     four wavefronts of a workgroup (the heads of one key/value
//                     group on one query block, so all four need the same
//                     causal range of keys) share each K / V block through LDS,
//                     filled by direct global->LDS loads, double buffered.
// V fragments are stored transposed with the keys of a block permuted so that
// the 8 keys a lane's probabilities stand for are 16 contiguous bytes.
// Where the q | k | v product has already written the fragments (its epilogue does for
// uniform batches at head_dim 128, q included), only attention_frag_kernel runs, in the
// form that reads its q fragments straight into registers (launch_attention_mfma_prepacked).
#include "common.hpp"


namespace brl {

namespace {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

struct PackArgs {
    const float* qkv;     // [B*S, ld]: q heads | k heads | v heads
    int ld, B, S, NRB, Hq, Hkv, dh;   // S: rows per state, or the bound on the state lengths with a SeqMap
    SeqMap sm;
    const float* cos_t;   // [S, dh/2]
    const float* sin_t;
    uint4* KVF;           // [B][Hkv][NRB][ K: [KS][hi,lo] | V: [DB][2][hi,lo] ][64 lanes]
};

__device__ inline uint4 pack8h(const float (&x)[8], bool lo_part) {
    v8h r;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const _Float16 hi = (_Float16)x[e];
        r[e] = lo_part ? (_Float16)(x[e] - (float)hi) : hi;
    }
    return __builtin_bit_cast(uint4, r);
}

template <int VW> struct VecOf;
template <> struct VecOf<4> { typedef float4 type; };
template <> struct VecOf<2> { typedef float2 type; };

// --- staging of one 32-row block of a q or k head -------------------------------------------
// A wavefront reads the rows with fully coalesced loads (VW floats per lane, one or two rows per
// instruction), rotates pairs (i, i + dh/2), scales, splits into fp16 hi / lo and parks both in a
// wave-private LDS region of 128 * DHP bytes: plane hi [32 rows][DHP halfs], then plane lo.  The
// 16-byte chunks of a row are XOR-swizzled so that the later fragment reads (lane = row) spread
// over all banks.  Components beyond dh and rows beyond n_valid are zero.
template <int DHP>
__device__ inline int plane_offset(int r, int chunk) {
    constexpr int RS = DHP * 2, CH = DHP / 8, RPB = 256 / RS;
    return r * RS + ((chunk ^ ((r / RPB) & (CH - 1))) << 4);
}

template <int DHP, int VW>
__device__ inline void stage_rope_rows(const float* rows, int ld, int n_valid, const float* cp, const float* sp,
                                       int dh, float scale, char* region, int lane, int it_begin = 0,
                                       int it_end = 32 / (64 / (DHP / VW))) {
    typedef typename VecOf<VW>::type V;
    constexpr int LPR = DHP / VW, RPI = 64 / LPR;     // lanes per row, rows per instruction
    const int half = dh / 2;
    const int c = lane % LPR, d = c * VW;
    // loads are unconditional (addresses clamped into the block, results masked) so that the
    // loads of many iterations can be in flight together
    const bool in_head = d < dh;
    const bool first = d < half;
    const int ds = in_head ? d : 0;
    const int i = in_head ? (first ? d : d - half) : 0;
    const int dp = in_head ? (first ? d + half : d - half) : 0;
#pragma unroll(32 / VW)
    for (int it = it_begin; it < it_end; ++it) {
        const int r = it * RPI + lane / LPR;
        const int rc = min(r, n_valid - 1);
        const float* row = rows + (size_t)rc * ld;
        const V xs = *reinterpret_cast<const V*>(row + ds);
        const V xp = *reinterpret_cast<const V*>(row + dp);
        const V cs = *reinterpret_cast<const V*>(cp + (size_t)rc * half + i);
        const V sn = *reinterpret_cast<const V*>(sp + (size_t)rc * half + i);
        const float* fs = reinterpret_cast<const float*>(&xs);
        const float* fp = reinterpret_cast<const float*>(&xp);
        const float* fc = reinterpret_cast<const float*>(&cs);
        const float* fn = reinterpret_cast<const float*>(&sn);
        const bool keep = in_head && r < n_valid;
        float v[VW];
#pragma unroll
        for (int e = 0; e < VW; ++e) {
            const float t = (first ? (fs[e] * fc[e] - fp[e] * fn[e]) : (fs[e] * fc[e] + fp[e] * fn[e])) * scale;
            v[e] = keep ? t : 0.f;
        }
        typedef _Float16 hv __attribute__((ext_vector_type(VW)));
        hv hi, lo;
#pragma unroll
        for (int e = 0; e < VW; ++e) {
            hi[e] = (_Float16)v[e];
            lo[e] = (_Float16)(v[e] - (float)hi[e]);
        }
        const int off = plane_offset<DHP>(r, d >> 3) + (d & 7) * 2;
        *reinterpret_cast<hv*>(region + off) = hi;
        *reinterpret_cast<hv*>(region + 64 * DHP + off) = lo;
    }
}

// fragment of k-step ks for lane (row = lane & 31, kg = lane >> 5): components 16 ks + 8 kg + 0..7
template <int DHP>
__device__ inline uint4 staged_fragment(const char* region, int ks, int lane, int lo_plane) {
    return *reinterpret_cast<const uint4*>(region + lo_plane * 64 * DHP +
                                           plane_offset<DHP>(lane & 31, 2 * ks + (lane >> 5)));
}

template <int DHP, int VW>
__global__ __launch_bounds__(256) void attn_pack_kernel(PackArgs a) {
    constexpr int KS = DHP / 16, DB = DHP / 32;
    constexpr int KVFR = KS * 2 + DB * 4;             // 1 KB fragments per key block
    __shared__ __attribute__((aligned(16))) char park[128 * DHP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hd = blockIdx.x % a.Hkv;
    const int rb = (blockIdx.x / a.Hkv) % a.NRB;
    const int b = blockIdx.x / (a.Hkv * a.NRB);
    const int half = a.dh / 2;
    const int dq = a.Hq * a.dh, dkv = a.Hkv * a.dh;
    const int n_valid = min(32, seq_len(a.sm, b, a.S) - rb * 32);
    if (n_valid <= 0) return;             // this state has no such key block (never read either)
    const float* rows = a.qkv + ((size_t)seq_row0(a.sm, b, a.S) + rb * 32) * a.ld;
    uint4* dst = a.KVF + ((size_t)(b * a.Hkv + hd) * a.NRB + rb) * KVFR * 64;

    // k head: each wavefront stages a quarter of the rows, then writes a quarter of the fragments
    constexpr int ITS = 32 / (64 / (DHP / VW));
    stage_rope_rows<DHP, VW>(rows + dq + hd * a.dh, a.ld, n_valid, a.cos_t + (size_t)rb * 32 * half,
                             a.sin_t + (size_t)rb * 32 * half, a.dh, 1.0f, park, lane, wave * (ITS / 4),
                             (wave + 1) * (ITS / 4));
    __syncthreads();
#pragma unroll
    for (int q = 0; q < KS / 2; ++q) {
        const int fr = wave * (KS / 2) + q;           // fragment = (k-step, plane)
        dst[fr * 64 + lane] = staged_fragment<DHP>(park, fr >> 1, lane, fr & 1);
    }
    // v head, transposed: lane (d, h) of (block r, step t) holds the keys 16 t + 8 (e >> 2) + 4 h + (e & 3)
    const int col0 = dq + dkv + hd * a.dh;
    for (int t = threadIdx.x; t < 128 * DB; t += 256) {
        const int dl = t & 31, h = (t >> 5) & 1, tt = (t >> 6) & 1, r = t >> 7;
        const int d = 32 * r + dl;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int row = 16 * tt + 8 * (e >> 2) + 4 * h + (e & 3);
            v[e] = (row < n_valid && d < a.dh) ? rows[(size_t)row * a.ld + col0 + d] : 0.f;
        }
        const int ln = h * 32 + dl;
        dst[(KS * 2 + (r * 2 + tt) * 2 + 0) * 64 + ln] = pack8h(v, false);
        dst[(KS * 2 + (r * 2 + tt) * 2 + 1) * 64 + ln] = pack8h(v, true);
    }
}

struct FragArgs {
    const float* qkv;     // [B*S, ld]: the q heads are read from here
    int ld;
    const float* cos_t;
    const float* sin_t;
    float qscale;         // softmax scale in log2 units, folded into q
    const uint4* KVF;
    const uint4* QF;      // q fragments [B][Hq][NRB][KS][hi,lo][64 lanes] (only where the producer wrote them)
    int B, S, NRB, Hq, Hkv, dh;
    SeqMap sm;
    int n_work;           // B * Hkv * chunks
    float* out;           // [B*S, Hq*dh]
};

template <int DHP>
struct AttnTile {
    static constexpr int KS = DHP / 16, DB = DHP / 32;
    static constexpr int KVFR = KS * 2 + DB * 4;      // 1 KB fragments per key block (K hi/lo, then V hi/lo)
    // the WPG wavefronts of a workgroup copy KVFR / WPG fragments each
    template <int WPG>
    static __device__ inline void issue(const uint4* src, uint4* st, int wave, int lane) {
        static_assert(KVFR % WPG == 0, "fragments divide evenly over the wavefronts");
#pragma unroll
        for (int c = 0; c < KVFR / WPG; ++c) {
            const int f = c * WPG + wave;
            __builtin_amdgcn_global_load_lds(src + f * 64 + lane, st + f * 64, 16, 0, 0);
        }
    }

    // one block of 32 keys against the wavefront's 32 queries
    static __device__ inline void compute(const uint4* st, const v8h (&qh)[KS], const v8h (&ql)[KS], v16f (&o)[DB],
                                          float& m_run, float& l_run, bool diagonal, int lane) {
        const int qi = lane & 31, h = lane >> 5;
        v16f s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const v8h kfh = __builtin_bit_cast(v8h, st[(ks * 2 + 0) * 64 + lane]);
            const v8h kfl = __builtin_bit_cast(v8h, st[(ks * 2 + 1) * 64 + lane]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfl, qh[ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfh, ql[ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfh, qh[ks], s, 0, 0, 0);
        }
        float bmax = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = 8 * (v >> 2) + 4 * h + (v & 3);     // position inside the block
            if (diagonal && key > qi) s[v] = -INFINITY;         // causal: keys of later blocks are never visited
            bmax = fmaxf(bmax, s[v]);
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float m_new = fmaxf(m_run, bmax);                 // finite: key 0 of the block is visible
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float psum = 0.f;
        v8h ph[2], pl[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float pv = __builtin_amdgcn_exp2f(s[v] - m_new);
            psum += pv;
            const _Float16 hi = (_Float16)pv;
            ph[v >> 3][v & 7] = hi;
            pl[v >> 3][v & 7] = (_Float16)(pv - (float)hi);
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int r = 0; r < DB; ++r) {
#pragma unroll
            for (int v = 0; v < 16; ++v) o[r][v] *= alpha;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const v8h vfh = __builtin_bit_cast(v8h, st[(KS * 2 + (r * 2 + t) * 2 + 0) * 64 + lane]);
                const v8h vfl = __builtin_bit_cast(v8h, st[(KS * 2 + (r * 2 + t) * 2 + 1) * 64 + lane]);
                o[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfl, ph[t], o[r], 0, 0, 0);
                o[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfh, pl[t], o[r], 0, 0, 0);
                o[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfh, ph[t], o[r], 0, 0, 0);
            }
        }
    }
};

// WPG wavefronts (a multiple of 4) = WPG units of one key/value head share every K / V block.
// Four is what is launched: eight halved the K / V traffic but ran 12-19 % slower on both
// measured shapes (fewer resident workgroups, longer tails).
constexpr int ATTN_WPG = 4;
constexpr int SHORT_MAX_WORK = 1024;      // beyond this many workgroups the two-kernel path keeps more of them resident
// QPRE: the q rows arrive as fragments (rotated, scaled, split by the kernel that produced them) and are read
// straight into the operand registers; otherwise they are staged from the fp32 rows here.
template <int DHP, int VW, int WPG, bool QPRE = false>
__global__ __launch_bounds__(WPG * 64, 2) void attention_frag_kernel(FragArgs a) {
    using T = AttnTile<DHP>;
    constexpr int KS = T::KS, DB = T::DB;
    __shared__ __attribute__((aligned(1024))) uint4 stage0[T::KVFR * 64];
    __shared__ __attribute__((aligned(1024))) uint4 stage1[T::KVFR * 64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int group = a.Hq / a.Hkv;
    const int U = group * a.NRB;                      // (query block, head in group) units of one key/value head
    const int chunks = (U + WPG - 1) / WPG;
    // consecutive work items (the chunks of one key/value head) run on one XCD and share its L2;
    // the longest chunks of a head come first
    const int per_xcd = (a.n_work + 7) >> 3;
    const int w = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (w >= a.n_work) return;
    const int c = chunks - 1 - w % chunks;
    const int j = (w / chunks) % a.Hkv;
    const int b = w / (chunks * a.Hkv);
    const int len = seq_len(a.sm, b, a.S);
    const int nrb = (len + 31) >> 5;                  // query / key blocks this state really has
    const size_t row0 = (size_t)seq_row0(a.sm, b, a.S);
    // unit u = (query block u / group, head u % group of the group): the wavefronts of a workgroup sit on
    // the same query block (or neighbouring ones), so they need the same key blocks and finish together
    const int u0 = WPG * c, u1 = min(U, u0 + WPG) - 1;
    if (u0 / group >= nrb) return;                    // none of the units exists in this state
    const int kb_max = min(u1 / group, nrb - 1);
    const int u = u0 + wave;
    const bool live = u < U && u / group < nrb;
    const int head = j * group + (live ? u % group : 0);
    const int qb = live ? u / group : -1;

    v8h qh[KS], ql[KS];
    const int qpos = qb * 32 + (lane & 31);
    if constexpr (QPRE) {
        const uint4* qf = a.QF + ((size_t)(b * a.Hq + head) * a.NRB + max(qb, 0)) * (KS * 2 * 64) + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qh[ks] = __builtin_bit_cast(v8h, qf[(ks * 2 + 0) * 64]);
            ql[ks] = __builtin_bit_cast(v8h, qf[(ks * 2 + 1) * 64]);
        }
    } else {
        // the stage buffers are free before the first key block arrives: the q rows are parked there,
        // four wavefronts at a time
        char* region = reinterpret_cast<char*>((wave & 2) ? stage1 : stage0) + (wave & 1) * (128 * DHP);
#pragma unroll
        for (int rnd = 0; rnd < WPG / 4; ++rnd) {
            const bool mine = (wave >> 2) == rnd;
            if (mine && live) {
                const int half = a.dh / 2;
                stage_rope_rows<DHP, VW>(a.qkv + (row0 + qb * 32) * a.ld + head * a.dh, a.ld,
                                         min(32, len - qb * 32), a.cos_t + (size_t)qb * 32 * half,
                                         a.sin_t + (size_t)qb * 32 * half, a.dh, a.qscale, region, lane);
            }
            __syncthreads();
            if (mine) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    qh[ks] = __builtin_bit_cast(v8h, staged_fragment<DHP>(region, ks, lane, 0));
                    ql[ks] = __builtin_bit_cast(v8h, staged_fragment<DHP>(region, ks, lane, 1));
                }
            }
            __syncthreads();
        }
    }
    v16f o[DB];
#pragma unroll
    for (int r = 0; r < DB; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[r][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const uint4* kv = a.KVF + (size_t)(b * a.Hkv + j) * a.NRB * T::KVFR * 64;
    T::template issue<WPG>(kv, stage0, wave, lane);
    int kb = 0;
    for (; kb + 1 <= kb_max; kb += 2) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        T::template issue<WPG>(kv + (size_t)(kb + 1) * T::KVFR * 64, stage1, wave, lane);
        if (kb <= qb) T::compute(stage0, qh, ql, o, m_run, l_run, kb == qb, lane);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (kb + 2 <= kb_max) T::template issue<WPG>(kv + (size_t)(kb + 2) * T::KVFR * 64, stage0, wave, lane);
        if (kb + 1 <= qb) T::compute(stage1, qh, ql, o, m_run, l_run, kb + 1 == qb, lane);
    }
    if (kb <= kb_max) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (kb <= qb) T::compute(stage0, qh, ql, o, m_run, l_run, kb == qb, lane);
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const int pos = qpos;
    if (live && pos < len) {
        const float inv = 1.0f / l_tot;
        const int h = lane >> 5;
        float* op = a.out + (row0 + pos) * ((size_t)a.Hq * a.dh) + (size_t)head * a.dh;
#pragma unroll
        for (int r = 0; r < DB; ++r)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int d = 32 * r + 8 * g4 + 4 * h;
                if (d < a.dh) {
                    float4 v;
                    v.x = o[r][4 * g4 + 0] * inv; v.y = o[r][4 * g4 + 1] * inv;
                    v.z = o[r][4 * g4 + 2] * inv; v.w = o[r][4 * g4 + 3] * inv;
                    *reinterpret_cast<float4*>(op + d) = v;
                }
            }
    }
}

// States of at most 32 tokens (one key block): one kernel, no fragment round trip through
// memory.  A workgroup = (state, key/value head, up to four query heads of its group).  All
// global reads are requested in one phase by two sets of wavefronts side by side: four stage
// one q head each, four stage a quarter of the k rows each and hold v in registers; after one
// barrier the k and v fragments are laid out in LDS exactly as attn_pack_kernel lays them out
// in memory, and the block is computed by the same code as in the general kernel.  Such a
// launch is latency bound.
template <int DHP, int VW>
__global__ __launch_bounds__(512) void attention_short_kernel(FragArgs a) {
    using T = AttnTile<DHP>;
    constexpr int KS = T::KS, DB = T::DB;
    constexpr int REG = 128 * DHP;                        // bytes of one staged 32-row block (hi and lo planes)
    __shared__ __attribute__((aligned(1024))) char qpark[4 * REG];
    __shared__ __attribute__((aligned(1024))) char kpark[REG];
    __shared__ __attribute__((aligned(1024))) uint4 kvst[T::KVFR * 64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int group = a.Hq / a.Hkv;
    const int chunks = (group + 3) / 4;
    const int w = blockIdx.x;
    const int c = w % chunks;
    const int j = (w / chunks) % a.Hkv;
    const int b = w / (chunks * a.Hkv);
    const int len = seq_len(a.sm, b, a.S);                // 1 .. 32
    if (len <= 0) return;
    const size_t row0 = (size_t)seq_row0(a.sm, b, a.S);
    const bool qside = wave < 4;                          // wavefronts 0-3: one q head each; 4-7: k and v
    const int u = 4 * c + (wave & 3);
    const bool live = qside && u < group;
    const int head = j * group + (live ? u : 0);
    const int dq = a.Hq * a.dh, dkv = a.Hkv * a.dh;
    const float* rows = a.qkv + row0 * a.ld;

    // ---- one phase of global reads, the two sides in parallel
    char* region = qpark + (wave & 3) * REG;
    constexpr int ITS = 32 / (64 / (DHP / VW));
    constexpr int VR = (128 * DB + 255) / 256;            // v: thread t of 128 * DB owns lane slot (d, h) of (block r, step tt)
    float vv[VR][8];
    const int tk = threadIdx.x - 256;
    if (qside) {
        if (live) stage_rope_rows<DHP, VW>(rows + head * a.dh, a.ld, len, a.cos_t, a.sin_t, a.dh, a.qscale, region, lane);
    } else {
        const int col0 = dq + dkv + j * a.dh;
#pragma unroll
        for (int q = 0; q < VR; ++q) {
            const int t = tk + 256 * q;
            const int dl = t & 31, h = (t >> 5) & 1, tt = (t >> 6) & 1, r = t >> 7;
            const int d = 32 * r + dl;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int row = 16 * tt + 8 * (e >> 2) + 4 * h + (e & 3);
                vv[q][e] = (t < 128 * DB && row < len && d < a.dh) ? rows[(size_t)row * a.ld + col0 + d] : 0.f;
            }
        }
        stage_rope_rows<DHP, VW>(rows + dq + j * a.dh, a.ld, len, a.cos_t, a.sin_t, a.dh, 1.0f, kpark, lane,
                                 (wave - 4) * (ITS / 4), (wave - 3) * (ITS / 4));
    }
    __syncthreads();

    v8h qh[KS], ql[KS];
    if (qside) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qh[ks] = __builtin_bit_cast(v8h, staged_fragment<DHP>(region, ks, lane, 0));
            ql[ks] = __builtin_bit_cast(v8h, staged_fragment<DHP>(region, ks, lane, 1));
        }
    } else {
#pragma unroll
        for (int q = 0; q < KS / 2; ++q) {
            const int fr = (wave - 4) * (KS / 2) + q;     // fragment = (k-step, plane)
            kvst[fr * 64 + lane] = staged_fragment<DHP>(kpark, fr >> 1, lane, fr & 1);
        }
#pragma unroll
        for (int q = 0; q < VR; ++q) {
            const int t = tk + 256 * q;
            if (t < 128 * DB) {
                const int dl = t & 31, h = (t >> 5) & 1, tt = (t >> 6) & 1, r = t >> 7;
                const int ln = h * 32 + dl;
                kvst[(KS * 2 + (r * 2 + tt) * 2 + 0) * 64 + ln] = pack8h(vv[q], false);
                kvst[(KS * 2 + (r * 2 + tt) * 2 + 1) * 64 + ln] = pack8h(vv[q], true);
            }
        }
    }
    __syncthreads();
    if (!qside) return;

    v16f o[DB];
#pragma unroll
    for (int r = 0; r < DB; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[r][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    T::compute(kvst, qh, ql, o, m_run, l_run, true, lane);

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const int pos = lane & 31;
    if (live && pos < len) {
        const float inv = 1.0f / l_tot;
        const int h = lane >> 5;
        float* op = a.out + (row0 + pos) * ((size_t)a.Hq * a.dh) + (size_t)head * a.dh;
#pragma unroll
        for (int r = 0; r < DB; ++r)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int d = 32 * r + 8 * g4 + 4 * h;
                if (d < a.dh) {
                    float4 v;
                    v.x = o[r][4 * g4 + 0] * inv; v.y = o[r][4 * g4 + 1] * inv;
                    v.z = o[r][4 * g4 + 2] * inv; v.w = o[r][4 * g4 + 3] * inv;
                    *reinterpret_cast<float4*>(op + d) = v;
                }
            }
    }
}

inline int padded_head_dim(int dh) { return dh <= 32 ? 32 : (dh <= 64 ? 64 : 128); }

}  // namespace

size_t attention_mfma_ws_bytes(int B, int S, int n_heads, int n_kv_heads, int head_dim, bool q_frags) {
    const int dhp = padded_head_dim(head_dim);
    const size_t nrb = (size_t)(S + 31) / 32, ks = dhp / 16, db = dhp / 32;
    return (size_t)B * n_kv_heads * nrb * (ks * 2 + db * 4) * 1024 + (q_frags ? (size_t)B * n_heads * nrb * ks * 2 * 1024 : 0);
}

void* attention_q_fragments(void* frag_ws, int B, int S, int n_kv_heads, int head_dim) {
    return static_cast<char*>(frag_ws) + attention_mfma_ws_bytes(B, S, 0, n_kv_heads, head_dim, false);
}

namespace {

template <int DHP, int VW>
void launch_pair(const PackArgs& p, const FragArgs& f, dim3 pgrid, int n_work, hipStream_t s) {
    if (p.NRB == 1 && n_work <= SHORT_MAX_WORK) {         // few short states: the one-kernel path
        const int chunks = (f.Hq / f.Hkv + 3) / 4;
        hipLaunchKernelGGL((attention_short_kernel<DHP, VW>), dim3((unsigned)(f.B * f.Hkv * chunks)), dim3(512), 0, s, f);
        return;
    }
    hipLaunchKernelGGL((attn_pack_kernel<DHP, VW>), pgrid, dim3(256), 0, s, p);
    const dim3 agrid((unsigned)(8 * ((n_work + 7) / 8)));
    hipLaunchKernelGGL((attention_frag_kernel<DHP, VW, ATTN_WPG>), agrid, dim3(ATTN_WPG * 64), 0, s, f);
}

}  // namespace

int launch_attention_mfma(const float* qkv, int ld, int B, int S, const SeqMap& sm, int n_heads, int n_kv_heads,
                          int head_dim, const float* cos_t, const float* sin_t, void* frag_ws, float* out, hipStream_t s) {
    if (head_dim % 4 != 0 || head_dim > 128 || ld % 4 != 0) {
        set_error("attention: head_dim %d must be a multiple of 4, at most 128 (row stride %d a multiple of 4)",
                  head_dim, ld);
        return BRL_EINVAL;
    }
    const int dhp = padded_head_dim(head_dim);
    const int nrb = (S + 31) / 32;
    const int group = n_heads / n_kv_heads;
    const int chunks = (group * nrb + ATTN_WPG - 1) / ATTN_WPG;
    PackArgs p;
    p.qkv = qkv; p.ld = ld; p.B = B; p.S = S; p.NRB = nrb; p.Hq = n_heads; p.Hkv = n_kv_heads; p.dh = head_dim;
    p.sm = sm;
    p.cos_t = cos_t; p.sin_t = sin_t;
    p.KVF = static_cast<uint4*>(frag_ws);
    FragArgs f;
    f.qkv = qkv; f.ld = ld; f.cos_t = cos_t; f.sin_t = sin_t;
    f.qscale = (float)(1.0 / sqrt((double)head_dim)) * 1.4426950408889634f;
    f.KVF = p.KVF; f.QF = nullptr; f.B = B; f.S = S; f.NRB = nrb; f.Hq = n_heads; f.Hkv = n_kv_heads; f.dh = head_dim;
    f.sm = sm;
    f.n_work = B * n_kv_heads * chunks;
    f.out = out;
    const dim3 pgrid((unsigned)((size_t)B * nrb * n_kv_heads));
    const bool v4 = (head_dim / 2) % 4 == 0;          // rotary halves and head rows 16-byte aligned
    LaunchTimer tm(BRL_KC_ATTENTION, s);
    if (dhp == 32) {
        if (v4) launch_pair<32, 4>(p, f, pgrid, f.n_work, s); else launch_pair<32, 2>(p, f, pgrid, f.n_work, s);
    } else if (dhp == 64) {
        if (v4) launch_pair<64, 4>(p, f, pgrid, f.n_work, s); else launch_pair<64, 2>(p, f, pgrid, f.n_work, s);
    } else {
        if (v4) launch_pair<128, 4>(p, f, pgrid, f.n_work, s); else launch_pair<128, 2>(p, f, pgrid, f.n_work, s);
    }
    BRL_LAUNCH_CHECK("attention_mfma");
    return BRL_OK;
}

// The fragments are already in frag_ws (K / V, then q): written by the epilogue of the q | k | v product.
int launch_attention_mfma_prepacked(int B, int S, int n_heads, int n_kv_heads, void* frag_ws, float* out, hipStream_t s) {
    constexpr int dh = 128;
    if (S % 32 != 0 || n_heads % n_kv_heads != 0) {
        set_error("attention: prepacked operands need 32 | S (S = %d) and whole head groups", S);
        return BRL_EINVAL;
    }
    const int nrb = S / 32;
    const int group = n_heads / n_kv_heads;
    const int chunks = (group * nrb + ATTN_WPG - 1) / ATTN_WPG;
    FragArgs f;
    f.qkv = nullptr; f.ld = 0; f.cos_t = nullptr; f.sin_t = nullptr;
    f.qscale = 0.f;
    f.KVF = static_cast<const uint4*>(frag_ws);
    f.QF = static_cast<const uint4*>(attention_q_fragments(frag_ws, B, S, n_kv_heads, dh));
    f.B = B; f.S = S; f.NRB = nrb; f.Hq = n_heads; f.Hkv = n_kv_heads; f.dh = dh;
    f.sm.cu = nullptr; f.sm.b0 = 0;
    f.n_work = B * n_kv_heads * chunks;
    f.out = out;
    LaunchTimer tm(BRL_KC_ATTENTION, s);
    const dim3 agrid((unsigned)(8 * ((f.n_work + 7) / 8)));
    hipLaunchKernelGGL((attention_frag_kernel<128, 4, ATTN_WPG, true>), agrid, dim3(ATTN_WPG * 64), 0, s, f);
    BRL_LAUNCH_CHECK("attention_mfma (prepacked)");
    return BRL_OK;
}

}  // namespace brl
