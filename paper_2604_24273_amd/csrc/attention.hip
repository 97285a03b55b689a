// Rotary causal grouped-query attention in fp32 on the vector ALUs.
//
// One thread owns one (query head, position) row: its rotated, pre-scaled query
// and its output accumulator live in registers.  A workgroup takes 256
// consecutive rows of one (state, key/value head) - rows are ordered (head in
// group, position), so the query heads that share a key/value head also share
// the LDS copy of K and V.  Keys are walked in blocks of 32 with the running
// max / running sum form of the softmax, so any S fits.
#include "common.hpp"

namespace brl {

namespace {

constexpr int AT_THREADS = 256;
constexpr int AT_KB = 32;

struct AttnArgs {
    const float* qkv;     // [B*S, ld]: q heads | k heads | v heads
    int ld;
    int B, S, Hq, Hkv;
    const float* cos_t;   // [S, dh/2]
    const float* sin_t;
    float* out;           // [B*S, Hq*dh]
    float scale;
};

__global__ void rope_table_kernel(float* cos_t, float* sin_t, int S, int half, int dh, double theta) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= S * half) return;
    const int p = idx / half, i = idx % half;
    const double inv_freq = pow(theta, -(2.0 * (double)i) / (double)dh);
    const double ang = (double)p * inv_freq;
    cos_t[idx] = (float)cos(ang);
    sin_t[idx] = (float)sin(ang);
}

template <int DH>
__global__ __launch_bounds__(AT_THREADS) void attention_f32_kernel(AttnArgs a) {
    constexpr int HALF = DH / 2;
    __shared__ __attribute__((aligned(16))) float Ks[AT_KB][DH];
    __shared__ __attribute__((aligned(16))) float Vs[AT_KB][DH];

    const int group = a.Hq / a.Hkv;
    const int R = group * a.S;
    const int chunks = (R + AT_THREADS - 1) / AT_THREADS;
    const int c = blockIdx.x % chunks;
    const int j = (blockIdx.x / chunks) % a.Hkv;
    const int b = blockIdx.x / (chunks * a.Hkv);
    const int rho0 = c * AT_THREADS;
    const int rho1 = min(R, rho0 + AT_THREADS) - 1;
    const int p_hi = (rho0 / a.S != rho1 / a.S) ? a.S - 1 : rho1 % a.S;

    const int rho = rho0 + threadIdx.x;
    const bool live = rho < R;
    const int h = j * group + (live ? rho / a.S : 0);
    const int p = live ? rho % a.S : 0;
    const int dq = a.Hq * DH, dkv = a.Hkv * DH;

    float q[DH], o[DH];
    {
        const float* qp = a.qkv + ((size_t)b * a.S + p) * a.ld + (size_t)h * DH;
        const float* cp = a.cos_t + (size_t)p * HALF;
        const float* sp = a.sin_t + (size_t)p * HALF;
#pragma unroll
        for (int i = 0; i < HALF; ++i) {
            const float x1 = live ? qp[i] : 0.f, x2 = live ? qp[i + HALF] : 0.f;
            const float cs = cp[i], sn = sp[i];
            q[i] = (x1 * cs - x2 * sn) * a.scale;
            q[i + HALF] = (x2 * cs + x1 * sn) * a.scale;
        }
#pragma unroll
        for (int d = 0; d < DH; ++d) o[d] = 0.f;
    }
    float m_run = -INFINITY, l_run = 0.f;

    const int n_blocks = p_hi / AT_KB + 1;
    for (int kb = 0; kb < n_blocks; ++kb) {
        __syncthreads();
        // stage K (rotated) and V of keys kb*32 .. kb*32+31
        for (int e = threadIdx.x; e < AT_KB * HALF; e += AT_THREADS) {
            const int jj = e / HALF, i = e % HALF;
            const int kp = kb * AT_KB + jj;
            float k1 = 0.f, k2 = 0.f, v1 = 0.f, v2 = 0.f, cs = 1.f, sn = 0.f;
            if (kp < a.S) {
                const float* row = a.qkv + ((size_t)b * a.S + kp) * a.ld;
                k1 = row[dq + j * DH + i];
                k2 = row[dq + j * DH + i + HALF];
                v1 = row[dq + dkv + j * DH + i];
                v2 = row[dq + dkv + j * DH + i + HALF];
                cs = a.cos_t[(size_t)kp * HALF + i];
                sn = a.sin_t[(size_t)kp * HALF + i];
            }
            Ks[jj][i] = k1 * cs - k2 * sn;
            Ks[jj][i + HALF] = k2 * cs + k1 * sn;
            Vs[jj][i] = v1;
            Vs[jj][i + HALF] = v2;
        }
        __syncthreads();
        if (!live || kb * AT_KB > p) continue;

        float s[AT_KB];
        float bmax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < AT_KB; ++jj) {
            float acc = 0.f;
#pragma unroll
            for (int d = 0; d < DH; d += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(&Ks[jj][d]);
                acc = fmaf(q[d], kv.x, acc);
                acc = fmaf(q[d + 1], kv.y, acc);
                acc = fmaf(q[d + 2], kv.z, acc);
                acc = fmaf(q[d + 3], kv.w, acc);
            }
            s[jj] = (kb * AT_KB + jj <= p) ? acc : -INFINITY;
            bmax = fmaxf(bmax, s[jj]);
        }
        const float m_new = fmaxf(m_run, bmax);          // finite: key kb*32 is visible
        const float alpha = expf(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int jj = 0; jj < AT_KB; ++jj) {
            s[jj] = expf(s[jj] - m_new);
            psum += s[jj];
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int d = 0; d < DH; ++d) o[d] *= alpha;
#pragma unroll
        for (int jj = 0; jj < AT_KB; ++jj) {
            const float pj = s[jj];
#pragma unroll
            for (int d = 0; d < DH; d += 4) {
                const float4 vv = *reinterpret_cast<const float4*>(&Vs[jj][d]);
                o[d] = fmaf(pj, vv.x, o[d]);
                o[d + 1] = fmaf(pj, vv.y, o[d + 1]);
                o[d + 2] = fmaf(pj, vv.z, o[d + 2]);
                o[d + 3] = fmaf(pj, vv.w, o[d + 3]);
            }
        }
    }
    if (live) {
        const float inv = 1.0f / l_run;
        float* op = a.out + ((size_t)b * a.S + p) * dq + (size_t)h * DH;
#pragma unroll
        for (int d = 0; d < DH; ++d) op[d] = o[d] * inv;
    }
}

// ---------------------------------------------------------------------------
// Matrix-core variant: fp16 hi + lo split operands, fp32 accumulation and softmax.
//
// Every fp32 operand x is carried as hi = fp16(x), lo = fp16(x - hi); a product is
// taken as hi*hi + hi*lo + lo*hi on the matrix cores (three
// v_mfma_f32_32x32x16_f16 per step), which keeps about 21 mantissa bits - the
// accuracy of fp32 attention at matrix-core speed.
//
// A wavefront owns 32 query rows (lane & 31 = query, lane >> 5 = k-group).  Per
// block of 32 keys it computes the transposed scores S^T = K Q^T, so that a lane
// ends up with 16 scores of ITS query: the softmax is lane-local apart from one
// exchange with lane ^ 32.  The probabilities stay in registers and become the
// B operand of O^T = V^T P^T, whose result again keeps one query per lane.  V is
// staged transposed in LDS with its key columns permuted so that the 8 keys a
// lane's probabilities stand for are 16 contiguous bytes.  Q and K pass through
// LDS with row-contiguous global reads, the rotary embedding applied on the way.
// ---------------------------------------------------------------------------
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int AM_ROWS = 128;      // query rows per workgroup: 4 wavefronts x 32

__device__ inline void split_store(_Float16* hi, _Float16* lo, int idx, float x) {
    const _Float16 xh = (_Float16)x;
    hi[idx] = xh;
    lo[idx] = (_Float16)(x - (float)xh);
}

__device__ inline uint32_t pack2h(_Float16 a, _Float16 b) {
    typedef _Float16 v2h __attribute__((ext_vector_type(2)));
    v2h t = {a, b};
    return __builtin_bit_cast(uint32_t, t);
}

// Rotate VW consecutive (i, i + half) pairs of one row and store them, split into
// hi + lo halves, at dst[i ..] and dst[i + half ..].  row == nullptr stores zeros.
template <int VW>
__device__ inline void rope_store(_Float16* dst_hi, _Float16* dst_lo, const float* row, const float* cs_p,
                                  const float* sn_p, int i, int half, float scale) {
    float x1[VW], x2[VW], cs[VW], sn[VW];
#pragma unroll
    for (int u = 0; u < VW; ++u) { x1[u] = 0.f; x2[u] = 0.f; cs[u] = 1.f; sn[u] = 0.f; }
    if (row) {
        if (VW == 4) {
            const float4 a1 = *reinterpret_cast<const float4*>(row + i), a2 = *reinterpret_cast<const float4*>(row + i + half);
            const float4 c4 = *reinterpret_cast<const float4*>(cs_p + i), s4 = *reinterpret_cast<const float4*>(sn_p + i);
            x1[0] = a1.x; x1[1] = a1.y; x1[2] = a1.z; x1[3] = a1.w;
            x2[0] = a2.x; x2[1] = a2.y; x2[2] = a2.z; x2[3] = a2.w;
            cs[0] = c4.x; cs[1] = c4.y; cs[2] = c4.z; cs[3] = c4.w;
            sn[0] = s4.x; sn[1] = s4.y; sn[2] = s4.z; sn[3] = s4.w;
        } else {
            const float2 a1 = *reinterpret_cast<const float2*>(row + i), a2 = *reinterpret_cast<const float2*>(row + i + half);
            const float2 c2 = *reinterpret_cast<const float2*>(cs_p + i), s2 = *reinterpret_cast<const float2*>(sn_p + i);
            x1[0] = a1.x; x1[1] = a1.y; x2[0] = a2.x; x2[1] = a2.y;
            cs[0] = c2.x; cs[1] = c2.y; sn[0] = s2.x; sn[1] = s2.y;
        }
    }
    _Float16 h1[VW], l1[VW], h2[VW], l2[VW];
#pragma unroll
    for (int u = 0; u < VW; ++u) {
        const float o1 = (x1[u] * cs[u] - x2[u] * sn[u]) * scale;
        const float o2 = (x2[u] * cs[u] + x1[u] * sn[u]) * scale;
        h1[u] = (_Float16)o1; l1[u] = (_Float16)(o1 - (float)h1[u]);
        h2[u] = (_Float16)o2; l2[u] = (_Float16)(o2 - (float)h2[u]);
    }
#pragma unroll
    for (int u = 0; u < VW; u += 2) {
        *reinterpret_cast<uint32_t*>(dst_hi + i + u) = pack2h(h1[u], h1[u + 1]);
        *reinterpret_cast<uint32_t*>(dst_lo + i + u) = pack2h(l1[u], l1[u + 1]);
        *reinterpret_cast<uint32_t*>(dst_hi + i + half + u) = pack2h(h2[u], h2[u + 1]);
        *reinterpret_cast<uint32_t*>(dst_lo + i + half + u) = pack2h(l2[u], l2[u + 1]);
    }
}

template <int DHP>
__global__ __launch_bounds__(256, 2) void attention_mfma_kernel(AttnArgs a, int dh) {
    constexpr int KS = DHP / 16;          // k-steps of the score MFMAs
    constexpr int DB = DHP / 32;          // 32-row blocks of O^T
    constexpr int KLD = DHP + 8;          // halfs per K row (padding spreads the 16-byte reads over banks)
    constexpr int VLD = 40;               // halfs per V^T row: 32 key slots + padding
    __shared__ __attribute__((aligned(16))) _Float16 Kh[32 * KLD];
    __shared__ __attribute__((aligned(16))) _Float16 Kl[32 * KLD];
    __shared__ __attribute__((aligned(16))) _Float16 Vh[DHP * VLD];
    __shared__ __attribute__((aligned(16))) _Float16 Vl[DHP * VLD];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ql = lane & 31, h = lane >> 5;
    const int group = a.Hq / a.Hkv;
    const int R = group * a.S;
    const int chunks = (R + AM_ROWS - 1) / AM_ROWS;
    const int c = blockIdx.x % chunks;
    const int j = (blockIdx.x / chunks) % a.Hkv;
    const int b = blockIdx.x / (chunks * a.Hkv);
    const int half = dh / 2;
    const int dq = a.Hq * dh, dkv = a.Hkv * dh;

    // key range of the workgroup and of this wavefront (rows are ordered head-major, position-minor)
    const int wg0 = c * AM_ROWS, wg1 = min(R, wg0 + AM_ROWS) - 1;
    const int p_hi_wg = (wg0 / a.S != wg1 / a.S) ? a.S - 1 : wg1 % a.S;
    const int w0 = wg0 + wave * 32, w1 = min(R, w0 + 32) - 1;
    const int p_hi_wave = (w0 > w1) ? -1 : ((w0 / a.S != w1 / a.S) ? a.S - 1 : w1 % a.S);

    const int rho = w0 + ql;
    const bool live = rho < R;
    const int head = j * group + (live ? rho / a.S : 0);
    const int p = live ? rho % a.S : 0;

    // zero both K buffers once: the padding columns d >= dh are never written again
    for (int e = threadIdx.x; e < 32 * KLD; e += 256) {
        Kh[e] = (_Float16)0.f;
        Kl[e] = (_Float16)0.f;
    }

    // Rotated, pre-scaled query fragments (lane holds q[16 ks + 8 h + 0..7]), staged
    // 32 rows at a time through the K buffers so that the global reads are row-contiguous.
    v8h qh[KS], ql_[KS];
    const float qscale = a.scale * 1.4426950408889634f;        // scores in log2 units
    for (int w = 0; w < 4; ++w) {
        __syncthreads();
        {
            const int vw = (half % 4 == 0) ? 4 : 2;
            const int tpr = half / vw;
            for (int t = threadIdx.x; t < 32 * tpr; t += 256) {
                const int r = t / tpr, i = (t % tpr) * vw;
                const int rr = wg0 + w * 32 + r;
                const float* row = nullptr;
                int pp = 0;
                if (rr < R) {
                    pp = rr % a.S;
                    row = a.qkv + ((size_t)b * a.S + pp) * a.ld + (size_t)(j * group + rr / a.S) * dh;
                }
                const float* cp = a.cos_t + (size_t)pp * half;
                const float* sp = a.sin_t + (size_t)pp * half;
                if (vw == 4) rope_store<4>(Kh + r * KLD, Kl + r * KLD, row, cp, sp, i, half, qscale);
                else rope_store<2>(Kh + r * KLD, Kl + r * KLD, row, cp, sp, i, half, qscale);
            }
        }
        __syncthreads();
        if (w == wave) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                qh[ks] = *reinterpret_cast<const v8h*>(&Kh[ql * KLD + 16 * ks + 8 * h]);
                ql_[ks] = *reinterpret_cast<const v8h*>(&Kl[ql * KLD + 16 * ks + 8 * h]);
            }
        }
    }

    v16f o[DB];
#pragma unroll
    for (int r = 0; r < DB; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[r][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int n_blocks = p_hi_wg / 32 + 1;
    for (int kb = 0; kb < n_blocks; ++kb) {
        __syncthreads();
        // stage K (rotated) as [key][d] and V as [d][slot(key)], both split into hi + lo
        {
            const int vw = (half % 4 == 0) ? 4 : 2;
            const int tpr = half / vw;
            for (int t = threadIdx.x; t < 32 * tpr; t += 256) {
                const int r = t / tpr, i = (t % tpr) * vw;
                const int kp = kb * 32 + r;
                const int kc = kp < a.S ? kp : 0;
                const float* row = kp < a.S ? a.qkv + ((size_t)b * a.S + kp) * a.ld + dq + (size_t)j * dh : nullptr;
                const float* cp = a.cos_t + (size_t)kc * half;
                const float* sp = a.sin_t + (size_t)kc * half;
                if (vw == 4) rope_store<4>(Kh + r * KLD, Kl + r * KLD, row, cp, sp, i, half, 1.0f);
                else rope_store<2>(Kh + r * KLD, Kl + r * KLD, row, cp, sp, i, half, 1.0f);
            }
            // V: a task takes 4 consecutive d of key rows 2u and 2u+1 (adjacent slots of V^T)
            for (int t = threadIdx.x; t < 16 * (DHP / 4); t += 256) {
                const int u = t / (DHP / 4), d = (t % (DHP / 4)) * 4;
                const int r = 2 * u;
                const int kp = kb * 32 + r;
                float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
                if (d < dh) {
                    const float* base = a.qkv + ((size_t)b * a.S + kp) * a.ld + dq + dkv + (size_t)j * dh + d;
                    if (kp < a.S) v0 = *reinterpret_cast<const float4*>(base);
                    if (kp + 1 < a.S) v1 = *reinterpret_cast<const float4*>(base + a.ld);
                }
                // key row r = 16 t + 8 a + 4 hh + e'  ->  slot 16 t + 8 hh + 4 a + e'
                const int slot = (r & 16) | ((r & 4) << 1) | ((r & 8) >> 1) | (r & 3);
                const float e0[4] = {v0.x, v0.y, v0.z, v0.w}, e1[4] = {v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const _Float16 h0 = (_Float16)e0[q], h1 = (_Float16)e1[q];
                    *reinterpret_cast<uint32_t*>(&Vh[(d + q) * VLD + slot]) = pack2h(h0, h1);
                    *reinterpret_cast<uint32_t*>(&Vl[(d + q) * VLD + slot]) =
                        pack2h((_Float16)(e0[q] - (float)h0), (_Float16)(e1[q] - (float)h1));
                }
            }
        }
        __syncthreads();
        if (kb * 32 > p_hi_wave) continue;

        v16f s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const v8h kfh = *reinterpret_cast<const v8h*>(&Kh[ql * KLD + 16 * ks + 8 * h]);
            const v8h kfl = *reinterpret_cast<const v8h*>(&Kl[ql * KLD + 16 * ks + 8 * h]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfl, qh[ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfh, ql_[ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfh, qh[ks], s, 0, 0, 0);
        }
        float bmax = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = kb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            s[v] = (live && key <= p) ? s[v] : -INFINITY;
            bmax = fmaxf(bmax, s[v]);
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float m_new = fmaxf(m_run, bmax);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        float psum = 0.f;
        v8h ph[2], pl[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float pv = __builtin_amdgcn_exp2f(s[v] - m_use);
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
                const v8h vfh = *reinterpret_cast<const v8h*>(&Vh[(32 * r + ql) * VLD + 16 * t + 8 * h]);
                const v8h vfl = *reinterpret_cast<const v8h*>(&Vl[(32 * r + ql) * VLD + 16 * t + 8 * h]);
                o[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfl, ph[t], o[r], 0, 0, 0);
                o[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfh, pl[t], o[r], 0, 0, 0);
                o[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfh, ph[t], o[r], 0, 0, 0);
            }
        }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (live) {
        const float inv = 1.0f / l_tot;
        float* op = a.out + ((size_t)b * a.S + p) * dq + (size_t)head * dh;
#pragma unroll
        for (int r = 0; r < DB; ++r)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int d = 32 * r + 8 * g4 + 4 * h;
                if (d < dh) {
                    float4 v;
                    v.x = o[r][4 * g4 + 0] * inv; v.y = o[r][4 * g4 + 1] * inv;
                    v.z = o[r][4 * g4 + 2] * inv; v.w = o[r][4 * g4 + 3] * inv;
                    *reinterpret_cast<float4*>(op + d) = v;
                }
            }
    }
}

}  // namespace

int launch_rope_table(float* cos_t, float* sin_t, int S, int head_dim, float theta, hipStream_t s) {
    const int half = head_dim / 2;
    const int n = S * half;
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, cos_t, sin_t, S, half, head_dim,
                       (double)theta);
    BRL_LAUNCH_CHECK("rope_table_kernel");
    return BRL_OK;
}

int launch_attention_f32(const float* qkv, int ld, int B, int S, int n_heads, int n_kv_heads, int head_dim,
                         const float* cos_t, const float* sin_t, float* out, hipStream_t s) {
    AttnArgs a;
    a.qkv = qkv; a.ld = ld; a.B = B; a.S = S; a.Hq = n_heads; a.Hkv = n_kv_heads;
    a.cos_t = cos_t; a.sin_t = sin_t; a.out = out;
    a.scale = (float)(1.0 / sqrt((double)head_dim));
    const int group = n_heads / n_kv_heads;
    const int chunks = (group * S + AT_THREADS - 1) / AT_THREADS;
    const dim3 grid((unsigned)((size_t)B * n_kv_heads * chunks));
    LaunchTimer tm(BRL_KC_ATTENTION, s);
    switch (head_dim) {
        case 16: hipLaunchKernelGGL(attention_f32_kernel<16>, grid, dim3(AT_THREADS), 0, s, a); break;
        case 32: hipLaunchKernelGGL(attention_f32_kernel<32>, grid, dim3(AT_THREADS), 0, s, a); break;
        case 64: hipLaunchKernelGGL(attention_f32_kernel<64>, grid, dim3(AT_THREADS), 0, s, a); break;
        case 100: hipLaunchKernelGGL(attention_f32_kernel<100>, grid, dim3(AT_THREADS), 0, s, a); break;
        case 128: hipLaunchKernelGGL(attention_f32_kernel<128>, grid, dim3(AT_THREADS), 0, s, a); break;
        default:
            set_error("attention: head_dim %d not in {16, 32, 64, 100, 128}", head_dim);
            return BRL_EINVAL;
    }
    BRL_LAUNCH_CHECK("attention_f32_kernel");
    return BRL_OK;
}

int launch_attention_mfma(const float* qkv, int ld, int B, int S, int n_heads, int n_kv_heads, int head_dim,
                         const float* cos_t, const float* sin_t, float* out, hipStream_t s) {
    AttnArgs a;
    a.qkv = qkv; a.ld = ld; a.B = B; a.S = S; a.Hq = n_heads; a.Hkv = n_kv_heads;
    a.cos_t = cos_t; a.sin_t = sin_t; a.out = out;
    a.scale = (float)(1.0 / sqrt((double)head_dim));
    const int group = n_heads / n_kv_heads;
    const int chunks = (group * S + AM_ROWS - 1) / AM_ROWS;
    const dim3 grid((unsigned)((size_t)B * n_kv_heads * chunks));
    LaunchTimer tm(BRL_KC_ATTENTION, s);
    if (head_dim % 4 != 0 || head_dim > 128) {
        set_error("attention: head_dim %d must be a multiple of 4, at most 128", head_dim);
        return BRL_EINVAL;
    }
    if (head_dim <= 32) hipLaunchKernelGGL(attention_mfma_kernel<32>, grid, dim3(256), 0, s, a, head_dim);
    else if (head_dim <= 64) hipLaunchKernelGGL(attention_mfma_kernel<64>, grid, dim3(256), 0, s, a, head_dim);
    else hipLaunchKernelGGL(attention_mfma_kernel<128>, grid, dim3(256), 0, s, a, head_dim);
    BRL_LAUNCH_CHECK("attention_mfma_kernel");
    return BRL_OK;
}

}  // namespace brl
