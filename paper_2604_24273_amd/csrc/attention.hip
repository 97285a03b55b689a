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
    int B, S, Hq, Hkv;    // S: rows per state, or the bound on the state lengths with a SeqMap
    SeqMap sm;
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
    const int len = seq_len(a.sm, b, a.S);
    const size_t row0 = (size_t)seq_row0(a.sm, b, a.S);
    const int p_hi = min((rho0 / a.S != rho1 / a.S) ? a.S - 1 : rho1 % a.S, len - 1);

    const int rho = rho0 + threadIdx.x;
    const bool live = rho < R && rho % a.S < len;
    const int h = j * group + (live ? rho / a.S : 0);
    const int p = live ? rho % a.S : 0;
    const int dq = a.Hq * DH, dkv = a.Hkv * DH;

    float q[DH], o[DH];
    {
        const float* qp = a.qkv + (row0 + p) * a.ld + (size_t)h * DH;
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

    const int n_blocks = p_hi < 0 ? 0 : p_hi / AT_KB + 1;
    for (int kb = 0; kb < n_blocks; ++kb) {
        __syncthreads();
        // stage K (rotated) and V of keys kb*32 .. kb*32+31
        for (int e = threadIdx.x; e < AT_KB * HALF; e += AT_THREADS) {
            const int jj = e / HALF, i = e % HALF;
            const int kp = kb * AT_KB + jj;
            float k1 = 0.f, k2 = 0.f, v1 = 0.f, v2 = 0.f, cs = 1.f, sn = 0.f;
            if (kp < len) {
                const float* row = a.qkv + (row0 + kp) * a.ld;
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
        float* op = a.out + (row0 + p) * dq + (size_t)h * DH;
#pragma unroll
        for (int d = 0; d < DH; ++d) op[d] = o[d] * inv;
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

int launch_attention_f32(const float* qkv, int ld, int B, int S, const SeqMap& sm, int n_heads, int n_kv_heads,
                         int head_dim, const float* cos_t, const float* sin_t, float* out, hipStream_t s) {
    AttnArgs a;
    a.qkv = qkv; a.ld = ld; a.B = B; a.S = S; a.sm = sm; a.Hq = n_heads; a.Hkv = n_kv_heads;
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

}  // namespace brl
