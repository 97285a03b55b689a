// PPO update of the trainable policy / value heads on cached encoder outputs (Sec. 3.1 Eq. 1,
// Sec. 3.2, Appendix hyper-parameter table), and the generalised advantage estimate.
//
// The backbone is frozen, so a rollout stores h_t once and the update touches only the two small
// MLPs: every mini-batch is a forward pass of both heads, the clipped-surrogate / entropy / value
// gradients at their outputs, back-propagation, one global gradient-norm clip and an Adam step.
// The products are tiny (64 x 2560 x 256), so the work is laid out as a few wide kernels per
// step, each with fp64 accumulation in a fixed order: results do not depend on scheduling.
// Parameters and optimiser state are fp32 in one flat buffer each (policy W_1, b_1, ..., W_L, b_L,
// then the value head likewise); activations, deltas and gradients of a step live in fp64 scratch.
#include "common.hpp"

#include <cmath>
#include <cstring>

namespace brl {

namespace {

constexpr int PPO_MAX_LAYERS = 8;

struct HeadShape {
    int n;                           // layers
    int dims[PPO_MAX_LAYERS + 1];
    size_t w_off[PPO_MAX_LAYERS];    // offsets into the flat parameter buffer
    size_t b_off[PPO_MAX_LAYERS];
};

struct Layout {
    HeadShape head[2];               // 0 policy, 1 value
    size_t n_params, n_policy;
    int max_dim;                     // widest layer output
};

int make_layout(const brl_ppo_config* c, Layout& L) {
    BRL_REQUIRE(c != nullptr, "ppo: null config");
    BRL_REQUIRE(c->policy_dims && c->value_dims, "ppo: null layer sizes");
    BRL_REQUIRE(c->policy_layers >= 1 && c->policy_layers <= PPO_MAX_LAYERS && c->value_layers >= 1 &&
                    c->value_layers <= PPO_MAX_LAYERS,
                "ppo: 1..%d layers per head", PPO_MAX_LAYERS);
    BRL_REQUIRE(c->act == BRL_ACT_TANH || c->act == BRL_ACT_RELU, "ppo: unknown activation %d", c->act);
    size_t off = 0;
    L.max_dim = 1;
    for (int hd = 0; hd < 2; ++hd) {
        HeadShape& H = L.head[hd];
        H.n = hd == 0 ? c->policy_layers : c->value_layers;
        const int* dims = hd == 0 ? c->policy_dims : c->value_dims;
        for (int i = 0; i <= H.n; ++i) {
            BRL_REQUIRE(dims[i] >= 1 && dims[i] <= (1 << 20), "ppo: layer size %d", dims[i]);
            H.dims[i] = dims[i];
            if (i > 0 && dims[i] > L.max_dim) L.max_dim = dims[i];
        }
        for (int l = 0; l < H.n; ++l) {
            H.w_off[l] = off;
            off += (size_t)H.dims[l + 1] * H.dims[l];
            H.b_off[l] = off;
            off += (size_t)H.dims[l + 1];
        }
        if (hd == 0) L.n_policy = off;
    }
    L.n_params = off;
    BRL_REQUIRE(L.head[0].dims[0] == L.head[1].dims[0], "ppo: the heads disagree on the input width");
    BRL_REQUIRE(L.head[1].dims[L.head[1].n] == 1, "ppo: the value head must end in one output");
    BRL_REQUIRE(L.head[0].dims[L.head[0].n] <= 1024, "ppo: at most 1024 actions");
    return BRL_OK;
}

// ---- kernels ---------------------------------------------------------------------------------

// adv[e, t], ret[e, t] for E independent rollouts of T steps, one thread per rollout, backwards in fp64:
// delta = r + gamma V' (1 - done) - V;  A = delta + gamma lambda (1 - done) A'
__global__ void gae_kernel(const float* __restrict__ rewards, const float* __restrict__ values,
                           const float* __restrict__ dones, const float* __restrict__ last_value, int E, int T,
                           double gamma, double lam, float* __restrict__ adv, float* __restrict__ ret) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    double nxt_adv = 0.0, nxt_val = (double)last_value[e];
    for (int t = T - 1; t >= 0; --t) {
        const size_t i = (size_t)e * T + t;
        const double live = 1.0 - (double)dones[i];
        const double v = (double)values[i];
        const double delta = (double)rewards[i] + gamma * nxt_val * live - v;
        nxt_adv = delta + gamma * lam * live * nxt_adv;
        adv[i] = (float)nxt_adv;
        ret[i] = (float)(nxt_adv + v);
        nxt_val = v;
    }
}

// out[b, o] = act(sum_i W[o, i] in(b, i) + bias[o]); a workgroup takes FO output units for FB consecutive
// samples (weight rows and inputs are read once for all of them); its four wavefronts take a quarter of the
// inputs each, sum in fp64 in lane order, fold, and the four parts are added in order.
// in(b, i) = in64[b, i], or for the first layer the cached encoder output h[rows[b], i].
// Rollout indices and actions are caller data read on the device: they are clamped into range so that a bad
// entry can never address memory outside the rollout or the logits (its result is then meaningless, not a fault).
__device__ inline int clamp_index(int v, int n) { return v < 0 ? 0 : (v >= n ? n - 1 : v); }

constexpr int FB = 4;        // samples per workgroup
constexpr int FO = 4;        // output units per workgroup
// One launch runs the same layer level of both heads (they read the same rows of h and depend on nothing of
// each other): the workgroups of problem 0 come first, then those of problem 1.
struct FwdProblem {
    const double* in64;      // null: first layer, inputs are rows of h
    const float* W;
    const float* bias;
    double* out;
    int in_dim, out_dim, last;
    unsigned blocks;
};
struct FwdArgs {
    FwdProblem p[2];
    int n;                   // 1 or 2 problems
    const float* h;
    const int32_t* rows;
    int B, act, T;
};
__global__ __launch_bounds__(256) void ppo_forward_kernel(FwdArgs a) {
    const int which = (a.n > 1 && blockIdx.x >= a.p[0].blocks) ? 1 : 0;
    const unsigned block = blockIdx.x - (which ? a.p[0].blocks : 0u);
    const double* __restrict__ in64 = which ? a.p[1].in64 : a.p[0].in64;
    const float* __restrict__ W = which ? a.p[1].W : a.p[0].W;
    const float* __restrict__ bias = which ? a.p[1].bias : a.p[0].bias;
    double* __restrict__ out = which ? a.p[1].out : a.p[0].out;
    const int in_dim = which ? a.p[1].in_dim : a.p[0].in_dim;
    const int out_dim = which ? a.p[1].out_dim : a.p[0].out_dim;
    const int last = which ? a.p[1].last : a.p[0].last;
    const float* __restrict__ h = a.h;
    const int32_t* __restrict__ rows = a.rows;
    const int B = a.B, act = a.act;
    // FO output units x FB samples per workgroup: a lane's weights and inputs are each loaded once and meet
    // in FO * FB accumulators.  Per (sample, unit) the sum is what it was with one unit per workgroup: lane-
    // strided over a quarter of the inputs per wavefront, butterfly, the four quarters in order.
    __shared__ double part[4][FO][FB];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int ogroups = (out_dim + FO - 1) / FO;
    const int bg = (int)(block / ogroups), og = (int)(block % ogroups);
    const float* w[FO];
#pragma unroll
    for (int u = 0; u < FO; ++u) w[u] = W + (size_t)min(og * FO + u, out_dim - 1) * in_dim;   // clamped duplicates are not stored
    const float* hrow[FB];
    const double* drow[FB];
#pragma unroll
    for (int q = 0; q < FB; ++q) {
        const int b = min(bg * FB + q, B - 1);
        hrow[q] = in64 ? nullptr : h + (size_t)clamp_index(rows[b], a.T) * in_dim;
        drow[q] = in64 ? in64 + (size_t)b * in_dim : nullptr;
    }
    const int quarter = (in_dim + 3) / 4;
    const int i_end = min(in_dim, (wave + 1) * quarter);
    double acc[FO][FB];
#pragma unroll
    for (int u = 0; u < FO; ++u)
#pragma unroll
        for (int q = 0; q < FB; ++q) acc[u][q] = 0.0;
#pragma unroll 2
    for (int i = wave * quarter + lane; i < i_end; i += 64) {
        double wi[FO], xi[FB];
#pragma unroll
        for (int u = 0; u < FO; ++u) wi[u] = (double)w[u][i];
#pragma unroll
        for (int q = 0; q < FB; ++q) xi[q] = in64 ? drow[q][i] : (double)hrow[q][i];
#pragma unroll
        for (int u = 0; u < FO; ++u)
#pragma unroll
            for (int q = 0; q < FB; ++q) acc[u][q] += wi[u] * xi[q];
    }
#pragma unroll
    for (int u = 0; u < FO; ++u)
#pragma unroll
        for (int q = 0; q < FB; ++q) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) acc[u][q] += __shfl_xor(acc[u][q], off, 64);
        }
    if (lane == 0) {
#pragma unroll
        for (int u = 0; u < FO; ++u)
#pragma unroll
            for (int q = 0; q < FB; ++q) part[wave][u][q] = acc[u][q];
    }
    __syncthreads();
    if (threadIdx.x < FO * FB) {
        const int u = threadIdx.x / FB, q = threadIdx.x % FB;
        const int b = bg * FB + q, o = og * FO + u;
        if (b < B && o < out_dim) {
            double z = ((part[0][u][q] + part[1][u][q]) + part[2][u][q]) + part[3][u][q] + (double)bias[o];
            if (!last) z = (act == BRL_ACT_RELU) ? fmax(z, 0.0) : tanh(z);
            out[(size_t)b * out_dim + o] = z;
        }
    }
}

struct LossArgs {
    const double* logits;     // [B, A]
    const double* v;          // [B]
    const int32_t* rows;      // [B] indices into the rollout
    const int32_t* actions;
    const float* logp_old;
    const float* adv;
    const float* returns;
    int B, A, T;
    double clip_eps, ent_coef, adv_eps;
    int normalize_adv;
    double* dlogits;          // [B, A]
    double* dv;               // [B]
    float* stats;             // [5]: policy loss, value loss, entropy, clip fraction, (gradient norm: written later) or null
    double* row_terms;        // [4, B] scratch
};

// One workgroup: advantage normalisation over the mini-batch, then one thread per sample for the
// clipped surrogate (Eq. 1), the entropy bonus and the value error, and their gradients at the heads' outputs.
__global__ __launch_bounds__(256) void ppo_loss_kernel(LossArgs a) {
    __shared__ double s_mean, s_inv;
    __shared__ double red[256];
    if (a.normalize_adv) {
        // mean and (n - 1) standard deviation over the mini-batch: strided partial sums, then a fixed tree
        double part = 0.0;
        for (int b = threadIdx.x; b < a.B; b += 256) part += (double)a.adv[clamp_index(a.rows[b], a.T)];
        red[threadIdx.x] = part;
        __syncthreads();
        for (int st = 128; st >= 1; st >>= 1) {
            if ((int)threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
            __syncthreads();
        }
        const double mean = red[0] / (double)a.B;
        __syncthreads();
        part = 0.0;
        for (int b = threadIdx.x; b < a.B; b += 256) {
            const double d = (double)a.adv[clamp_index(a.rows[b], a.T)] - mean;
            part += d * d;
        }
        red[threadIdx.x] = part;
        __syncthreads();
        for (int st = 128; st >= 1; st >>= 1) {
            if ((int)threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            const double sd = a.B > 1 ? sqrt(red[0] / (double)(a.B - 1)) : 0.0;
            s_mean = mean;
            s_inv = 1.0 / (sd + a.adv_eps);
        }
    } else if (threadIdx.x == 0) {
        s_mean = 0.0;
        s_inv = 1.0;
    }
    __syncthreads();
    // LG adjacent lanes share a sample: each takes every LG-th action; maxima and sums meet by butterfly
    constexpr int LG = 4;
    const int part = threadIdx.x % LG;
    for (int b0 = 0; b0 < a.B; b0 += 256 / LG) {
        const int b = b0 + (int)threadIdx.x / LG;
        const bool live = b < a.B;
        const int bc = live ? b : a.B - 1;              // idle lanes shadow the last sample and store nothing
        const int r = clamp_index(a.rows[bc], a.T);
        const double A = ((double)a.adv[r] - s_mean) * s_inv;
        const double* z = a.logits + (size_t)bc * a.A;
        double m = z[0];
        for (int k = part; k < a.A; k += LG) m = fmax(m, z[k]);
#pragma unroll
        for (int off = 1; off < LG; off <<= 1) m = fmax(m, __shfl_xor(m, off, 64));
        double se = 0.0;
        for (int k = part; k < a.A; k += LG) se += exp(z[k] - m);
#pragma unroll
        for (int off = 1; off < LG; off <<= 1) se += __shfl_xor(se, off, 64);
        const double lse = m + log(se);
        const int act = clamp_index(a.actions[r], a.A);
        const double logp = z[act] - lse;
        const double ratio = exp(logp - (double)a.logp_old[r]);
        const double surr1 = ratio * A;
        const double clipped = fmin(fmax(ratio, 1.0 - a.clip_eps), 1.0 + a.clip_eps);
        const double surr2 = clipped * A;
        const double active = surr1 <= surr2 ? 1.0 : 0.0;
        double ent = 0.0;
        for (int k = part; k < a.A; k += LG) {
            const double lp = z[k] - lse;
            ent -= exp(lp) * lp;
        }
#pragma unroll
        for (int off = 1; off < LG; off <<= 1) ent += __shfl_xor(ent, off, 64);
        const double coef = -(active * A * ratio);
        if (live) {
            for (int k = part; k < a.A; k += LG) {
                const double lp = z[k] - lse, p = exp(lp);
                a.dlogits[(size_t)b * a.A + k] = (coef * ((k == act ? 1.0 : 0.0) - p) + a.ent_coef * p * (lp + ent)) / (double)a.B;
            }
            if (part == 0) {
                const double diff = a.v[b] - (double)a.returns[r];
                a.dv[b] = diff / (double)a.B;
                a.row_terms[0 * a.B + b] = fmin(surr1, surr2);
                a.row_terms[1 * a.B + b] = ent;
                a.row_terms[2 * a.B + b] = diff * diff;
                a.row_terms[3 * a.B + b] = 1.0 - active;
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0 && a.stats) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        for (int b = 0; b < a.B; ++b) {
            s0 += a.row_terms[0 * a.B + b];
            s1 += a.row_terms[1 * a.B + b];
            s2 += a.row_terms[2 * a.B + b];
            s3 += a.row_terms[3 * a.B + b];
        }
        const double n = (double)a.B;
        a.stats[0] = (float)(-s0 / n - a.ent_coef * s1 / n);
        a.stats[1] = (float)(0.5 * s2 / n);
        a.stats[2] = (float)(s1 / n);
        a.stats[3] = (float)(s3 / n);
    }
}

// dW[o, i] = sum_b delta[b, o] in(b, i), db[o] = sum_b delta[b, o].  A wavefront takes GO output units and 64
// consecutive inputs and sums over the samples in order; the four wavefronts of a workgroup take neighbouring
// input chunks and share nothing.  The squares of a wavefront's gradients are summed (fixed tree) to one slot
// of partial[] for the global norm.
constexpr int GO = 4;
struct GradProblem {
    const double* delta;
    const double* in64;      // null: first layer, inputs are rows of h
    double* gW;
    double* gb;
    double* partial;
    int in_dim, out_dim;
    unsigned blocks;
};
struct GradArgs {
    GradProblem p[2];
    int n;
    const float* h;
    const int32_t* rows;
    int B, T;
};
__global__ __launch_bounds__(256) void ppo_weight_grad_kernel(GradArgs a) {
    const int which = (a.n > 1 && blockIdx.x >= a.p[0].blocks) ? 1 : 0;
    const unsigned block = blockIdx.x - (which ? a.p[0].blocks : 0u);
    const double* __restrict__ delta = which ? a.p[1].delta : a.p[0].delta;
    const double* __restrict__ in64 = which ? a.p[1].in64 : a.p[0].in64;
    double* __restrict__ gW = which ? a.p[1].gW : a.p[0].gW;
    double* __restrict__ gb = which ? a.p[1].gb : a.p[0].gb;
    double* __restrict__ partial = which ? a.p[1].partial : a.p[0].partial;
    const int in_dim = which ? a.p[1].in_dim : a.p[0].in_dim;
    const int out_dim = which ? a.p[1].out_dim : a.p[0].out_dim;
    const float* __restrict__ h = a.h;
    const int32_t* __restrict__ rows = a.rows;
    const int B = a.B;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int ichunks = (in_dim + 63) / 64;
    const int cpw = (ichunks + 3) / 4;                 // groups of four input chunks, one chunk per wavefront
    const int og = (int)(block / cpw), chunk = (int)(block % cpw) * 4 + wave;
    if (chunk >= ichunks) return;
    const int o0 = og * GO;
    const int i = chunk * 64 + lane;
    const int ii = min(i, in_dim - 1);
    double acc[GO], accb[GO];
#pragma unroll
    for (int q = 0; q < GO; ++q) { acc[q] = 0.0; accb[q] = 0.0; }
#pragma unroll 8
    for (int b = 0; b < B; ++b) {
        const double x = in64 ? in64[(size_t)b * in_dim + ii] : (double)h[(size_t)clamp_index(rows[b], a.T) * in_dim + ii];
#pragma unroll
        for (int q = 0; q < GO; ++q) {
            const double d = delta[(size_t)b * out_dim + min(o0 + q, out_dim - 1)];
            acc[q] += d * x;
            accb[q] += d;
        }
    }
    double sq = 0.0;
#pragma unroll
    for (int q = 0; q < GO; ++q) {
        if (o0 + q < out_dim && i < in_dim) {
            gW[(size_t)(o0 + q) * in_dim + i] = acc[q];
            sq += acc[q] * acc[q];
            if (i == 0) {
                gb[o0 + q] = accb[q];
                sq += accb[q] * accb[q];
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off, 64);
    if (lane == 0) partial[og * ichunks + chunk] = sq;
}

// delta_prev[b, i] = (sum_o delta[b, o] W[o, i]) * act'(a[b, i]), a = the activated output of the layer below
struct DeltaProblem {
    const double* delta;
    const float* W;
    const double* a_prev;
    double* delta_prev;
    int in_dim, out_dim;
    unsigned blocks;
};
struct DeltaArgs {
    DeltaProblem p[2];
    int n, B, act;
};
__global__ __launch_bounds__(256) void ppo_delta_kernel(DeltaArgs a) {
    const int which = (a.n > 1 && blockIdx.x >= a.p[0].blocks) ? 1 : 0;
    const unsigned block = blockIdx.x - (which ? a.p[0].blocks : 0u);
    const double* __restrict__ delta = which ? a.p[1].delta : a.p[0].delta;
    const float* __restrict__ W = which ? a.p[1].W : a.p[0].W;
    const double* __restrict__ a_prev = which ? a.p[1].a_prev : a.p[0].a_prev;
    double* __restrict__ delta_prev = which ? a.p[1].delta_prev : a.p[0].delta_prev;
    const int in_dim = which ? a.p[1].in_dim : a.p[0].in_dim;
    const int out_dim = which ? a.p[1].out_dim : a.p[0].out_dim;
    const int B = a.B, act = a.act;
    const size_t idx = (size_t)block * 256 + threadIdx.x;
    if (idx >= (size_t)B * in_dim) return;
    const int b = (int)(idx / in_dim), i = (int)(idx % in_dim);
    double acc = 0.0;
    for (int o = 0; o < out_dim; ++o) acc += delta[(size_t)b * out_dim + o] * (double)W[(size_t)o * in_dim + i];
    const double av = a_prev[idx];
    delta_prev[idx] = acc * (act == BRL_ACT_RELU ? (av > 0.0 ? 1.0 : 0.0) : 1.0 - av * av);
}

// scal[0] = global L2 norm of the gradients, scal[1] = min(1, max_norm / (norm + 1e-6)); the partial sums are
// added in a fixed order (thread t takes partials t, t + 256, ..., then a fixed tree): same result every run.
__global__ __launch_bounds__(256) void ppo_norm_kernel(const double* __restrict__ partial, int n, double max_norm,
                                                        double* __restrict__ scal, float* __restrict__ stats) {
    __shared__ double red[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int st = 128; st >= 1; st >>= 1) {
        if ((int)threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double norm = sqrt(red[0]);
        scal[0] = norm;
        scal[1] = fmin(1.0, max_norm / (norm + 1e-6));
        if (stats) stats[4] = (float)norm;
    }
}

// Adam with bias correction on the clipped gradient: p -= lr (m / c1) / (sqrt(v / c2) + eps)
__global__ __launch_bounds__(256) void ppo_adam_kernel(float* __restrict__ p, float* __restrict__ m, float* __restrict__ v,
                                                        const double* __restrict__ g, const double* __restrict__ scal,
                                                        size_t n, size_t n_policy, double lr_policy, double lr_value,
                                                        double b1, double b2, double c1, double c2, double eps) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const double gi = g[i] * scal[1];
    const double mi = b1 * (double)m[i] + (1.0 - b1) * gi;
    const double vi = b2 * (double)v[i] + (1.0 - b2) * gi * gi;
    m[i] = (float)mi;
    v[i] = (float)vi;
    const double lr = i < n_policy ? lr_policy : lr_value;
    p[i] = (float)((double)p[i] - lr * (mi / c1) / (sqrt(vi / c2) + eps));
}

// ---- workspace ---------------------------------------------------------------------------------

struct PpoWs {
    size_t act_off[2][PPO_MAX_LAYERS];   // layer outputs [batch, dims[l+1]] fp64
    size_t delta_off[2][2];              // ping-pong deltas per head [batch, max_dim] fp64
    size_t dv_off, grad_off, partial_off, scal_off, rows_off, total;
    int n_partials;
    int partial_first[2][PPO_MAX_LAYERS];
};

constexpr size_t PPO_ALIGN = 256;

PpoWs ppo_ws_layout(const Layout& L, int batch) {
    PpoWs W;
    memset(&W, 0, sizeof(W));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up_sz(bytes, PPO_ALIGN);
        return at;
    };
    for (int hd = 0; hd < 2; ++hd)
        for (int l = 0; l < L.head[hd].n; ++l) W.act_off[hd][l] = take((size_t)batch * L.head[hd].dims[l + 1] * 8);
    for (int hd = 0; hd < 2; ++hd)
        for (int k = 0; k < 2; ++k) W.delta_off[hd][k] = take((size_t)batch * L.max_dim * 8);
    W.dv_off = take((size_t)batch * 8);
    W.grad_off = take(L.n_params * 8);
    int np = 0;
    for (int hd = 0; hd < 2; ++hd)
        for (int l = 0; l < L.head[hd].n; ++l) {
            W.partial_first[hd][l] = np;
            np += ((L.head[hd].dims[l + 1] + GO - 1) / GO) * ((L.head[hd].dims[l] + 63) / 64);
        }
    W.n_partials = np;
    W.partial_off = take((size_t)np * 8);
    W.scal_off = take(2 * 8);
    W.rows_off = take((size_t)4 * batch * 8);
    W.total = off;
    return W;
}

}  // namespace

}  // namespace brl

using namespace brl;

extern "C" {

size_t brl_ppo_param_count(const brl_ppo_config* cfg) {
    Layout L;
    if (make_layout(cfg, L) != BRL_OK) return 0;
    return L.n_params;
}

int brl_ppo_param_offsets(const brl_ppo_config* cfg, size_t* w_offsets, size_t* b_offsets) {
    Layout L;
    if (int rc = make_layout(cfg, L)) return rc;
    BRL_REQUIRE(w_offsets && b_offsets, "ppo_param_offsets: null pointer");
    int k = 0;
    for (int hd = 0; hd < 2; ++hd)
        for (int l = 0; l < L.head[hd].n; ++l, ++k) {
            w_offsets[k] = L.head[hd].w_off[l];
            b_offsets[k] = L.head[hd].b_off[l];
        }
    return BRL_OK;
}

size_t brl_ppo_workspace_bytes(const brl_ppo_config* cfg, int batch) {
    Layout L;
    if (batch < 1 || make_layout(cfg, L) != BRL_OK) return 0;
    return ppo_ws_layout(L, batch).total;
}

int ppo_gae(const float* rewards, const float* values, const float* dones, const float* last_value, int n_envs, int T,
            float gamma, float lam, float* adv, float* returns, void* stream) {
    BRL_REQUIRE(rewards && values && dones && last_value && adv && returns, "ppo_gae: null pointer");
    BRL_REQUIRE(n_envs >= 1 && T >= 1, "ppo_gae: n_envs = %d, T = %d", n_envs, T);
    BRL_REQUIRE(gamma >= 0.f && gamma <= 1.f && lam >= 0.f && lam <= 1.f, "ppo_gae: gamma and lambda must lie in [0, 1]");
    hipStream_t s = static_cast<hipStream_t>(stream);
    LaunchTimer tm(BRL_KC_OTHER, s);
    hipLaunchKernelGGL(gae_kernel, dim3((n_envs + 63) / 64), dim3(64), 0, s, rewards, values, dones, last_value, n_envs, T,
                       (double)gamma, (double)lam, adv, returns);
    BRL_LAUNCH_CHECK("gae_kernel");
    return BRL_OK;
}

int ppo_head_update(const brl_ppo_config* cfg, float* params, float* adam_m, float* adam_v, long long* adam_step,
                    const float* h, const int32_t* actions, const float* logp_old, const float* adv, const float* returns,
                    int T, const int32_t* perm, int epochs, int batch, float* stats, void* workspace, size_t ws_bytes,
                    void* stream) {
    Layout L;
    if (int rc = make_layout(cfg, L)) return rc;
    BRL_REQUIRE(params && adam_m && adam_v && adam_step && h && actions && logp_old && adv && returns && perm && workspace,
                "ppo_head_update: null pointer");
    BRL_REQUIRE(T >= 1 && epochs >= 0 && batch >= 1 && batch <= T, "ppo_head_update: T = %d, epochs = %d, batch = %d", T,
                epochs, batch);
    BRL_REQUIRE(*adam_step >= 0, "ppo_head_update: negative step count");
    BRL_REQUIRE(!cfg->normalize_adv || batch >= 2, "ppo_head_update: advantage normalisation needs batch >= 2");
    BRL_REQUIRE(cfg->clip_eps >= 0.f && cfg->max_grad_norm > 0.f && cfg->adam_eps > 0.f && cfg->adam_b1 >= 0.f &&
                    cfg->adam_b1 < 1.f && cfg->adam_b2 >= 0.f && cfg->adam_b2 < 1.f && cfg->adv_eps >= 0.f,
                "ppo_head_update: bad hyper-parameter");
    const PpoWs W = ppo_ws_layout(L, batch);
    if (ws_bytes < W.total) {
        set_error("ppo_head_update: workspace %zu < %zu", ws_bytes, W.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    double* grads = reinterpret_cast<double*>(base + W.grad_off);
    double* partial = reinterpret_cast<double*>(base + W.partial_off);
    double* scal = reinterpret_cast<double*>(base + W.scal_off);
    double* dv = reinterpret_cast<double*>(base + W.dv_off);
    double* delta[2][2];
    for (int hd = 0; hd < 2; ++hd)
        for (int k = 0; k < 2; ++k) delta[hd][k] = reinterpret_cast<double*>(base + W.delta_off[hd][k]);
    const int A = L.head[0].dims[L.head[0].n];
    const int steps_per_epoch = T / batch;
    LaunchTimer tm(BRL_KC_OTHER, s);
    long long step = *adam_step;
    for (int e = 0; e < epochs; ++e) {
        for (int mb = 0; mb < steps_per_epoch; ++mb) {
            const int32_t* rows = perm + (size_t)e * T + (size_t)mb * batch;
            float* st = stats ? stats + ((size_t)e * steps_per_epoch + mb) * 5 : nullptr;
            // forward: level l of both heads in one launch
            const int depth = L.head[0].n > L.head[1].n ? L.head[0].n : L.head[1].n;
            for (int l = 0; l < depth; ++l) {
                FwdArgs fa;
                memset(&fa, 0, sizeof(fa));
                fa.h = h; fa.rows = rows; fa.B = batch; fa.act = cfg->act; fa.T = T;
                unsigned blocks = 0;
                for (int hd = 0; hd < 2; ++hd) {
                    const HeadShape& H = L.head[hd];
                    if (l >= H.n) continue;
                    FwdProblem& P = fa.p[fa.n++];
                    P.in64 = l == 0 ? nullptr : reinterpret_cast<const double*>(base + W.act_off[hd][l - 1]);
                    P.W = params + H.w_off[l];
                    P.bias = params + H.b_off[l];
                    P.out = reinterpret_cast<double*>(base + W.act_off[hd][l]);
                    P.in_dim = H.dims[l]; P.out_dim = H.dims[l + 1]; P.last = l == H.n - 1 ? 1 : 0;
                    P.blocks = (unsigned)(((batch + FB - 1) / FB) * ((H.dims[l + 1] + FO - 1) / FO));
                    blocks += P.blocks;
                }
                hipLaunchKernelGGL(ppo_forward_kernel, dim3(blocks), dim3(256), 0, s, fa);
            }
            // gradients at the outputs
            LossArgs la;
            la.logits = reinterpret_cast<const double*>(base + W.act_off[0][L.head[0].n - 1]);
            la.v = reinterpret_cast<const double*>(base + W.act_off[1][L.head[1].n - 1]);
            la.rows = rows; la.actions = actions; la.logp_old = logp_old; la.adv = adv; la.returns = returns;
            la.B = batch; la.A = A; la.T = T;
            la.clip_eps = (double)cfg->clip_eps; la.ent_coef = (double)cfg->ent_coef; la.adv_eps = (double)cfg->adv_eps;
            la.normalize_adv = cfg->normalize_adv;
            la.dlogits = delta[0][0];
            la.dv = dv;
            la.stats = st;
            la.row_terms = reinterpret_cast<double*>(base + W.rows_off);
            hipLaunchKernelGGL(ppo_loss_kernel, dim3(1), dim3(256), 0, s, la);
            // backward: the same distance from the output of both heads in one launch; each head ping-pongs
            // between its own two delta buffers (the policy head's first one holds dlogits)
            const double* dcur[2] = {delta[0][0], dv};
            int pp[2] = {1, 0};
            for (int t = 0; t < depth; ++t) {
                GradArgs ga;
                DeltaArgs da;
                memset(&ga, 0, sizeof(ga));
                memset(&da, 0, sizeof(da));
                ga.h = h; ga.rows = rows; ga.B = batch; ga.T = T;
                da.B = batch; da.act = cfg->act;
                unsigned gblocks = 0, dblocks = 0;
                const double* dnext[2] = {dcur[0], dcur[1]};
                for (int hd = 0; hd < 2; ++hd) {
                    const HeadShape& H = L.head[hd];
                    const int l = H.n - 1 - t;
                    if (l < 0) continue;
                    const double* in64 = l == 0 ? nullptr : reinterpret_cast<const double*>(base + W.act_off[hd][l - 1]);
                    GradProblem& G = ga.p[ga.n++];
                    G.delta = dcur[hd]; G.in64 = in64;
                    G.gW = grads + H.w_off[l]; G.gb = grads + H.b_off[l];
                    G.partial = partial + W.partial_first[hd][l];
                    G.in_dim = H.dims[l]; G.out_dim = H.dims[l + 1];
                    G.blocks = (unsigned)(((H.dims[l + 1] + GO - 1) / GO) * (((H.dims[l] + 63) / 64 + 3) / 4));
                    gblocks += G.blocks;
                    if (l > 0) {
                        DeltaProblem& D = da.p[da.n++];
                        D.delta = dcur[hd]; D.W = params + H.w_off[l]; D.a_prev = in64;
                        D.delta_prev = delta[hd][pp[hd]];
                        D.in_dim = H.dims[l]; D.out_dim = H.dims[l + 1];
                        D.blocks = (unsigned)(((size_t)batch * H.dims[l] + 255) / 256);
                        dblocks += D.blocks;
                        dnext[hd] = D.delta_prev;
                        pp[hd] ^= 1;
                    }
                }
                hipLaunchKernelGGL(ppo_weight_grad_kernel, dim3(gblocks), dim3(256), 0, s, ga);
                if (da.n > 0) hipLaunchKernelGGL(ppo_delta_kernel, dim3(dblocks), dim3(256), 0, s, da);
                dcur[0] = dnext[0];
                dcur[1] = dnext[1];
            }
            hipLaunchKernelGGL(ppo_norm_kernel, dim3(1), dim3(256), 0, s, partial, W.n_partials, (double)cfg->max_grad_norm, scal, st);
            ++step;
            const double c1 = 1.0 - pow((double)cfg->adam_b1, (double)step);
            const double c2 = 1.0 - pow((double)cfg->adam_b2, (double)step);
            hipLaunchKernelGGL(ppo_adam_kernel, dim3((unsigned)((L.n_params + 255) / 256)), dim3(256), 0, s, params, adam_m, adam_v,
                               grads, scal, L.n_params, L.n_policy, (double)cfg->lr_policy, (double)cfg->lr_value,
                               (double)cfg->adam_b1, (double)cfg->adam_b2, c1, c2, (double)cfg->adam_eps);
        }
    }
    BRL_LAUNCH_CHECK("ppo_head_update");
    *adam_step = step;
    return BRL_OK;
}

}  // extern "C"
