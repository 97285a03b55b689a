// C ABI of the library (see include/bitrl.h): argument checks, workspace
// carving and kernel sequencing.  No arithmetic of the method happens here.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "common.hpp"

namespace brl {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char* what) {
    set_error("HIP error %d (%s) at %s", (int)e, hipGetErrorString(e), what);
    return BRL_EHIP;
}

// ---- launch timing ----
namespace {
std::mutex g_tm_mu;
bool g_tm_on = false;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_tm_events[BRL_KC_COUNT];
std::vector<hipEvent_t> g_tm_free;
double g_tm_ops[BRL_KC_COUNT];

hipEvent_t tm_get_event() {
    if (!g_tm_free.empty()) {
        hipEvent_t e = g_tm_free.back();
        g_tm_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

LaunchTimer::LaunchTimer(int kernel_class, hipStream_t s, double int8_ops) : stop_(nullptr), s_(s), on_(false) {
    std::lock_guard<std::mutex> lk(g_tm_mu);
    if (!g_tm_on) return;
    hipEvent_t a = tm_get_event(), b = tm_get_event();
    if (!a || !b) return;
    (void)hipEventRecord(a, s);
    g_tm_events[kernel_class].push_back(std::make_pair(a, b));
    g_tm_ops[kernel_class] += int8_ops;
    stop_ = b;
    on_ = true;
}

LaunchTimer::~LaunchTimer() {
    if (on_) (void)hipEventRecord(stop_, s_);
}

namespace {

constexpr size_t ALIGN = 256;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Carver {
    char* base;
    size_t off;
    explicit Carver(void* p) : base(static_cast<char*>(p)), off(0) {}
    template <class T>
    T* take(size_t count) {
        T* r = reinterpret_cast<T*>(base + off);
        off += round_up_sz(count * sizeof(T), ALIGN);
        return r;
    }
};

size_t actbuf_bytes(int M, int K) {
    const size_t Mp = round_up(M, NB), Kp = round_up(K, SBK);
    return round_up_sz(Mp * Kp, ALIGN) + 3 * round_up_sz(Mp * 4, ALIGN) + round_up_sz(splitk_capacity_ints(M) * 4, ALIGN);
}

ActBuf take_actbuf(Carver& c, int M, int K) {
    const size_t Mp = round_up(M, NB), Kp = round_up(K, SBK);
    ActBuf a;
    a.q = c.take<int8_t>(Mp * Kp);
    a.absmax = c.take<float>(Mp);
    a.dscale = c.take<float>(Mp);
    a.sumq = c.take<int32_t>(Mp);
    a.splitk_ints = splitk_capacity_ints(M);
    a.splitk = a.splitk_ints ? c.take<int32_t>(a.splitk_ints) : nullptr;
    return a;
}

int check_linear_shape(int N, int K, const char* who) {
    BRL_REQUIRE(N >= 1 && K >= 1, "%s: N = %d, K = %d must be positive", who, N, K);
    BRL_REQUIRE(K % 8 == 0, "%s: K = %d must be a multiple of 8", who, K);
    BRL_REQUIRE(K <= MAX_K, "%s: K = %d exceeds the supported %d", who, K, MAX_K);
    return BRL_OK;
}

WeightSegs one_seg(const void* packed, const float* beta, int N, int w8 = 0) {
    WeightSegs w;
    memset(&w, 0, sizeof(w));
    w.count = 1;
    w.w8 = w8;
    w.packed[0] = static_cast<const uint32_t*>(packed);
    w.beta[0] = beta;
    w.nb_end[0] = round_up(N, NB) / NB;
    w.n_end[0] = N;
    return w;
}

void add_seg(WeightSegs& w, const void* packed, const float* beta, int N) {
    const int i = w.count++;
    w.packed[i] = static_cast<const uint32_t*>(packed);
    w.beta[i] = beta;
    w.nb_end[i] = (i ? w.nb_end[i - 1] : 0) + round_up(N, NB) / NB;
    w.n_end[i] = (i ? w.n_end[i - 1] : 0) + N;
}

// the quantised activations of the MFMA path (the 1..4 token path needs no scratch)
struct BitlinearWs {
    size_t act_off, total;
};

BitlinearWs bitlinear_ws_layout(int M, int N, int K) {
    BitlinearWs L;
    (void)N;
    L.act_off = 0;
    L.total = L.act_off + actbuf_bytes(M, K);
    return L;
}

struct FfnWs {
    size_t act1_off, gu_off, act2_off, total;
};

FfnWs ffn_ws_layout(int M, int d, int f) {
    FfnWs L;
    L.act1_off = 0;
    L.gu_off = L.act1_off + actbuf_bytes(M, d);
    L.act2_off = L.gu_off + round_up_sz((size_t)M * f * 4, ALIGN);
    L.total = L.act2_off + actbuf_bytes(M, f);
    return L;
}

int check_ffn(const brl_ffn_weights* w, int d, int f, const char* who) {
    BRL_REQUIRE(w != nullptr, "%s: null weights", who);
    BRL_REQUIRE(w->norm_g && w->gate_packed && w->gate_beta && w->up_packed && w->up_beta && w->subln_g &&
                    w->down_packed && w->down_beta,
                "%s: null pointer in brl_ffn_weights", who);
    BRL_REQUIRE(aligned16(w->norm_g) && aligned16(w->gate_packed) && aligned16(w->up_packed) && aligned16(w->subln_g) &&
                    aligned16(w->down_packed),
                "%s: weight pointers must be 16-byte aligned", who);
    if (int rc = check_linear_shape(f, d, who)) return rc;
    if (int rc = check_linear_shape(d, f, who)) return rc;
    return BRL_OK;
}

// shared by ffn_block_forward and encoder_forward: x [M, d] fp32 -> y = x + down(...)
int run_ffn(const brl_ffn_weights* w, int w8, const float* x32, const void* xin, int x_dtype, int M, int d, int f,
            float eps_norm, float eps_act, float* y, const ActBuf& act1, float* gu, const ActBuf& act2, hipStream_t s) {
    QuantArgs qa;
    memset(&qa, 0, sizeof(qa));
    qa.x = xin; qa.x_dtype = x_dtype; qa.gain = w->norm_g;
    qa.eps_norm = eps_norm; qa.eps_act = eps_act; qa.M = M; qa.K = d;
    if (int rc = launch_act_quant(qa, act1, s)) return rc;
    WeightSegs gu_w;
    memset(&gu_w, 0, sizeof(gu_w));
    gu_w.w8 = w8;
    add_seg(gu_w, w->gate_packed, w->gate_beta, f);
    add_seg(gu_w, w->up_packed, w->up_beta, f);
    // gate | up GEMM with the squared-ReLU GLU in its epilogue: gu receives h [M, f]
    if (int rc = launch_gemm(act1, gu_w, M, 2 * f, d, gu, f, nullptr, nullptr, 1, s)) return rc;
    QuantArgs qb;
    memset(&qb, 0, sizeof(qb));
    qb.x = gu; qb.x_dtype = BRL_F32; qb.gain = w->subln_g;
    qb.eps_norm = eps_norm; qb.eps_act = eps_act; qb.M = M; qb.K = f;
    if (int rc = launch_act_quant(qb, act2, s)) return rc;
    const WeightSegs dn = one_seg(w->down_packed, w->down_beta, d, w8);
    // the residual is the block input itself: read as bf16 where the caller gave bf16 (no widened copy)
    if (x32 == nullptr) return launch_gemm(act2, dn, M, d, f, y, d, static_cast<const float*>(xin), nullptr, 0, s, 1);
    return launch_gemm(act2, dn, M, d, f, y, d, x32, nullptr, 0, s);
}

struct EncWs {
    int states_mb;      // states per micro-batch
    size_t x_off, act_off, big_off, cos_off, sin_off, rinv_off, frag_off, total;
    int big_ld_qkv;
    bool q_frags;       // the fragment area also has room for q fragments (q | k | v product with the attention-operand epilogue)
};

constexpr int ENC_MB_TOKENS = 32768;

EncWs encoder_ws_layout(const brl_encoder* e, int B, int S) {
    EncWs L;
    int smb = ENC_MB_TOKENS / S;
    if (smb < 1) smb = 1;
    if (smb > B) smb = B;
    L.states_mb = smb;
    const size_t Mt = (size_t)smb * S;
    const int dq = e->n_heads * e->head_dim, dkv = e->n_kv_heads * e->head_dim;
    int kmax = e->d;
    if (dq > kmax) kmax = dq;
    if (e->f > kmax) kmax = e->f;
    L.x_off = 0;
    L.act_off = round_up_sz(Mt * e->d * 4, ALIGN);
    L.big_off = L.act_off + actbuf_bytes((int)Mt, kmax);
    const size_t attn_cols = (size_t)dq + 2 * dkv + dq;      // qkv | attention output
    const size_t big_cols = attn_cols > (size_t)e->f ? attn_cols : (size_t)e->f;
    L.cos_off = L.big_off + round_up_sz(Mt * big_cols * 4, ALIGN);
    const size_t tbl = round_up_sz((size_t)S * (e->head_dim / 2) * 4, ALIGN);
    L.sin_off = L.cos_off + tbl;
    L.rinv_off = L.sin_off + tbl;
    L.frag_off = L.rinv_off + round_up_sz(Mt * 4, ALIGN);
    L.q_frags = e->attn_precision == BRL_ATTN_MFMA && e->weight_format != BRL_W_INT8 && e->head_dim == 128 && S % 32 == 0;
    L.total = L.frag_off +
              round_up_sz(attention_mfma_ws_bytes(smb, S, e->n_heads, e->n_kv_heads, e->head_dim, L.q_frags), ALIGN);
    L.big_ld_qkv = dq + 2 * dkv;
    return L;
}

int check_encoder(const brl_encoder* e) {
    BRL_REQUIRE(e != nullptr, "encoder: null config");
    BRL_REQUIRE(e->n_layers >= 0 && e->d >= 8 && e->n_heads >= 1 && e->n_kv_heads >= 1 && e->f >= 8 && e->vocab >= 1,
                "encoder: bad sizes");
    BRL_REQUIRE(e->n_heads % e->n_kv_heads == 0, "encoder: n_heads %d not a multiple of n_kv_heads %d", e->n_heads,
                e->n_kv_heads);
    BRL_REQUIRE(e->head_dim == 16 || e->head_dim == 32 || e->head_dim == 64 || e->head_dim == 100 || e->head_dim == 128,
                "encoder: head_dim %d not in {16, 32, 64, 100, 128}", e->head_dim);
    BRL_REQUIRE(e->d % 8 == 0 && e->f % 8 == 0 && (e->n_kv_heads * e->head_dim) % 4 == 0,
                "encoder: d and f must be multiples of 8");
    BRL_REQUIRE(e->attn_precision == BRL_ATTN_F32 || e->attn_precision == BRL_ATTN_MFMA,
                "encoder: unknown attn_precision %d", e->attn_precision);
    BRL_REQUIRE(e->weight_format == BRL_W_TERNARY || e->weight_format == BRL_W_INT8, "encoder: unknown weight_format %d",
                e->weight_format);
    const int dq = e->n_heads * e->head_dim;
    if (int rc = check_linear_shape(dq, e->d, "encoder")) return rc;
    if (int rc = check_linear_shape(e->d, dq, "encoder")) return rc;
    BRL_REQUIRE(e->embedding && e->final_norm_g && aligned16(e->embedding) && aligned16(e->final_norm_g),
                "encoder: embedding / final_norm_g null or misaligned");
    BRL_REQUIRE(e->n_layers == 0 || e->layers != nullptr, "encoder: null layer table");
    for (int l = 0; l < e->n_layers; ++l) {
        const brl_layer_weights& w = e->layers[l];
        BRL_REQUIRE(w.attn_norm_g && w.wq_packed && w.wq_beta && w.wk_packed && w.wk_beta && w.wv_packed && w.wv_beta &&
                        w.attn_subln_g && w.wo_packed && w.wo_beta,
                    "encoder: null pointer in layer %d", l);
        BRL_REQUIRE(aligned16(w.attn_norm_g) && aligned16(w.wq_packed) && aligned16(w.wk_packed) &&
                        aligned16(w.wv_packed) && aligned16(w.attn_subln_g) && aligned16(w.wo_packed),
                    "encoder: misaligned pointer in layer %d", l);
        if (int rc = check_ffn(&w.ffn, e->d, e->f, "encoder")) return rc;
    }
    return BRL_OK;
}

int check_mlp(const brl_mlp* m, const char* who, int out_expected) {
    BRL_REQUIRE(m->n_layers >= 1 && m->n_layers <= 8, "%s: n_layers %d out of 1..8", who, m->n_layers);
    BRL_REQUIRE(m->dims && m->W && m->b, "%s: null tables", who);
    for (int i = 0; i <= m->n_layers; ++i) BRL_REQUIRE(m->dims[i] >= 1, "%s: dims[%d] = %d", who, i, m->dims[i]);
    for (int i = 0; i < m->n_layers; ++i) BRL_REQUIRE(m->W[i] && m->b[i], "%s: null parameter in layer %d", who, i);
    BRL_REQUIRE(m->act == BRL_ACT_TANH || m->act == BRL_ACT_RELU, "%s: unknown activation %d", who, m->act);
    if (out_expected > 0)
        BRL_REQUIRE(m->dims[m->n_layers] == out_expected, "%s: output width %d, expected %d", who, m->dims[m->n_layers],
                    out_expected);
    return BRL_OK;
}

size_t mlp_hidden_max(const brl_mlp* m) {
    size_t mx = 1;
    for (int i = 1; i < m->n_layers; ++i)
        if ((size_t)m->dims[i] > mx) mx = (size_t)m->dims[i];
    return mx;
}

int run_mlp(const brl_mlp* m, const float* h, int B, float* out, double* buf0, double* buf1, hipStream_t s) {
    const double* in64 = nullptr;
    const float* in32 = h;
    double* bufs[2] = {buf0, buf1};
    for (int i = 0; i < m->n_layers; ++i) {
        const bool last = i + 1 == m->n_layers;
        double* o64 = last ? nullptr : bufs[i & 1];
        if (int rc = launch_mlp_layer(in64, in32, m->W[i], m->b[i], B, m->dims[i], m->dims[i + 1], m->act, o64,
                                      last ? out : nullptr, s))
            return rc;
        in64 = o64;
        in32 = nullptr;
    }
    return BRL_OK;
}

}  // namespace
}  // namespace brl

using namespace brl;

extern "C" {

const char* brl_last_error(void) { return g_err; }

int brl_abi_version(void) { return 2; }

int brl_timing_enable(int on) {
    std::lock_guard<std::mutex> lk(g_tm_mu);
    g_tm_on = on != 0;
    return BRL_OK;
}

int brl_timing_read(int kernel_class, long long* launches, double* total_ms) {
    double ops = 0.0;
    return brl_timing_read_ops(kernel_class, launches, total_ms, &ops);
}

int brl_timing_read_ops(int kernel_class, long long* launches, double* total_ms, double* int8_ops) {
    BRL_REQUIRE(kernel_class >= 0 && kernel_class < BRL_KC_COUNT, "timing_read: unknown class %d", kernel_class);
    BRL_REQUIRE(launches && total_ms && int8_ops, "timing_read: null pointer");
    std::vector<std::pair<hipEvent_t, hipEvent_t>> evs;
    {
        std::lock_guard<std::mutex> lk(g_tm_mu);
        evs.swap(g_tm_events[kernel_class]);
        *int8_ops = g_tm_ops[kernel_class];
        g_tm_ops[kernel_class] = 0.0;
    }
    double sum = 0.0;
    int rc = BRL_OK;
    for (auto& pr : evs) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(pr.second);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, pr.first, pr.second);
        if (e != hipSuccess && rc == BRL_OK) rc = hip_fail(e, "timing_read");
        sum += (double)ms;
    }
    {
        std::lock_guard<std::mutex> lk(g_tm_mu);
        for (auto& pr : evs) {
            g_tm_free.push_back(pr.first);
            g_tm_free.push_back(pr.second);
        }
    }
    *launches = (long long)evs.size();
    *total_ms = sum;
    return rc;
}

size_t brl_packed_bytes(int n_out, int k_in) {
    if (n_out < 1 || k_in < 1) return 0;
    return (size_t)round_up(n_out, NB) * (size_t)round_up(k_in, SBK) / 4;
}

size_t brl_quantize_workspace_bytes(int n_out, int k_in) {
    (void)n_out; (void)k_in;
    return 1024 * sizeof(double) + ALIGN;
}

int bitlinear_quantize_weights(const float* W, int n_out, int k_in, float eps, void* packed_out, float* beta_out,
                               int8_t* codes_dbg, void* workspace, size_t ws_bytes, void* stream) {
    BRL_REQUIRE(W && packed_out && beta_out && workspace, "quantize_weights: null pointer");
    BRL_REQUIRE(aligned16(W) && aligned16(packed_out) && aligned16(workspace), "quantize_weights: misaligned pointer");
    BRL_REQUIRE(n_out >= 1 && k_in >= 1, "quantize_weights: bad shape %d x %d", n_out, k_in);
    BRL_REQUIRE(eps >= 0.f, "quantize_weights: negative eps");
    if (ws_bytes < brl_quantize_workspace_bytes(n_out, k_in)) {
        set_error("quantize_weights: workspace %zu < %zu", ws_bytes, brl_quantize_workspace_bytes(n_out, k_in));
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver c(workspace);
    double* partials = c.take<double>(1024);
    int* flag = c.take<int>(1);
    if (int rc = launch_quantize_weights(W, n_out, k_in, eps, static_cast<uint32_t*>(packed_out), beta_out, codes_dbg,
                                         partials, flag, s))
        return rc;
    int bad = 0;
    BRL_HIP_CHECK(hipMemcpyAsync(&bad, flag, sizeof(int), hipMemcpyDeviceToHost, s));
    BRL_HIP_CHECK(hipStreamSynchronize(s));
    BRL_REQUIRE(bad == 0, "quantize_weights: mean|W| is not finite");
    return BRL_OK;
}

int brl_unpack_codes(const void* packed, int n_out, int k_in, int8_t* codes_out, void* stream) {
    BRL_REQUIRE(packed && codes_out && aligned16(packed), "unpack_codes: null or misaligned pointer");
    BRL_REQUIRE(n_out >= 1 && k_in >= 1, "unpack_codes: bad shape");
    return launch_unpack_codes(static_cast<const uint32_t*>(packed), n_out, k_in, codes_out,
                               static_cast<hipStream_t>(stream));
}

size_t brl_bitlinear_workspace_bytes(int M, int N, int K) {
    if (M < 1 || N < 1 || K < 1) return 0;
    return bitlinear_ws_layout(M, N, K).total;
}

int bitlinear_forward(const void* packed, const float* beta, int N, int K, const void* x, int x_dtype, int M,
                      float eps_act, float* y, const float* residual, int8_t* xq_dbg, float* absmax_dbg,
                      int32_t* acc_dbg, void* workspace, size_t ws_bytes, void* stream) {
    BRL_REQUIRE(packed && beta && x && y && workspace, "bitlinear_forward: null pointer");
    BRL_REQUIRE(aligned16(packed) && aligned16(x) && aligned16(y) && aligned16(workspace) &&
                    (!residual || aligned16(residual)),
                "bitlinear_forward: pointers must be 16-byte aligned");
    BRL_REQUIRE(M >= 1, "bitlinear_forward: M = %d", M);
    BRL_REQUIRE(x_dtype == BRL_F32 || x_dtype == BRL_BF16, "bitlinear_forward: unknown x_dtype %d", x_dtype);
    BRL_REQUIRE(eps_act > 0.f, "bitlinear_forward: eps_act must be positive");
    if (int rc = check_linear_shape(N, K, "bitlinear_forward")) return rc;
    const BitlinearWs L = bitlinear_ws_layout(M, N, K);
    if (ws_bytes < L.total) {
        set_error("bitlinear_forward: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    if (M <= 4) {
        return launch_gemv(x, x_dtype, M, K, N, static_cast<const uint32_t*>(packed), beta, eps_act, y, residual, xq_dbg,
                           absmax_dbg, acc_dbg, s);
    }
    Carver c(base + L.act_off);
    const ActBuf act = take_actbuf(c, M, K);
    QuantArgs qa;
    memset(&qa, 0, sizeof(qa));
    qa.x = x; qa.x_dtype = x_dtype; qa.gain = nullptr; qa.eps_norm = 0.f; qa.eps_act = eps_act;
    qa.M = M; qa.K = K; qa.xq_rowmajor = xq_dbg; qa.absmax_tap = absmax_dbg;
    if (int rc = launch_act_quant(qa, act, s)) return rc;
    const WeightSegs w = one_seg(packed, beta, N);
    return launch_gemm(act, w, M, N, K, y, N, residual, acc_dbg, 0, s);
}

// ---- bitlinear_forward for callers that cannot allocate: the quantised activations live in a
// file-scope device array instead of a caller workspace.  The array's name is only a host-side
// handle; its device address is looked up once per device and used from then on.
static __device__ __align__(256) unsigned char scratch[BRL_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES];     // device address of `scratch` on each device, 0 until first use there

int scratch_of_current_device(char** out) {
    int dev = -1;
    BRL_HIP_CHECK(hipGetDevice(&dev));
    BRL_REQUIRE(dev >= 0 && dev < MAX_DEVICES, "bitlinear_forward_static: device index %d not supported", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        BRL_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        BRL_REQUIRE(p != nullptr, "bitlinear_forward_static: no address for the scratch array on device %d", dev);
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char*>(g_scratch_ptr[dev]);
    return BRL_OK;
}

// the quantised activations alone: no k-split partial tiles (products that would cut k run uncut, same bits)
size_t static_actbuf_bytes(int M, int K) {
    const size_t Mp = round_up(M, NB), Kp = round_up(K, SBK);
    return round_up_sz(Mp * Kp, ALIGN) + 3 * round_up_sz(Mp * 4, ALIGN);
}
}  // namespace

int bitlinear_forward_static(const void* packed, const float* beta, int N, int K, const void* x, int x_dtype, int M,
                             float eps_act, float* y, const float* residual, int8_t* xq_dbg, float* absmax_dbg,
                             int32_t* acc_dbg, void* stream) {
    BRL_REQUIRE(packed && beta && x && y, "bitlinear_forward_static: null pointer");
    BRL_REQUIRE(aligned16(packed) && aligned16(x) && aligned16(y) && (!residual || aligned16(residual)),
                "bitlinear_forward_static: pointers must be 16-byte aligned");
    BRL_REQUIRE(M >= 1, "bitlinear_forward_static: M = %d", M);
    BRL_REQUIRE(x_dtype == BRL_F32 || x_dtype == BRL_BF16, "bitlinear_forward_static: unknown x_dtype %d", x_dtype);
    BRL_REQUIRE(eps_act > 0.f, "bitlinear_forward_static: eps_act must be positive");
    if (int rc = check_linear_shape(N, K, "bitlinear_forward_static")) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (M <= 4) {      // the 1..4 token path keeps everything in registers and LDS
        return launch_gemv(x, x_dtype, M, K, N, static_cast<const uint32_t*>(packed), beta, eps_act, y, residual, xq_dbg,
                           absmax_dbg, acc_dbg, s);
    }
    const size_t need = static_actbuf_bytes(M, K);
    if (need > (size_t)BRL_STATIC_SCRATCH_BYTES) {
        set_error("bitlinear_forward_static: %d tokens x %d features need %zu bytes of scratch, the built-in array holds %zu; "
                  "use bitlinear_forward with a workspace",
                  M, K, need, (size_t)BRL_STATIC_SCRATCH_BYTES);
        return BRL_ENOSPC;
    }
    char* base = nullptr;
    if (int rc = scratch_of_current_device(&base)) return rc;
    const size_t Mp = round_up(M, NB), Kp = round_up(K, SBK);
    Carver c(base);
    ActBuf act;
    act.q = c.take<int8_t>(Mp * Kp);
    act.absmax = c.take<float>(Mp);
    act.dscale = c.take<float>(Mp);
    act.sumq = c.take<int32_t>(Mp);
    act.splitk = nullptr;
    act.splitk_ints = 0;
    QuantArgs qa;
    memset(&qa, 0, sizeof(qa));
    qa.x = x; qa.x_dtype = x_dtype; qa.gain = nullptr; qa.eps_norm = 0.f; qa.eps_act = eps_act;
    qa.M = M; qa.K = K; qa.xq_rowmajor = xq_dbg; qa.absmax_tap = absmax_dbg;
    if (int rc = launch_act_quant(qa, act, s)) return rc;
    const WeightSegs w = one_seg(packed, beta, N);
    return launch_gemm(act, w, M, N, K, y, N, residual, acc_dbg, 0, s);
}

size_t brl_packed_int8_bytes(int n_out, int k_in) {
    if (n_out < 1 || k_in < 1) return 0;
    return (size_t)round_up(n_out, NB) * (size_t)round_up(k_in, SBK);
}

int bitlinear_quantize_weights_int8(const float* W, int n_out, int k_in, float eps, int qmax, void* packed_out,
                                    float* scale_out, int8_t* codes_dbg, void* workspace, size_t ws_bytes, void* stream) {
    BRL_REQUIRE(W && packed_out && scale_out && workspace, "quantize_weights_int8: null pointer");
    BRL_REQUIRE(aligned16(W) && aligned16(packed_out) && aligned16(workspace), "quantize_weights_int8: misaligned pointer");
    BRL_REQUIRE(n_out >= 1 && k_in >= 1, "quantize_weights_int8: bad shape %d x %d", n_out, k_in);
    BRL_REQUIRE(eps > 0.f, "quantize_weights_int8: eps must be positive");
    BRL_REQUIRE(qmax >= 1 && qmax <= 127, "quantize_weights_int8: qmax = %d out of 1..127", qmax);
    if (ws_bytes < brl_quantize_workspace_bytes(n_out, k_in)) {
        set_error("quantize_weights_int8: workspace %zu < %zu", ws_bytes, brl_quantize_workspace_bytes(n_out, k_in));
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver c(workspace);
    float* partials = c.take<float>(1024);
    int* flag = c.take<int>(1);
    if (int rc = launch_quantize_weights_int8(W, n_out, k_in, eps, qmax, static_cast<int8_t*>(packed_out), scale_out, codes_dbg,
                                              partials, flag, s))
        return rc;
    int bad = 0;
    BRL_HIP_CHECK(hipMemcpyAsync(&bad, flag, sizeof(int), hipMemcpyDeviceToHost, s));
    BRL_HIP_CHECK(hipStreamSynchronize(s));
    BRL_REQUIRE(bad == 0, "quantize_weights_int8: max|W| is not finite");
    return BRL_OK;
}

int brl_unpack_codes_int8(const void* packed, int n_out, int k_in, int8_t* codes_out, void* stream) {
    BRL_REQUIRE(packed && codes_out && aligned16(packed), "unpack_codes_int8: null or misaligned pointer");
    BRL_REQUIRE(n_out >= 1 && k_in >= 1, "unpack_codes_int8: bad shape");
    return launch_unpack_codes_int8(static_cast<const int8_t*>(packed), n_out, k_in, codes_out,
                                    static_cast<hipStream_t>(stream));
}

int bitlinear_int8_forward(const void* packed, const float* scale, int N, int K, const void* x, int x_dtype, int M,
                           float eps_act, float* y, const float* residual, int8_t* xq_dbg, float* absmax_dbg,
                           int32_t* acc_dbg, void* workspace, size_t ws_bytes, void* stream) {
    BRL_REQUIRE(packed && scale && x && y && workspace, "bitlinear_int8_forward: null pointer");
    BRL_REQUIRE(aligned16(packed) && aligned16(x) && aligned16(y) && aligned16(workspace) &&
                    (!residual || aligned16(residual)),
                "bitlinear_int8_forward: pointers must be 16-byte aligned");
    BRL_REQUIRE(M >= 1, "bitlinear_int8_forward: M = %d", M);
    BRL_REQUIRE(x_dtype == BRL_F32 || x_dtype == BRL_BF16, "bitlinear_int8_forward: unknown x_dtype %d", x_dtype);
    BRL_REQUIRE(eps_act > 0.f, "bitlinear_int8_forward: eps_act must be positive");
    if (int rc = check_linear_shape(N, K, "bitlinear_int8_forward")) return rc;
    const BitlinearWs L = bitlinear_ws_layout(M, N, K);
    if (ws_bytes < L.total) {
        set_error("bitlinear_int8_forward: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver c(static_cast<char*>(workspace) + L.act_off);
    const ActBuf act = take_actbuf(c, M, K);
    QuantArgs qa;
    memset(&qa, 0, sizeof(qa));
    qa.x = x; qa.x_dtype = x_dtype; qa.gain = nullptr; qa.eps_norm = 0.f; qa.eps_act = eps_act;
    qa.M = M; qa.K = K; qa.xq_rowmajor = xq_dbg; qa.absmax_tap = absmax_dbg;
    if (int rc = launch_act_quant(qa, act, s)) return rc;
    const WeightSegs w = one_seg(packed, scale, N, 1);
    return launch_gemm(act, w, M, N, K, y, N, residual, acc_dbg, 0, s);
}

int bitlinear_forward_batch(const void* const* packed, const float* const* beta, int N, int K, const void* const* x,
                            int x_dtype, int M, float eps_act, float* const* y, int count, void* stream) {
    BRL_REQUIRE(packed && beta && x && y, "bitlinear_forward_batch: null pointer array");
    BRL_REQUIRE(M >= 1 && M <= 4, "bitlinear_forward_batch: M = %d out of range 1..4", M);
    BRL_REQUIRE(count >= 0, "bitlinear_forward_batch: count = %d", count);
    BRL_REQUIRE(x_dtype == BRL_F32 || x_dtype == BRL_BF16, "bitlinear_forward_batch: unknown x_dtype %d", x_dtype);
    BRL_REQUIRE(eps_act > 0.f, "bitlinear_forward_batch: eps_act must be positive");
    if (int rc = check_linear_shape(N, K, "bitlinear_forward_batch")) return rc;
    return launch_gemv_batch(packed, beta, N, K, x, x_dtype, M, eps_act, y, count, static_cast<hipStream_t>(stream));
}

size_t brl_ffn_workspace_bytes(int M, int d, int f) {
    if (M < 1 || d < 1 || f < 1) return 0;
    return ffn_ws_layout(M, d, f).total;
}

int ffn_block_forward(const brl_ffn_weights* w, const void* x, int x_dtype, int M, int d, int f, float eps_norm,
                      float eps_act, float* y, void* workspace, size_t ws_bytes, void* stream) {
    if (int rc = check_ffn(w, d, f, "ffn_block_forward")) return rc;
    BRL_REQUIRE(x && y && workspace && aligned16(x) && aligned16(y) && aligned16(workspace),
                "ffn_block_forward: null or misaligned pointer");
    BRL_REQUIRE(x != (const void*)y, "ffn_block_forward: y must not alias x");
    BRL_REQUIRE(M >= 1, "ffn_block_forward: M = %d", M);
    BRL_REQUIRE(x_dtype == BRL_F32 || x_dtype == BRL_BF16, "ffn_block_forward: unknown x_dtype %d", x_dtype);
    BRL_REQUIRE(eps_act > 0.f && eps_norm >= 0.f, "ffn_block_forward: bad eps");
    const FfnWs L = ffn_ws_layout(M, d, f);
    if (ws_bytes < L.total) {
        set_error("ffn_block_forward: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    const float* x32 = x_dtype == BRL_BF16 ? nullptr : static_cast<const float*>(x);   // null: residual read as bf16
    Carver c1(base + L.act1_off);
    const ActBuf act1 = take_actbuf(c1, M, d);
    Carver c2(base + L.act2_off);
    const ActBuf act2 = take_actbuf(c2, M, f);
    float* gu = reinterpret_cast<float*>(base + L.gu_off);
    return run_ffn(w, 0, x32, x, x_dtype, M, d, f, eps_norm, eps_act, y, act1, gu, act2, s);
}

size_t brl_encoder_workspace_bytes(const brl_encoder* enc, int B, int S) {
    if (!enc || B < 1 || S < 1 || enc->d < 1 || enc->f < 1 || enc->head_dim < 2) return 0;
    return encoder_ws_layout(enc, B, S).total;
}

namespace {

// One micro-batch through embedding, all layers, final norm and pooling.  nb states, Mt token rows
// (nb * S in the uniform layout), S = rows per state or the bound on the state lengths.
int run_encoder_microbatch(const brl_encoder* enc, const EncWs& L, char* base, const int32_t* ids, int nb, int Mt, int S,
                           int rows_cap, const SeqMap& sm, const int32_t* lengths, float* h_out, hipStream_t s) {
    const int d = enc->d, f = enc->f, dh = enc->head_dim;
    const int dq = enc->n_heads * dh, dkv = enc->n_kv_heads * dh;
    const int w8 = enc->weight_format == BRL_W_INT8 ? 1 : 0;
    float* x = reinterpret_cast<float*>(base + L.x_off);
    float* big = reinterpret_cast<float*>(base + L.big_off);
    float* cos_t = reinterpret_cast<float*>(base + L.cos_off);
    float* sin_t = reinterpret_cast<float*>(base + L.sin_off);
    float* rinv = reinterpret_cast<float*>(base + L.rinv_off);
    Carver c(base + L.act_off);
    int kmax = d > dq ? d : dq;
    if (f > kmax) kmax = f;
    const ActBuf act = take_actbuf(c, rows_cap, kmax);
    float* qkv = big;
    float* att = big + (size_t)Mt * L.big_ld_qkv;
    if (int rc = launch_embed(enc->embedding, ids, Mt, d, enc->vocab, x, s)) return rc;
    for (int l = 0; l < enc->n_layers; ++l) {
        const brl_layer_weights& w = enc->layers[l];
        QuantArgs qa;
        memset(&qa, 0, sizeof(qa));
        qa.x = x; qa.x_dtype = BRL_F32; qa.gain = w.attn_norm_g; qa.eps_norm = enc->eps_norm; qa.eps_act = enc->eps_act;
        qa.M = Mt; qa.K = d;
        if (int rc = launch_act_quant(qa, act, s)) return rc;
        WeightSegs wqkv;
        memset(&wqkv, 0, sizeof(wqkv));
        wqkv.w8 = w8;
        add_seg(wqkv, w.wq_packed, w.wq_beta, dq);
        add_seg(wqkv, w.wk_packed, w.wk_beta, dkv);
        add_seg(wqkv, w.wv_packed, w.wv_beta, dkv);
        // Uniform batches at head_dim 128 with enough rows for the wide tile: the product writes the attention
        // kernel's operands itself (no fp32 q | k | v rows, no pack kernel); same bits as the two-step form.
        const bool fused = L.q_frags && !sm.cu && !w8 && enc->attn_precision == BRL_ATTN_MFMA &&
                           gemm_attn_eligible(Mt, enc->n_heads, enc->n_kv_heads, dh, S);
        if (fused) {
            AttnOperands ao;
            ao.cos_t = cos_t; ao.sin_t = sin_t;
            ao.qscale = (float)(1.0 / sqrt((double)dh)) * 1.4426950408889634f;
            ao.kvf = base + L.frag_off;
            ao.qf = attention_q_fragments(base + L.frag_off, nb, S, enc->n_kv_heads, dh);
            ao.S = S; ao.n_heads = enc->n_heads; ao.n_kv_heads = enc->n_kv_heads;
            if (int rc = launch_gemm_attn(act, wqkv, Mt, d, ao, s)) return rc;
            if (int rc = launch_attention_mfma_prepacked(nb, S, enc->n_heads, enc->n_kv_heads, base + L.frag_off, att, s))
                return rc;
        } else {
        if (int rc = launch_gemm(act, wqkv, Mt, dq + 2 * dkv, d, qkv, L.big_ld_qkv, nullptr, nullptr, 0, s)) return rc;
        if (enc->attn_precision == BRL_ATTN_MFMA) {
            if (int rc = launch_attention_mfma(qkv, L.big_ld_qkv, nb, S, sm, enc->n_heads, enc->n_kv_heads, dh, cos_t,
                                               sin_t, base + L.frag_off, att, s))
                return rc;
        } else {
            if (int rc = launch_attention_f32(qkv, L.big_ld_qkv, nb, S, sm, enc->n_heads, enc->n_kv_heads, dh, cos_t,
                                              sin_t, att, s))
                return rc;
        }
        }
        QuantArgs qo;
        memset(&qo, 0, sizeof(qo));
        qo.x = att; qo.x_dtype = BRL_F32; qo.gain = w.attn_subln_g; qo.eps_norm = enc->eps_norm; qo.eps_act = enc->eps_act;
        qo.M = Mt; qo.K = dq;
        if (int rc = launch_act_quant(qo, act, s)) return rc;
        const WeightSegs wo = one_seg(w.wo_packed, w.wo_beta, d, w8);
        if (int rc = launch_gemm(act, wo, Mt, d, dq, x, d, x, nullptr, 0, s)) return rc;
        if (int rc = run_ffn(&w.ffn, w8, x, x, BRL_F32, Mt, d, f, enc->eps_norm, enc->eps_act, x, act, big, act, s))
            return rc;
    }
    return launch_final_pool(x, enc->final_norm_g, nb, S, Mt, d, lengths, sm, enc->eps_norm, rinv, h_out, s);
}

}  // namespace

int encoder_forward(const brl_encoder* enc, const int32_t* ids, int B, int S, const int32_t* lengths, float* h,
                    void* workspace, size_t ws_bytes, void* stream) {
    if (int rc = check_encoder(enc)) return rc;
    BRL_REQUIRE(ids && h && workspace && aligned16(h) && aligned16(workspace), "encoder_forward: null or misaligned pointer");
    BRL_REQUIRE(B >= 1 && S >= 1, "encoder_forward: B = %d, S = %d", B, S);
    BRL_REQUIRE((long long)S <= (1 << 20), "encoder_forward: S too large");
    BRL_REQUIRE(enc->eps_act > 0.f && enc->eps_norm >= 0.f && enc->rope_theta > 0.f, "encoder_forward: bad eps / theta");
    const EncWs L = encoder_ws_layout(enc, B, S);
    if (ws_bytes < L.total) {
        set_error("encoder_forward: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    if (int rc = launch_rope_table(reinterpret_cast<float*>(base + L.cos_off), reinterpret_cast<float*>(base + L.sin_off), S,
                                   enc->head_dim, enc->rope_theta, s))
        return rc;
    SeqMap uniform;
    uniform.cu = nullptr;
    uniform.b0 = 0;
    for (int b0 = 0; b0 < B; b0 += L.states_mb) {
        const int nb = (B - b0 < L.states_mb) ? B - b0 : L.states_mb;
        if (int rc = run_encoder_microbatch(enc, L, base, ids + (size_t)b0 * S, nb, nb * S, S, L.states_mb * S, uniform,
                                            lengths ? lengths + b0 : nullptr, h + (size_t)b0 * enc->d, s))
            return rc;
    }
    return BRL_OK;
}

namespace {

constexpr int PACK_MB_STATES = 2048;      // states per micro-batch of the packed layout

// Packed layout: micro-batches hold at most ENC_MB_TOKENS token rows (at least one whole state) and
// at most PACK_MB_STATES states.
EncWs encoder_packed_ws_layout(const brl_encoder* e, int B, int T, int max_len) {
    EncWs L;
    L.q_frags = false;       // states stored back to back do not start at multiples of 32 rows
    memset(&L, 0, sizeof(L));
    L.states_mb = B < PACK_MB_STATES ? B : PACK_MB_STATES;
    size_t Mt = (size_t)(T < ENC_MB_TOKENS ? T : ENC_MB_TOKENS);
    if (Mt < (size_t)max_len) Mt = (size_t)max_len;
    const int dq = e->n_heads * e->head_dim, dkv = e->n_kv_heads * e->head_dim;
    int kmax = e->d;
    if (dq > kmax) kmax = dq;
    if (e->f > kmax) kmax = e->f;
    L.x_off = 0;
    L.act_off = round_up_sz(Mt * e->d * 4, ALIGN);
    L.big_off = L.act_off + actbuf_bytes((int)Mt, kmax);
    const size_t attn_cols = (size_t)dq + 2 * dkv + dq;
    const size_t big_cols = attn_cols > (size_t)e->f ? attn_cols : (size_t)e->f;
    L.cos_off = L.big_off + round_up_sz(Mt * big_cols * 4, ALIGN);
    const size_t tbl = round_up_sz((size_t)max_len * (e->head_dim / 2) * 4, ALIGN);
    L.sin_off = L.cos_off + tbl;
    L.rinv_off = L.sin_off + tbl;
    L.frag_off = L.rinv_off + round_up_sz(Mt * 4, ALIGN);
    L.total = L.frag_off +
              round_up_sz(attention_mfma_ws_bytes(L.states_mb, max_len, e->n_heads, e->n_kv_heads, e->head_dim), ALIGN);
    L.big_ld_qkv = dq + 2 * dkv;
    return L;
}

}  // namespace

size_t brl_encoder_packed_workspace_bytes(const brl_encoder* enc, int B, int T, int max_len) {
    if (!enc || B < 1 || T < B || max_len < 1 || enc->d < 1 || enc->f < 1 || enc->head_dim < 2) return 0;
    return encoder_packed_ws_layout(enc, B, T, max_len).total;
}

int encoder_forward_packed(const brl_encoder* enc, const int32_t* ids, const int32_t* cu_seqlens,
                           const int32_t* cu_seqlens_host, int B, int max_len, float* h, void* workspace,
                           size_t ws_bytes, void* stream) {
    if (int rc = check_encoder(enc)) return rc;
    BRL_REQUIRE(ids && cu_seqlens && cu_seqlens_host && h && workspace && aligned16(h) && aligned16(workspace),
                "encoder_forward_packed: null or misaligned pointer");
    BRL_REQUIRE(B >= 1 && max_len >= 1 && max_len <= ENC_MB_TOKENS, "encoder_forward_packed: B = %d, max_len = %d", B,
                max_len);
    BRL_REQUIRE(enc->eps_act > 0.f && enc->eps_norm >= 0.f && enc->rope_theta > 0.f,
                "encoder_forward_packed: bad eps / theta");
    BRL_REQUIRE(cu_seqlens_host[0] == 0, "encoder_forward_packed: cu_seqlens[0] must be 0");
    for (int b = 0; b < B; ++b) {
        const long long n = (long long)cu_seqlens_host[b + 1] - cu_seqlens_host[b];
        BRL_REQUIRE(n >= 1 && n <= max_len, "encoder_forward_packed: state %d has %lld tokens (1..%d allowed)", b, n,
                    max_len);
    }
    const int T = cu_seqlens_host[B];
    const EncWs L = encoder_packed_ws_layout(enc, B, T, max_len);
    if (ws_bytes < L.total) {
        set_error("encoder_forward_packed: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    if (int rc = launch_rope_table(reinterpret_cast<float*>(base + L.cos_off), reinterpret_cast<float*>(base + L.sin_off),
                                   max_len, enc->head_dim, enc->rope_theta, s))
        return rc;
    const int rows_cap = (T < ENC_MB_TOKENS ? T : ENC_MB_TOKENS) < max_len ? max_len : (T < ENC_MB_TOKENS ? T : ENC_MB_TOKENS);
    int b0 = 0;
    while (b0 < B) {
        int b1 = b0 + 1;                   // a micro-batch takes whole states while they fit
        while (b1 < B && b1 - b0 < L.states_mb && cu_seqlens_host[b1 + 1] - cu_seqlens_host[b0] <= ENC_MB_TOKENS) ++b1;
        SeqMap sm;
        sm.cu = cu_seqlens;
        sm.b0 = b0;
        const int Mt = cu_seqlens_host[b1] - cu_seqlens_host[b0];
        // the longest state of this micro-batch bounds its attention (states of at most 32 tokens take the
        // one-kernel path whatever max_len says); results do not depend on the bound
        int longest = 1;
        for (int b = b0; b < b1; ++b) {
            const int n = cu_seqlens_host[b + 1] - cu_seqlens_host[b];
            if (n > longest) longest = n;
        }
        if (int rc = run_encoder_microbatch(enc, L, base, ids + cu_seqlens_host[b0], b1 - b0, Mt, longest, rows_cap, sm,
                                            nullptr, h + (size_t)b0 * enc->d, s))
            return rc;
        b0 = b1;
    }
    return BRL_OK;
}

namespace {

struct AttnWs {
    size_t cos_off, sin_off, frag_off, total;
};

AttnWs attention_ws_layout(int B, int S, int n_heads, int n_kv_heads, int head_dim) {
    AttnWs L;
    const size_t tbl = round_up_sz((size_t)S * (head_dim / 2) * 4, ALIGN);
    L.cos_off = 0;
    L.sin_off = tbl;
    L.frag_off = 2 * tbl;
    L.total = L.frag_off + round_up_sz(attention_mfma_ws_bytes(B, S, n_heads, n_kv_heads, head_dim), ALIGN);
    return L;
}

bool attention_shape_ok(int B, int S, int n_heads, int n_kv_heads, int head_dim) {
    return B >= 1 && S >= 1 && S <= (1 << 20) && n_heads >= 1 && n_kv_heads >= 1 && n_heads % n_kv_heads == 0 &&
           (head_dim == 16 || head_dim == 32 || head_dim == 64 || head_dim == 100 || head_dim == 128);
}

}  // namespace

size_t brl_attention_workspace_bytes(int B, int S, int n_heads, int n_kv_heads, int head_dim) {
    if (!attention_shape_ok(B, S, n_heads, n_kv_heads, head_dim)) return 0;
    return attention_ws_layout(B, S, n_heads, n_kv_heads, head_dim).total;
}

int attention_forward(const float* qkv, int B, int S, const int32_t* cu_seqlens, const int32_t* cu_seqlens_host,
                      int n_heads, int n_kv_heads, int head_dim, float rope_theta, int attn_precision, float* out,
                      void* workspace, size_t ws_bytes, void* stream) {
    BRL_REQUIRE(qkv && out && workspace && aligned16(qkv) && aligned16(out) && aligned16(workspace),
                "attention_forward: null or misaligned pointer");
    BRL_REQUIRE(attention_shape_ok(B, S, n_heads, n_kv_heads, head_dim),
                "attention_forward: bad shape (B %d, S %d, heads %d / %d, head_dim %d not in {16, 32, 64, 100, 128})", B, S,
                n_heads, n_kv_heads, head_dim);
    BRL_REQUIRE(rope_theta > 0.f, "attention_forward: rope_theta must be positive");
    BRL_REQUIRE(attn_precision == BRL_ATTN_F32 || attn_precision == BRL_ATTN_MFMA,
                "attention_forward: unknown attn_precision %d", attn_precision);
    BRL_REQUIRE((cu_seqlens == nullptr) == (cu_seqlens_host == nullptr),
                "attention_forward: cu_seqlens needs both its device and its host copy");
    if (cu_seqlens_host) {
        BRL_REQUIRE(cu_seqlens_host[0] == 0, "attention_forward: cu_seqlens[0] must be 0");
        for (int b = 0; b < B; ++b) {
            const long long n = (long long)cu_seqlens_host[b + 1] - cu_seqlens_host[b];
            BRL_REQUIRE(n >= 1 && n <= S, "attention_forward: state %d has %lld tokens (1..%d allowed)", b, n, S);
        }
    }
    const AttnWs L = attention_ws_layout(B, S, n_heads, n_kv_heads, head_dim);
    if (ws_bytes < L.total) {
        set_error("attention_forward: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    float* cos_t = reinterpret_cast<float*>(base + L.cos_off);
    float* sin_t = reinterpret_cast<float*>(base + L.sin_off);
    if (int rc = launch_rope_table(cos_t, sin_t, S, head_dim, rope_theta, s)) return rc;
    SeqMap sm;
    sm.cu = cu_seqlens;
    sm.b0 = 0;
    const int ld = (n_heads + 2 * n_kv_heads) * head_dim;
    if (attn_precision == BRL_ATTN_MFMA)
        return launch_attention_mfma(qkv, ld, B, S, sm, n_heads, n_kv_heads, head_dim, cos_t, sin_t, base + L.frag_off, out, s);
    return launch_attention_f32(qkv, ld, B, S, sm, n_heads, n_kv_heads, head_dim, cos_t, sin_t, out, s);
}

size_t brl_head_workspace_bytes(const brl_head* head, int B) {
    if (!head || B < 1) return 0;
    if (!head->policy.dims || !head->value.dims || head->policy.n_layers < 1 || head->value.n_layers < 1 ||
        head->policy.n_layers > 8 || head->value.n_layers > 8)
        return 0;
    size_t mx = mlp_hidden_max(&head->policy);
    const size_t mv = mlp_hidden_max(&head->value);
    if (mv > mx) mx = mv;
    return 2 * round_up_sz((size_t)B * mx * sizeof(double), ALIGN);
}

int policy_value_head(const brl_head* head, const float* h, int B, float* logits, float* value, void* workspace,
                      size_t ws_bytes, void* stream) {
    BRL_REQUIRE(head && h && logits && value && workspace, "policy_value_head: null pointer");
    BRL_REQUIRE(B >= 1, "policy_value_head: B = %d", B);
    if (int rc = check_mlp(&head->policy, "policy head", 0)) return rc;
    if (int rc = check_mlp(&head->value, "value head", 1)) return rc;
    BRL_REQUIRE(head->policy.dims[0] == head->value.dims[0], "policy_value_head: heads disagree on input width");
    const size_t need = brl_head_workspace_bytes(head, B);
    if (ws_bytes < need) {
        set_error("policy_value_head: workspace %zu < %zu", ws_bytes, need);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    double* buf0 = static_cast<double*>(workspace);
    double* buf1 = reinterpret_cast<double*>(static_cast<char*>(workspace) + need / 2);
    if (int rc = run_mlp(&head->policy, h, B, logits, buf0, buf1, s)) return rc;
    return run_mlp(&head->value, h, B, value, buf0, buf1, s);
}

namespace {

int check_ensemble(const brl_mlp* members, int n_members, const char* who) {
    BRL_REQUIRE(members != nullptr, "%s: null member table", who);
    BRL_REQUIRE(n_members >= 1 && n_members <= MAX_ENSEMBLE, "%s: %d members, 1..%d supported", who, n_members, MAX_ENSEMBLE);
    for (int e = 0; e < n_members; ++e) {
        if (int rc = check_mlp(&members[e], "value ensemble member", 1)) return rc;
        BRL_REQUIRE(members[e].n_layers == members[0].n_layers && members[e].act == members[0].act,
                    "%s: member %d differs from member 0 in depth or activation", who, e);
        for (int i = 0; i <= members[0].n_layers; ++i)
            BRL_REQUIRE(members[e].dims[i] == members[0].dims[i], "%s: member %d differs from member 0 in dims[%d]", who, e, i);
    }
    return BRL_OK;
}

struct EnsembleWs {
    size_t buf0_off, buf1_off, each_off, total;
};

EnsembleWs ensemble_ws_layout(const brl_mlp* members, int n_members, int B) {
    EnsembleWs L;
    const size_t hid = round_up_sz((size_t)n_members * B * mlp_hidden_max(&members[0]) * sizeof(double), ALIGN);
    L.buf0_off = 0;
    L.buf1_off = hid;
    L.each_off = 2 * hid;
    L.total = L.each_off + round_up_sz((size_t)n_members * B * sizeof(float), ALIGN);
    return L;
}

}  // namespace

size_t brl_value_ensemble_workspace_bytes(const brl_mlp* members, int n_members, int B) {
    if (!members || n_members < 1 || n_members > MAX_ENSEMBLE || B < 1) return 0;
    if (!members[0].dims || members[0].n_layers < 1 || members[0].n_layers > 8) return 0;
    return ensemble_ws_layout(members, n_members, B).total;
}

int value_ensemble_forward(const brl_mlp* members, int n_members, const float* h, int B, float* value_mean,
                           float* values_each, void* workspace, size_t ws_bytes, void* stream) {
    BRL_REQUIRE(h && value_mean && workspace && aligned16(workspace), "value_ensemble_forward: null or misaligned pointer");
    BRL_REQUIRE(B >= 1, "value_ensemble_forward: B = %d", B);
    if (int rc = check_ensemble(members, n_members, "value_ensemble_forward")) return rc;
    const EnsembleWs L = ensemble_ws_layout(members, n_members, B);
    if (ws_bytes < L.total) {
        set_error("value_ensemble_forward: workspace %zu < %zu", ws_bytes, L.total);
        return BRL_ENOSPC;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    double* bufs[2] = {reinterpret_cast<double*>(base + L.buf0_off), reinterpret_cast<double*>(base + L.buf1_off)};
    float* each = values_each ? values_each : reinterpret_cast<float*>(base + L.each_off);
    const brl_mlp& m0 = members[0];
    const double* in64 = nullptr;
    for (int i = 0; i < m0.n_layers; ++i) {
        EnsembleLayer a;
        memset(&a, 0, sizeof(a));
        for (int e = 0; e < n_members; ++e) {
            a.W[e] = members[e].W[i];
            a.bias[e] = members[e].b[i];
        }
        a.n_members = n_members; a.B = B; a.in_dim = m0.dims[i]; a.out_dim = m0.dims[i + 1]; a.act = m0.act;
        a.last = (i + 1 == m0.n_layers) ? 1 : 0;
        a.in64 = in64; a.in32 = h;
        a.out64 = a.last ? nullptr : bufs[i & 1];
        a.out32 = a.last ? each : nullptr;
        if (int rc = launch_ensemble_layer(a, s)) return rc;
        in64 = a.out64;
    }
    return launch_ensemble_mean(each, n_members, B, value_mean, s);
}

}  // extern "C"
