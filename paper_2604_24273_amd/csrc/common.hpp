// Shared declarations of the gfx950 kernels: layouts, launch helpers, errors.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "bitrl.h"

namespace brl {

// ---- error plumbing (host) ----
void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);

#define BRL_HIP_CHECK(expr)                                   \
    do {                                                      \
        hipError_t e__ = (expr);                              \
        if (e__ != hipSuccess) return ::brl::hip_fail(e__, #expr); \
    } while (0)

#define BRL_LAUNCH_CHECK(name)                                \
    do {                                                      \
        hipError_t e__ = hipGetLastError();                   \
        if (e__ != hipSuccess) return ::brl::hip_fail(e__, name); \
    } while (0)

#define BRL_REQUIRE(cond, ...)                                \
    do {                                                      \
        if (!(cond)) { ::brl::set_error(__VA_ARGS__); return BRL_EINVAL; } \
    } while (0)

// ---- optional per-launch timing (host): brackets a launch with two events ----
struct LaunchTimer {
    LaunchTimer(int kernel_class, hipStream_t s, double int8_ops = 0.0);
    ~LaunchTimer();
    LaunchTimer(const LaunchTimer&) = delete;
    LaunchTimer& operator=(const LaunchTimer&) = delete;
  private:
    hipEvent_t stop_;
    hipStream_t s_;
    bool on_;
};

// ---- sizes ----
constexpr int WAVE = 64;
constexpr int NB = 32;        // rows of one weight block / tokens of one activation block
constexpr int SBK = 128;      // columns of one super-block (four MFMA k-steps of 32)
constexpr int MAX_K = 9216;   // widest token row the quantisation kernels hold in registers (4 wavefronts x 9 float4 per lane)

__host__ __device__ inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
__host__ __device__ inline size_t round_up_sz(size_t v, size_t m) { return (v + m - 1) / m * m; }

// Offset of the 32-bit word holding weights (row n, columns 16*kk .. 16*kk+15)
// in the packed blob; nsb = Kp / 128.
__host__ __device__ inline size_t packed_word_index(int n, int kk, int nsb) {
    int nb = n >> 5, r = n & 31;
    int sb = kk >> 3, dd = (kk >> 1) & 3, hh = kk & 1;
    return (((size_t)nb * nsb + sb) * 64 + (hh * 32 + r)) * 4 + dd;
}

// Byte offset of activation (token m, column k) in the tiled int8 buffer: a
// token block of 32 rows x 128 columns is 4 KB, made of four 1 KB fragments
// (one per MFMA k-step) in which lane (m & 31) + 32 * ((k >> 4) & 1) owns 16
// consecutive bytes.
__host__ __device__ inline size_t tiled_act_offset(int m, int k, int nsb) {
    int mb = m >> 5, r = m & 31;
    int sb = k >> 7, dd = (k >> 5) & 3, hh = (k >> 4) & 1, i = k & 15;
    return ((((size_t)mb * nsb + sb) * 4 + dd) * 64 + (hh * 32 + r)) * 16 + i;
}

// ---- quantised activations of one GEMM input (device buffers in a workspace) ----
struct ActBuf {
    int8_t* q;        // tiled int8 [Mp/32][nsb][4][64][16]
    float* absmax;    // [Mp] clamped absmax a'
    float* dscale;    // [Mp] a' / 127
    int32_t* sumq;    // [Mp] sum_k q (for the offset-code correction)
    int32_t* splitk;  // scratch for the partial tiles of a k-split GEMM reading this buffer (or nullptr)
    size_t splitk_ints;
};

// k-split GEMM: used when fewer than SPLITK_MAX_TILES 128 x 128 tiles exist; aims at SPLITK_TARGET_WGS
// workgroups.  splits * tiles <= target + tiles, so the partial tiles never exceed SPLITK_INTS.
constexpr int SPLITK_MAX_TILES = 128;
constexpr int SPLITK_TARGET_WGS = 512;
constexpr int SPLITK_MIN_SB = 32;           // super-blocks of k (4096 columns) below which k is never cut
constexpr size_t SPLITK_INTS = (size_t)(SPLITK_TARGET_WGS + SPLITK_MAX_TILES) * 128 * 128;
inline size_t splitk_capacity_ints(int M) {       // by token count alone: 0 where no k-split can happen
    const int nmb = round_up(M, NB) / NB;
    return (nmb <= 4 || (nmb + 3) / 4 >= SPLITK_MAX_TILES) ? 0 : SPLITK_INTS;
}

// ---- up to three weight matrices sharing one activation (q|k|v, gate|up) ----
struct WeightSegs {
    const uint32_t* packed[3];
    const float* beta[3];
    int nb_end[3];    // exclusive end, in 32-row blocks, of each segment
    int n_end[3];     // exclusive end, in rows
    int count;
    int w8;           // 0: 2-bit ternary blobs; 1: int8 blobs in the activations' fragment layout
};

// ---- kernel launchers (host) ----
// weight ternarisation
int launch_quantize_weights(const float* W, int N, int K, float eps, uint32_t* packed, float* beta,
                            int8_t* codes_dbg, double* partials, int* flag, hipStream_t s);
int launch_unpack_codes(const uint32_t* packed, int N, int K, int8_t* codes, hipStream_t s);
int quantize_partials_count(int N, int K);
// per-tensor absmax int8 weights, written in the tiled layout of tiled_act_offset (row n in place of token m)
int launch_quantize_weights_int8(const float* W, int N, int K, float eps, int qmax, int8_t* packed, float* scale,
                                 int8_t* codes_dbg, float* partials, int* flag, hipStream_t s);
int launch_unpack_codes_int8(const int8_t* packed, int N, int K, int8_t* codes, hipStream_t s);

// activation quantisation (plain, or RMSNorm first)
struct QuantArgs {
    const void* x;          // [M, K] fp32 or bf16
    int x_dtype;
    const float* gain;      // RMSNorm gain [K] or nullptr (no norm)
    float eps_norm, eps_act;
    int M, K;
    int8_t* xq_rowmajor;    // optional tap [M, K]
    float* absmax_tap;      // optional tap [M]
};
int launch_act_quant(const QuantArgs& a, const ActBuf& out, hipStream_t s);

// int8 MFMA GEMM with fused dequant epilogue
// glu = 1: w holds (gate, up); y [M, N/2] receives (max(G,0) * max(G,0)) * U
// res_bf16 = 1: `residual` points at bf16 bit patterns [M, ldy] (widened exactly when read)
int launch_gemm(const ActBuf& a, const WeightSegs& w, int M, int N, int K,
                float* y, int ldy, const float* residual, int32_t* acc_dbg, int glu, hipStream_t s, int res_bf16 = 0);

// The q | k | v product of a uniform batch (head_dim 128, 32 | S) written as the operands of the matrix-core
// attention kernel instead of fp32 rows: rotated q (scaled) and k as fp16 hi / lo fragments, v transposed.
struct AttnOperands {
    const float* cos_t;   // [S][64]
    const float* sin_t;
    float qscale;
    void* kvf;            // K / V fragments, as attn_pack_kernel lays them out
    void* qf;             // q fragments [B][Hq][S/32][8][hi,lo][64 lanes] of 16 bytes
    int S, n_heads, n_kv_heads;
};
bool gemm_attn_eligible(int M, int n_heads, int n_kv_heads, int head_dim, int S);
int launch_gemm_attn(const ActBuf& a, const WeightSegs& w, int M, int K, const AttnOperands& out, hipStream_t s);

// bandwidth-bound GEMV (M <= 4), activation quantisation fused
int launch_gemv(const void* x, int x_dtype, int M, int K, int N, const uint32_t* packed, const float* beta,
                float eps_act, float* y, const float* residual, int8_t* xq_dbg, float* absmax_dbg,
                int32_t* acc_dbg, hipStream_t s);
int launch_gemv_batch(const void* const* packed, const float* const* beta, int N, int K, const void* const* x,
                      int x_dtype, int M, float eps_act, float* const* y, int count, hipStream_t s);

// attention, embedding, pooling, heads
// Where the rows of state b of a micro-batch live.  cu == nullptr: every state has S rows, state b
// starts at row b * S.  Otherwise cu holds cumulative state lengths of the whole call; the micro-batch
// starts at state b0 and its rows are counted from cu[b0]; S then only bounds the lengths.
struct SeqMap {
    const int32_t* cu;
    int b0;
};
__device__ inline int seq_row0(const SeqMap& m, int b, int S) { return m.cu ? m.cu[m.b0 + b] - m.cu[m.b0] : b * S; }
__device__ inline int seq_len(const SeqMap& m, int b, int S) {
    if (!m.cu) return S;
    const int n = m.cu[m.b0 + b + 1] - m.cu[m.b0 + b];
    return n < 0 ? 0 : (n > S ? S : n);
}

int launch_rope_table(float* cos_t, float* sin_t, int S, int head_dim, float theta, hipStream_t s);
int launch_attention_f32(const float* qkv, int ld, int B, int S, const SeqMap& sm, int n_heads, int n_kv_heads,
                         int head_dim, const float* cos_t, const float* sin_t, float* out, hipStream_t s);
size_t attention_mfma_ws_bytes(int B, int S, int n_heads, int n_kv_heads, int head_dim, bool q_frags = false);
void* attention_q_fragments(void* frag_ws, int B, int S, int n_kv_heads, int head_dim);   // where the q fragments start
int launch_attention_mfma_prepacked(int B, int S, int n_heads, int n_kv_heads, void* frag_ws, float* out, hipStream_t s);
int launch_attention_mfma(const float* qkv, int ld, int B, int S, const SeqMap& sm, int n_heads, int n_kv_heads,
                          int head_dim, const float* cos_t, const float* sin_t, void* frag_ws, float* out, hipStream_t s);
int launch_embed(const uint16_t* table, const int32_t* ids, int M, int d, int vocab, float* x, hipStream_t s);
// M rows in all; lengths (or nullptr) applies to the uniform layout only
int launch_final_pool(const float* x, const float* gain, int B, int S, int M, int d, const int32_t* lengths,
                      const SeqMap& sm, float eps_norm, float* rinv, float* h, hipStream_t s);
int launch_mlp_layer(const double* in64, const float* in32, const float* W, const float* b, int B, int in_dim,
                     int out_dim, int act, double* out64, float* out32, hipStream_t s);
// one layer of up to 8 equally shaped heads (an ensemble of critics) in one launch
constexpr int MAX_ENSEMBLE = 8;
struct EnsembleLayer {
    const float* W[MAX_ENSEMBLE];
    const float* bias[MAX_ENSEMBLE];
    int n_members, B, in_dim, out_dim, act, last;
    const double* in64;     // [n_members, B, in_dim] or nullptr: then every member reads in32
    const float* in32;      // [B, in_dim]
    double* out64;          // [n_members, B, out_dim] (hidden layers)
    float* out32;           // [n_members, B] (last layer, out_dim == 1)
};
int launch_ensemble_layer(const EnsembleLayer& a, hipStream_t s);
int launch_ensemble_mean(const float* each, int n, int B, float* mean, hipStream_t s);

}  // namespace brl
