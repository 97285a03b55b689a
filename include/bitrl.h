/*
 * bitrl.h - C ABI of the MI355X (gfx950) forward pass of BitRL's frozen
 * ternary state encoder and its fp32 policy / value heads, and of the PPO
 * update of those heads on cached encoder outputs.
 *
 * The library computes h_t = f(token ids) and (logits, V) = (g(h_t), v(h_t))
 * (paper Sec. 3.1, Eq. 3) for a BitNet-b1.58 style backbone whose linear
 * layers are BitLinear: ternary weights (Sec. 3.1, Eq. 2), per-token int8
 * activations, integer accumulation, fp32 rescale; and one clipped-surrogate
 * update (Sec. 3.1, Eq. 1; Sec. 3.2) of the head parameters.
 *
 * Conventions for every function
 * ------------------------------
 *  - Plain C, no exceptions.  The return value is a status code (BRL_OK = 0).
 *    On failure nothing was enqueued and brl_last_error() describes the cause
 *    (thread-local string, valid until the next failing call on that thread).
 *  - Every tensor pointer is a DEVICE pointer unless its comment says HOST.
 *    Tensors are row-major and contiguous; pointers must be 16-byte aligned.
 *    Structs passed by pointer (weights tables, configs) are read on the HOST
 *    during the call and need not outlive it; the device buffers they point to
 *    must stay valid until the enqueued work has run.
 *  - The caller owns all memory.  The library never allocates or frees device
 *    memory: scratch space comes in through `workspace` / `ws_bytes`, whose
 *    minimum size the matching brl_*_workspace_bytes() query returns.  A
 *    workspace carries no state between calls (its contents may be anything on
 *    entry); calls that share a workspace must be ordered on one stream.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    *_forward calls only enqueue kernels: no host synchronisation, no
 *    device-to-host copy.  bitlinear_quantize_weights (an offline step)
 *    synchronises the stream once so that it can report bad weights.
 *  - Non-finite activations are not checked: results are then unspecified
 *    (never out-of-bounds accesses).  Token ids outside [0, vocab) are clamped.
 *  - Limits: 1 <= K <= 9216 input features per BitLinear (a token row is
 *    held in the registers of the wavefronts that quantise it), any N, any M.
 */
#ifndef BITRL_H
#define BITRL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---- */
#define BRL_OK      0   /* work enqueued */
#define BRL_EINVAL  1   /* bad shape, null or misaligned pointer, unsupported size, bad weights */
#define BRL_ENOSPC  2   /* workspace smaller than the query says */
#define BRL_EHIP    3   /* a HIP runtime call failed */

/* ---- element types of activation inputs ---- */
#define BRL_F32   0
#define BRL_BF16  1    /* widened to fp32 exactly on load */

/* ---- head activation ---- */
#define BRL_ACT_TANH 0
#define BRL_ACT_RELU 1

/* ---- attention arithmetic ---- */
#define BRL_ATTN_F32  0   /* fp32 FMA on the vector ALUs */
#define BRL_ATTN_MFMA 1   /* matrix cores: every operand as fp16 hi + lo pair (three MFMAs per product,
                             about 21 mantissa bits), fp32 softmax and accumulation; q, k, v must lie
                             within the fp16 range (|x| < 65504) */

/* format of the weight blobs of an encoder */
#define BRL_W_TERNARY 0   /* 2-bit blobs from bitlinear_quantize_weights */
#define BRL_W_INT8    1   /* int8 blobs from bitlinear_quantize_weights_int8 (higher-precision critic backbone) */

const char* brl_last_error(void);
int         brl_abi_version(void);

/* ------------------------------------------------------------------------
 * BitLinear weights (Sec. 3.1, Eq. 2: Q(W) = sign(W) * 1[|W| > tau]).
 *
 * tau = beta / 2 with beta = mean|W| + eps over the whole matrix (one scale
 * per matrix; the mean is accumulated in fp64 and rounded to fp32 once).
 * |w| == tau gives code 0.  beta is also the dequantisation scale.
 *
 * Packed format (version 1): rows padded to a multiple of 32, columns to a
 * multiple of 128, 2 bits per weight holding code + 1 in {0, 1, 2}; padding
 * holds code 0.  The 32-bit word with index ((nb * (Kp/128) + sb) * 64 + lane)
 * * 4 + dd holds the 16 weights of row n = 32 nb + (lane & 31) at columns
 * k = 128 sb + 32 dd + 16 (lane >> 5) + i, i = 0..15, weight i = 4 j + b at
 * bits [2 j + 8 b, 2 j + 8 b + 1].  So (word >> 2 j) & 0x03030303 is four
 * consecutive-k bytes ready for an int8 dot product, and a wavefront reading
 * 16 bytes per lane gets one 32 x 128 block in the int8 MFMA operand order.
 * The blob may be stored and reloaded; it carries no header.
 * ------------------------------------------------------------------------ */
size_t brl_packed_bytes(int n_out, int k_in);
size_t brl_quantize_workspace_bytes(int n_out, int k_in);

/* W [n_out, k_in] fp32  ->  packed_out [brl_packed_bytes], beta_out [1] fp32.
 * codes_dbg: optional [n_out, k_in] int8 plain codes in {-1, 0, 1} (or NULL).
 * Returns BRL_EINVAL if mean|W| is not finite (outputs then unspecified).
 * Synchronises `stream`. */
int bitlinear_quantize_weights(const float* W, int n_out, int k_in, float eps,
                               void* packed_out, float* beta_out, int8_t* codes_dbg,
                               void* workspace, size_t ws_bytes, void* stream);

/* packed -> plain int8 codes [n_out, k_in] in {-1, 0, 1}. */
int brl_unpack_codes(const void* packed, int n_out, int k_in, int8_t* codes_out, void* stream);

/* ------------------------------------------------------------------------
 * BitLinear forward: y = dequant(ternary_matmul(quant(x), W)) (+ residual).
 * Sec. 3.1 (Framework Architecture, last paragraph): the backbone runs its
 * ternary weights (Eq. 2) through integer-only kernels, no floating-point
 * multiply-accumulate.  The paper does not define the activation side; it is
 * taken from the BitNet b1.58 scheme the paper names as its backbone: one
 * symmetric int8 scale per token from the absolute maximum (Qb = 127,
 * round-half-to-even), int32 accumulation, and one fp32 rescale by the token
 * scale and the matrix scale beta of Eq. 2's threshold.
 *
 * Per token t: a = max(max_k |x_tk|, eps_act); q_tk = clamp(rne(x_tk *
 * (127 / a)), -127, 127); acc_tn = sum_k q_tk code_nk (int32, exact);
 * y_tn = (float(acc_tn) * (a / 127)) * beta (+ residual_tn), each fp32
 * operation rounded once, in that order.  No normalisation happens inside.
 *
 * x [M, K] of x_dtype; y [M, N] fp32; residual [M, N] fp32 or NULL (may alias
 * y).  Optional taps (NULL to skip): xq_dbg [M, K] int8, absmax_dbg [M] fp32
 * (the clamped a), acc_dbg [M, N] int32.
 * M <= 4 takes the bandwidth-bound GEMV path, larger M the int8 MFMA path.
 * ------------------------------------------------------------------------ */
size_t brl_bitlinear_workspace_bytes(int M, int N, int K);
int bitlinear_forward(const void* packed, const float* beta, int N, int K,
                      const void* x, int x_dtype, int M, float eps_act,
                      float* y, const float* residual,
                      int8_t* xq_dbg, float* absmax_dbg, int32_t* acc_dbg,
                      void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * bitlinear_forward for callers that cannot allocate device memory or hand over
 * a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments (no workspace), same kernels, same
 * bits in y and in the taps.  The quantised activations (int8 tiles, per-token
 * scale and code sum: 32-row x 128-column padded M x K bytes + 12 bytes per
 * token) are kept in an array built into the library,
 * BRL_STATIC_SCRATCH_BYTES per GPU, held until the process ends.  Larger
 * products return BRL_ENOSPC (nothing enqueued); M <= 4 needs no scratch.
 * The call makes no hipMalloc / hipFree and no allocating library call; the
 * first call on a device looks the array's address up (make it outside graph
 * capture).  Every call on one GPU shares that GPU's array: the contents are
 * rewritten by each call (nothing has to start at zero), and calls that
 * overlap in time on one GPU (different streams or threads) race - order them.
 * Products that bitlinear_forward would cut along k run uncut here (integer
 * sums: identical results).
 * ------------------------------------------------------------------------ */
#define BRL_STATIC_SCRATCH_BYTES (16u << 20)
int bitlinear_forward_static(const void* packed, const float* beta, int N, int K,
                             const void* x, int x_dtype, int M, float eps_act,
                             float* y, const float* residual,
                             int8_t* xq_dbg, float* absmax_dbg, int32_t* acc_dbg,
                             void* stream);

/* ------------------------------------------------------------------------
 * Int8-weight BitLinear for a higher-precision critic backbone (Sec. 5.3,
 * component ablations: the "INT8 critic + 1-bit policy" rows; the paper names
 * the configuration, the quantiser below is this library's reading of it).
 *
 * Weights, one scale per matrix, the mirror of the per-token activation
 * quantiser: a = max(max|W|, eps); s = qmax / a (fp32 divide); code =
 * clamp(rne(w * s), -qmax, qmax); scale = a / qmax.  qmax = 127 is the int8
 * critic; qmax = 7 gives the grid of the table's "INT4 critic" (1 <= qmax <=
 * 127; the codes are stored one per byte whatever qmax is, so this reproduces
 * the int4 critic's arithmetic, not its memory footprint).  Forward: per-token int8
 * activations exactly as in bitlinear_forward, acc = sum_k q code (int32,
 * exact), y = (float(acc) * (a_t / 127)) * scale (+ residual).
 *
 * Packed format: rows padded to a multiple of 32, columns to a multiple of
 * 128, one byte per weight, zero padding; the byte of (n, k) sits at
 * ((((n/32) * (Kp/128) + k/128) * 4 + (k/32)%4) * 64 + 32 * ((k/16)%2) + n%32) * 16 + k%16
 * (the int8 MFMA operand order, the same layout the quantised activations
 * use).  The blob carries no header.
 * Arguments, taps and errors as for the ternary entry points; every M runs
 * the int8 MFMA kernel (there is no separate 1..4 token path).
 * An encoder with weight_format = BRL_W_INT8 uses such blobs in every layer.
 * ------------------------------------------------------------------------ */
size_t brl_packed_int8_bytes(int n_out, int k_in);
int bitlinear_quantize_weights_int8(const float* W, int n_out, int k_in, float eps, int qmax,
                                    void* packed_out, float* scale_out, int8_t* codes_dbg,
                                    void* workspace /* brl_quantize_workspace_bytes */, size_t ws_bytes, void* stream);
int brl_unpack_codes_int8(const void* packed, int n_out, int k_in, int8_t* codes_out, void* stream);
int bitlinear_int8_forward(const void* packed, const float* scale, int N, int K,
                           const void* x, int x_dtype, int M, float eps_act,
                           float* y, const float* residual,
                           int8_t* xq_dbg, float* absmax_dbg, int32_t* acc_dbg,
                           void* workspace /* brl_bitlinear_workspace_bytes */, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Many independent few-token BitLinear problems of one shape in one launch:
 *   y[i] = BitLinear(x[i]; packed[i], beta[i]),  i = 0 .. count-1,
 * each computed exactly as bitlinear_forward computes it (Section 3.1: the
 * frozen encoder is evaluated once per environment step on a single short
 * state, where the ternary matmul is bound by streaming the weights).  With
 * one token a 2560 x 6912 matrix is 4.4 MB of weights and far below the cost
 * of a kernel launch; this entry point lets a caller that has many such
 * products queued (several encoders, adapters or layers whose inputs are
 * already known) stream them at HBM rate.
 *
 * packed, beta, x, y: DEVICE arrays of count device pointers (packed[i] from
 * bitlinear_quantize_weights for an [N, K] matrix; beta[i] [1]; x[i] [M, K]
 * of x_dtype; y[i] [M, N] fp32).  1 <= M <= 4.  Entries may repeat in packed /
 * beta / x; the y[i] must be distinct buffers.  No workspace, no taps.
 * The pointer arrays are read on the device only: the host cannot check them.
 * ------------------------------------------------------------------------ */
int bitlinear_forward_batch(const void* const* packed, const float* const* beta, int N, int K,
                            const void* const* x, int x_dtype, int M, float eps_act,
                            float* const* y, int count, void* stream);

/* ------------------------------------------------------------------------
 * One feed-forward block of the frozen backbone f of Sec. 3.1, Eq. 3 (the
 * paper cites the BitNet b1.58 architecture for f and gives no block
 * internals; this is that architecture's block: pre-norm, gate / up BitLinear
 * sharing one quantised input, squared-ReLU gated unit, sub-layer norm, down
 * BitLinear, residual):
 *   n = RMSNorm_d(x; norm_g);  (G, U) = BitLinear_gate(n), BitLinear_up(n)
 *   (n is quantised once, each matrix keeps its own beta);
 *   h = (max(G,0) * max(G,0)) * U;  m = RMSNorm_f(h; subln_g);
 *   y = x + BitLinear_down(m).
 * RMSNorm: r = fp32(1 / sqrt(mean_k x_k^2 + eps_norm)) with the statistic in
 * fp64; out_k = (x_k * r) * g_k in fp32.
 * x [M, d] of x_dtype, y [M, d] fp32 (must not alias x).
 * ------------------------------------------------------------------------ */
typedef struct brl_ffn_weights {
    const float* norm_g;        /* [d] */
    const void*  gate_packed;   /* [f, d] packed */
    const float* gate_beta;     /* [1] */
    const void*  up_packed;     /* [f, d] packed */
    const float* up_beta;       /* [1] */
    const float* subln_g;       /* [f] */
    const void*  down_packed;   /* [d, f] packed */
    const float* down_beta;     /* [1] */
} brl_ffn_weights;

size_t brl_ffn_workspace_bytes(int M, int d, int f);
int ffn_block_forward(const brl_ffn_weights* w /* HOST */, const void* x, int x_dtype,
                      int M, int d, int f, float eps_norm, float eps_act,
                      float* y, void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Frozen encoder (Sec. 3.1, Eq. 3: h_t = f(serialize(s_t)), from token ids).
 *
 * x = E[ids] (bf16 table, widened); per layer: x += o(subLN(attn(q(n), k(n),
 * v(n)))) with n = RMSNorm(x), rotary embedding on pairs (i, i + head_dim/2)
 * at position = index inside the state, causal softmax(q k^T / sqrt(head_dim))
 * v, query head h reading key/value head h / (n_heads / n_kv_heads); then the
 * feed-forward block above.  h[b] = mean over the first lengths[b] positions
 * (all S if lengths is NULL) of RMSNorm(x; final_norm_g), summed in fp64
 * (mean pooling is the only pooling; the paper says only that h_t is a vector
 * of the hidden width).
 * States are independent; large batches are processed in micro-batches of
 * whole states inside the call.  How the stages are cut into kernels depends
 * on the shapes only (with head_dim 128, S a multiple of 32 and a few thousand
 * token rows the q | k | v product writes the attention operands itself instead
 * of fp32 rows); a state's result does not: it has the same bits in a batch of
 * any size, padded or stored back to back.  Like every *_forward here the call only
 * enqueues kernels on `stream` (no allocation, no synchronisation), so a
 * sequence of calls can be captured into a HIP graph - after one ordinary call
 * of the same shapes, because the first use of a kernel queries the device's
 * occupancy limits once.
 * ids [B, S] int32, lengths [B] int32 in [1, S] or NULL, h [B, d] fp32.
 * ------------------------------------------------------------------------ */
typedef struct brl_layer_weights {
    const float* attn_norm_g;   /* [d] */
    const void*  wq_packed;  const float* wq_beta;   /* [n_heads*head_dim, d] */
    const void*  wk_packed;  const float* wk_beta;   /* [n_kv_heads*head_dim, d] */
    const void*  wv_packed;  const float* wv_beta;   /* [n_kv_heads*head_dim, d] */
    const float* attn_subln_g;  /* [n_heads*head_dim] */
    const void*  wo_packed;  const float* wo_beta;   /* [d, n_heads*head_dim] */
    brl_ffn_weights ffn;
} brl_layer_weights;

typedef struct brl_encoder {
    int   n_layers, d, n_heads, n_kv_heads, head_dim, f, vocab;
    float rope_theta, eps_norm, eps_act;
    int   attn_precision;               /* BRL_ATTN_*: fp32 vector ALUs, or fp16 hi + lo pairs on the matrix
                                           cores (fp32-grade; there is no plain 16-bit mode: its error is
                                           amplified by the int8 re-quantisation of every later layer) */
    int   weight_format;                /* BRL_W_*: what every *_packed pointer of the layers holds; with
                                           BRL_W_INT8 each *_beta is the scale from bitlinear_quantize_weights_int8 */
    const uint16_t* embedding;          /* [vocab, d] bf16 bit patterns */
    const float*    final_norm_g;       /* [d] */
    const brl_layer_weights* layers;    /* HOST array of n_layers entries */
} brl_encoder;

size_t brl_encoder_workspace_bytes(const brl_encoder* enc /* HOST */, int B, int S);
int encoder_forward(const brl_encoder* enc /* HOST */, const int32_t* ids, int B, int S,
                    const int32_t* lengths, float* h,
                    void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The same encoder on states of different lengths stored back to back, with
 * no padding (Sec. 5.2: a serialised state is 15 to 40 tokens): state b owns
 * the token rows cu_seqlens[b] .. cu_seqlens[b+1]-1, positions count from 0
 * inside each state, attention never crosses a state boundary, and
 * h[b] = mean over the state's own positions.  Each state's result equals
 * what encoder_forward gives for that state alone.
 *
 * ids [T] int32 (device), T = cu_seqlens[B]; cu_seqlens [B+1] int32, given
 * twice: a DEVICE copy read by the kernels and a HOST copy used to check the
 * lengths (cu[0] = 0, 1 <= length <= max_len, else BRL_EINVAL) and to cut the
 * batch into micro-batches of whole states; max_len bounds every length and
 * sizes the rotary table.  h [B, d] fp32.
 * ------------------------------------------------------------------------ */
size_t brl_encoder_packed_workspace_bytes(const brl_encoder* enc /* HOST */, int B, int T, int max_len);
int encoder_forward_packed(const brl_encoder* enc /* HOST */, const int32_t* ids,
                           const int32_t* cu_seqlens /* DEVICE */, const int32_t* cu_seqlens_host /* HOST */,
                           int B, int max_len, float* h,
                           void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The attention stage of an encoder layer on its own (the softmax attention of
 * the backbone f of Sec. 3.1, Eq. 3; the paper gives no internals, the form is
 * that of the BitNet b1.58 decoder it cites): rotary embedding of q and k on
 * pairs (i, i + head_dim/2) at position = index inside the state, causal
 * softmax(q k^T / sqrt(head_dim)) v, query head h reading key/value head
 * h / (n_heads / n_kv_heads).  encoder_forward runs exactly these kernels on
 * the output of its q | k | v BitLinear; this entry point exposes them so that
 * the stage can be checked by itself.
 *
 * qkv [T, (n_heads + 2 n_kv_heads) * head_dim] fp32, a row = q heads | k heads
 * | v heads; out [T, n_heads * head_dim] fp32.  cu_seqlens NULL (both copies):
 * B states of S rows each, T = B * S.  Otherwise state b owns rows
 * cu_seqlens[b] .. cu_seqlens[b+1]-1 (DEVICE and HOST copies of the same
 * [B+1] int32 array, lengths in 1..S, else BRL_EINVAL) and S bounds the
 * lengths.  head_dim in {16, 32, 64, 100, 128}; attn_precision BRL_ATTN_*.
 * With BRL_ATTN_MFMA, states of at most 32 tokens (up to 1024 workgroups) take
 * a one-kernel path, everything else the pack + fragment kernels.
 * ------------------------------------------------------------------------ */
size_t brl_attention_workspace_bytes(int B, int S, int n_heads, int n_kv_heads, int head_dim);
int attention_forward(const float* qkv, int B, int S,
                      const int32_t* cu_seqlens /* DEVICE or NULL */, const int32_t* cu_seqlens_host /* HOST or NULL */,
                      int n_heads, int n_kv_heads, int head_dim, float rope_theta, int attn_precision,
                      float* out, void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * State-to-token front end: serialize(s_t) of Sec. 3.1, Eq. 3 ("converts
 * environment states to natural language text"; Sec. 5.2: a state of 17 - 27
 * dimensions is 15 - 40 tokens, about 1.2 ms of host time on the paper's
 * device).  HOST code, HOST pointers, no GPU work.  The paper gives neither
 * the text format nor the tokenizer, and the backbone's own tokenizer is not
 * part of this library; this is a documented stand-in whose ids have the right
 * number and range:
 *   text    "state:" then, per dimension, " v" with v the value clamped to
 *           [-9.9, 9.9] and written with one decimal, correctly rounded from
 *           the exact fp32 value (exact ties to the even digit), zero without
 *           a sign, NaN as 0.0;
 *   ids     0 begin-of-state, 1 "state:", 2 .. 200 the number strings " -9.9"
 *           .. " 9.9" (id = 101 + 10 v), 201 .. 456 the single bytes; text is
 *           tokenised greedily, longest entry first, after id 0.
 * A state of n_dims values is n_dims + 2 tokens.
 *
 * brl_serialize_text: writes the NUL-terminated text if cap > the returned
 *   length; returns the text length in bytes either way (0 for bad arguments).
 * brl_tokenize: ids of any byte string (free text falls back to byte ids);
 *   *n_ids is the token count; BRL_ENOSPC if it exceeds max_ids (the first
 *   max_ids ids are still written).
 * serialize_states: states [B, n_dims] fp32 -> ids_out [B * (n_dims + 2)] and
 *   cu_seqlens_out [B + 1], the layout encoder_forward_packed takes (copy ids
 *   and cu_seqlens to the device, pass cu_seqlens_out as its host copy);
 *   BRL_EINVAL if the encoder's vocab is below BRL_SERIALIZE_VOCAB.
 * ------------------------------------------------------------------------ */
#define BRL_SERIALIZE_VOCAB 457
size_t brl_serialize_text(const float* state /* HOST */, int n_dims, char* text_out /* HOST */, size_t cap);
int brl_tokenize(const char* text /* HOST */, size_t n_bytes, int32_t* ids_out /* HOST */, int max_ids, int* n_ids /* HOST */);
int serialize_states(const float* states /* HOST */, int B, int n_dims, int vocab,
                     int32_t* ids_out /* HOST */, int32_t* cu_seqlens_out /* HOST */);

/* ------------------------------------------------------------------------
 * Policy and value heads (Sec. 3.1, Eq. 3; fp32 parameters, Appendix table):
 * each is an MLP, out = W_L act(... act(W_1 h + b_1) ...) + b_L, accumulated
 * in fp64 and rounded to fp32 once at the output.  The softmax over the
 * logits is the caller's.  h [B, dims[0]], logits [B, A], value [B].
 * ------------------------------------------------------------------------ */
typedef struct brl_mlp {
    int n_layers;                 /* number of weight matrices, 1..8 */
    const int* dims;              /* HOST [n_layers + 1]: in, hidden..., out */
    const float* const* W;        /* HOST array of DEVICE pointers, W[i] is [dims[i+1], dims[i]] */
    const float* const* b;        /* HOST array of DEVICE pointers, b[i] is [dims[i+1]] */
    int act;                      /* BRL_ACT_* between layers */
} brl_mlp;

typedef struct brl_head {
    brl_mlp policy;               /* dims[n_layers] = number of actions A */
    brl_mlp value;                /* dims[n_layers] = 1 */
} brl_head;

size_t brl_head_workspace_bytes(const brl_head* head /* HOST */, int B);
int policy_value_head(const brl_head* head /* HOST */, const float* h, int B,
                      float* logits, float* value,
                      void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Ensemble critic (Sec. 5.3, component ablations: "3x / 5x 1-bit critics
 * (avg)"): n_members value heads of identical shape read the same h; every
 * layer of all members runs in one launch.  values_each[e][b] is member e's
 * head output exactly as policy_value_head computes a value; value_mean[b] =
 * (sum over members in member order, in fp64) / n_members, rounded to fp32.
 * members: HOST array of n_members (1..8) heads with equal n_layers, dims and
 * act, output width 1.  h [B, dims[0]]; value_mean [B]; values_each
 * [n_members, B] or NULL.
 * ------------------------------------------------------------------------ */
size_t brl_value_ensemble_workspace_bytes(const brl_mlp* members /* HOST */, int n_members, int B);
int value_ensemble_forward(const brl_mlp* members /* HOST */, int n_members, const float* h, int B,
                           float* value_mean, float* values_each,
                           void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Training of the two heads on a cached rollout (Sec. 3.1 Eq. 1; Sec. 3.2;
 * Appendix hyper-parameter table).  The backbone is frozen, so the encoder
 * output h_t of every rollout step is stored once and an update touches only
 * the heads.
 *
 * ppo_gae: generalised advantage estimate of n_envs independent rollouts of T
 * steps (arrays [n_envs, T], env-major; last_value [n_envs] bootstraps V after
 * the last step; dones[e, t] = 1 when the episode ended with step t):
 *   delta_t = r_t + gamma V_{t+1} (1 - done_t) - V_t,
 *   A_t = delta_t + gamma lambda (1 - done_t) A_{t+1},   returns = A + V,
 * accumulated backwards in fp64, stored as fp32.
 *
 * ppo_head_update: for epoch e = 0 .. epochs-1 the rollout indices perm[e, :]
 * (DEVICE [epochs, T] int32, the shuffles are the caller's random draws) are
 * cut into T / batch mini-batches (a remainder is dropped); each mini-batch is
 * one optimiser step on both heads:
 *   advantages normalised over the mini-batch, (A - mean) / (std_{n-1} + adv_eps),
 *     if normalize_adv;
 *   L_pi = -mean min(r A, clip(r, 1 - clip_eps, 1 + clip_eps) A) - ent_coef mean H,
 *     r = exp(log pi(a_t | h_t) - logp_old_t), H the entropy of pi(. | h_t);
 *   L_V = 0.5 mean (V(h_t) - returns_t)^2;
 *   all gradients scaled by min(1, max_grad_norm / (||g||_2 + 1e-6)), one norm
 *     over both heads;
 *   Adam with bias correction, rate lr_policy on the policy head's tensors and
 *     lr_value on the value head's.
 * Parameters live in ONE flat fp32 DEVICE buffer (policy W_1, b_1, ..., W_L,
 * b_L, then the value head likewise; brl_ppo_param_offsets gives each tensor's
 * offset so a brl_head for policy_value_head can point into it), adam_m and
 * adam_v likewise (zero them before the first update).  *adam_step (HOST)
 * counts optimiser steps across calls.  h [T, dims[0]] fp32, actions [T]
 * int32, logp_old / adv / returns [T] fp32.  stats (DEVICE, or NULL):
 * [epochs * (T / batch), 5] = policy loss, value loss, mean entropy, fraction
 * of clipped samples, gradient norm before clipping.  Sums run in fp64 in a
 * fixed order: the result does not depend on scheduling.
 * perm entries must lie in [0, T) and actions in [0, A): they are read on the
 * device only and clamped into range there (an entry outside the range gives a
 * meaningless update, never an out-of-bounds access).
 * The Adam bias corrections of each optimiser step are computed on the HOST
 * from *adam_step and passed to the kernels by value: do not capture
 * ppo_head_update into a HIP graph - a replay would reuse the corrections (and
 * step count) of the captured call.
 * ------------------------------------------------------------------------ */
typedef struct brl_ppo_config {
    int policy_layers;            /* 1..8 weight matrices */
    const int* policy_dims;       /* HOST [policy_layers + 1]: in, hidden..., actions */
    int value_layers;
    const int* value_dims;        /* HOST [value_layers + 1]: in, hidden..., 1 */
    int act;                      /* BRL_ACT_* between layers */
    float clip_eps, ent_coef, max_grad_norm, lr_policy, lr_value;
    float adam_b1, adam_b2, adam_eps, adv_eps;
    int normalize_adv;
} brl_ppo_config;

size_t brl_ppo_param_count(const brl_ppo_config* cfg /* HOST */);
int brl_ppo_param_offsets(const brl_ppo_config* cfg, size_t* w_offsets, size_t* b_offsets /* HOST [policy_layers + value_layers] each */);
size_t brl_ppo_workspace_bytes(const brl_ppo_config* cfg, int batch);
int ppo_gae(const float* rewards, const float* values, const float* dones, const float* last_value,
            int n_envs, int T, float gamma, float lam, float* adv, float* returns, void* stream);
int ppo_head_update(const brl_ppo_config* cfg /* HOST */, float* params, float* adam_m, float* adam_v,
                    long long* adam_step /* HOST */,
                    const float* h, const int32_t* actions, const float* logp_old, const float* adv,
                    const float* returns, int T, const int32_t* perm, int epochs, int batch,
                    float* stats, void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Per-kernel timing with HIP events, for measurement harnesses (off by
 * default; not a paper operation).  While enabled, every kernel launch of the
 * library is bracketed by two events recorded on the launch stream.
 * brl_timing_read() waits for the events recorded so far in one class, returns
 * their number and summed elapsed milliseconds, and forgets them.  Enabling
 * costs two event records per launch; do not enable under graph capture.
 * ------------------------------------------------------------------------ */
#define BRL_KC_QUANTIZE_WEIGHTS 0
#define BRL_KC_ACT_QUANT        1   /* activation quantisation incl. fused norm / GLU */
#define BRL_KC_GEMM             2   /* int8 MFMA BitLinear, 128 x 256 workgroup tile (the many-token kernel) */
#define BRL_KC_GEMV             3   /* 1..4 token BitLinear */
#define BRL_KC_ATTENTION        4
#define BRL_KC_OTHER            5   /* embedding, pooling, heads, fills */
#define BRL_KC_GEMM_NARROW      6   /* int8 MFMA BitLinear, 128 x 128 tile and the few-token kernels */
#define BRL_KC_GEMM_QKV_ATTN    7   /* the 128 x 256 tile on the q | k | v product, writing the attention kernel's operands */
#define BRL_KC_COUNT            8

int brl_timing_enable(int on);
int brl_timing_read(int kernel_class, long long* launches, double* total_ms);
/* Same, and also the int8 operations (2 per multiply-accumulate, padding excluded) of the
 * launches read; 0 for classes that are not matrix products. */
int brl_timing_read_ops(int kernel_class, long long* launches, double* total_ms, double* int8_ops);

#ifdef __cplusplus
}
#endif
#endif /* BITRL_H */
