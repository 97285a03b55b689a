"""CPU oracle for the frozen ternary-encoder forward pass of BitRL.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
GPU library is checked against.  Nothing in the product path may import it:
only the test-suite, the smoke check and the CPU-baseline leg of the benchmark
do.  It shares no code, tables or helpers with the HIP path and imports
nothing from the package.

Everything is NumPy on the host.  Each fp32 operation below is one NumPy
ufunc call on float32 arrays, i.e. one individually rounded IEEE operation in
the written order (NumPy never contracts a*b+c into an FMA across ufuncs).
Integer stages are exact.  Statistics that feed a rounding decision (the
absmean of a weight matrix, the mean square of RMSNorm) are accumulated in
fp64 and rounded to fp32 once.

What the paper fixes and what it leaves open
--------------------------------------------
The paper defines the ternary code as sign(W) * 1[|W| > tau] (Sec. 3.1,
Eq. 2) with tau depending on the weight distribution (Sec. 4, Def. 4.1), the
composition h_t = f(serialize(s_t)), pi = softmax(g(h_t)), V = v(h_t)
(Sec. 3.1, Eq. 3), integer-only ternary matmul (Sec. 3.1, last paragraph) and
fp32 heads (Appendix, hyper-parameter table).  It is silent on the activation
quantiser, scales, norms, attention and pooling; those follow the BitNet
b1.58 scheme the paper cites as its backbone (absmean weights with
tau = (mean|W| + eps)/2, per-token absmax int8 activations with Qb = 127 and
round-half-to-even, int32 accumulation, RMSNorm / sub-layer-norm blocks,
squared-ReLU GLU, rotary causal grouped-query attention).  Every such reading
is listed in the design document of the repository.

Parity pins: every function here is pinned by tests/test_oracle_pins.py
against brute force, closed forms, hand-computed cases or invariants, except
the end-to-end value of `encoder_forward`, for which nothing independent
exists beyond the composition of its pinned stages ("parity unpinned" beyond
stage composition).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32
F64 = np.float64

QB = 127  # int8 activation range bound (Qb), symmetric: codes in [-127, 127]


# --------------------------------------------------------------------------
# BitLinear: weights (Sec. 3.1, Eq. 2)
# --------------------------------------------------------------------------

def ternary_quantize(W: np.ndarray, eps: float = 1e-5) -> Tuple[np.ndarray, np.float32]:
    """Ternary code of a weight matrix W[N, K] (Sec. 3.1, Eq. 2).

    gamma = mean |W| over the whole matrix (fp64 sum, one rounding to fp32);
    beta  = gamma + eps (fp32 add); tau = beta / 2 (exact in fp32);
    code  = +1 where W > tau, -1 where W < -tau, else 0.  The strict
    inequality of Eq. 2 sends |w| == tau to 0.  beta is also the dequant
    scale: beta * code is the weight the matmul stands for.

    Returns (codes int8 [N, K], beta float32 scalar).
    """
    W = np.asarray(W, dtype=F32)
    if W.ndim != 2:
        raise ValueError("W must be [N, K]")
    n, k = W.shape
    total = np.sum(np.abs(W).astype(F64))
    if not np.isfinite(total):
        raise ValueError("non-finite weights")
    gamma = F32(total / float(n * k))
    beta = F32(gamma + F32(eps))
    tau = F32(0.5) * beta
    codes = (W > tau).astype(np.int8) - (W < -tau).astype(np.int8)
    return codes, beta


# --------------------------------------------------------------------------
# BitLinear: activations
# --------------------------------------------------------------------------

def act_quant(x: np.ndarray, eps: float = 1e-5) -> Tuple[np.ndarray, np.ndarray]:
    """Per-token absmax int8 quantisation of x[M, K] (fp32).

    a_t = max_k |x_tk|; a'_t = max(a_t, eps); s_t = 127 / a'_t (fp32 divide);
    q_tk = clamp(round_half_even(x_tk * s_t), -127, 127).

    Returns (q int8 [M, K], a' float32 [M]).
    """
    x = np.asarray(x, dtype=F32)
    a = np.max(np.abs(x), axis=-1)
    a_c = np.maximum(a, F32(eps)).astype(F32)
    s = (F32(QB) / a_c).astype(F32)
    t = (x * s[:, None]).astype(F32)
    q = np.clip(np.rint(t), -QB, QB).astype(np.int8)
    return q, a_c


def ternary_matmul(q: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """acc[t, n] = sum_k q[t, k] * codes[n, k], exact, as int32.

    The contraction is done by the fp64 BLAS on integer-valued operands: every
    partial sum is an integer of magnitude <= 127 * 127 * K < 2**53 (codes of
    magnitude up to 127 are allowed: the int8-weight critic variant shares this
    routine), so each fp64 operation is exact and the result equals the
    integer sum in any order.
    """
    q = np.asarray(q)
    codes = np.asarray(codes)
    k = q.shape[-1]
    assert codes.shape[-1] == k
    assert QB * QB * k < 2 ** 31
    acc = q.astype(F64) @ codes.astype(F64).T
    return np.rint(acc).astype(np.int32)


def dequant(acc: np.ndarray, a_c: np.ndarray, beta, residual: Optional[np.ndarray] = None) -> np.ndarray:
    """y[t, n] = (float(acc[t, n]) * (a'_t / 127)) * beta (+ residual), fp32."""
    d = (np.asarray(a_c, dtype=F32) / F32(QB)).astype(F32)
    y = (acc.astype(F32) * d[:, None]).astype(F32)
    y = (y * F32(beta)).astype(F32)
    if residual is not None:
        y = (y + np.asarray(residual, dtype=F32)).astype(F32)
    return y


def bitlinear_forward(x: np.ndarray, codes: np.ndarray, beta, eps: float = 1e-5,
                      residual: Optional[np.ndarray] = None, taps: Optional[dict] = None) -> np.ndarray:
    """BitLinear: quantise activations, integer matmul, rescale.

    No normalisation happens inside; norms are explicit members of the blocks.
    `taps`, if given, receives the integer stages (xq, absmax, acc).
    """
    q, a_c = act_quant(x, eps)
    acc = ternary_matmul(q, codes)
    if taps is not None:
        taps.update(xq=q, absmax=a_c, acc=acc)
    return dequant(acc, a_c, beta, residual)


# --------------------------------------------------------------------------
# Norms and the FFN block
# --------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, g: np.ndarray, eps_n: float = 1e-5) -> np.ndarray:
    """y_k = (x_k * r) * g_k with r = fp32(1 / sqrt(mean_k x_k^2 + eps_n)).

    The statistic is taken in fp64 (eps_n enters as the fp32 value widened),
    the scaling in fp32: first by r, then by the gain.
    """
    x = np.asarray(x, dtype=F32)
    g = np.asarray(g, dtype=F32)
    k = x.shape[-1]
    x64 = x.astype(F64)
    ms = np.sum(x64 * x64, axis=-1) / float(k)
    r = (1.0 / np.sqrt(ms + F64(F32(eps_n)))).astype(F32)
    y = (x * r[..., None]).astype(F32)
    return (y * g).astype(F32)


def squared_relu_glu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """h = (max(gate, 0) * max(gate, 0)) * up, fp32, in that order."""
    p = np.maximum(np.asarray(gate, dtype=F32), F32(0))
    return ((p * p).astype(F32) * np.asarray(up, dtype=F32)).astype(F32)


@dataclass
class TernaryLinear:
    """A frozen BitLinear weight: ternary codes [N, K] and its scale beta."""
    codes: np.ndarray
    beta: np.float32

    @staticmethod
    def from_fp32(W: np.ndarray, eps: float = 1e-5) -> "TernaryLinear":
        c, b = ternary_quantize(W, eps)
        return TernaryLinear(c, b)


@dataclass
class FFNWeights:
    norm_g: np.ndarray      # [d]   gain of the pre-FFN RMSNorm
    gate: TernaryLinear     # [f, d]
    up: TernaryLinear       # [f, d]
    subln_g: np.ndarray     # [f]   gain of the sub-layer norm before `down`
    down: TernaryLinear     # [d, f]


def ffn_block_forward(x: np.ndarray, w: FFNWeights, eps: float = 1e-5, eps_n: float = 1e-5,
                      taps: Optional[dict] = None) -> np.ndarray:
    """y = x + down(subLN(sqReLU-GLU(gate(n), up(n)))), n = RMSNorm(x).

    n is quantised once and shared by gate and up (each with its own beta).
    x holds fp32 values (a bf16 input is widened by the caller, exactly).
    """
    x = np.asarray(x, dtype=F32)
    n = rmsnorm(x, w.norm_g, eps_n)
    q, a_c = act_quant(n, eps)
    G = dequant(ternary_matmul(q, w.gate.codes), a_c, w.gate.beta)
    U = dequant(ternary_matmul(q, w.up.codes), a_c, w.up.beta)
    h = squared_relu_glu(G, U)
    m = rmsnorm(h, w.subln_g, eps_n)
    q2, a2 = act_quant(m, eps)
    acc2 = ternary_matmul(q2, w.down.codes)
    if taps is not None:
        taps.update(xq=q, absmax=a_c, gate=G, up=U, h=h, hq=q2, habsmax=a2, acc_down=acc2)
    return dequant(acc2, a2, w.down.beta, residual=x)


# --------------------------------------------------------------------------
# Attention (plain definition, fp64)
# --------------------------------------------------------------------------

def rope(x: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding of x[S, H, dh] in fp64, rotate-half pairing (i, i+dh/2).

    Position p is the index inside the state; pair i turns by p * theta**(-2i/dh).
    """
    s, _, dh = x.shape
    half = dh // 2
    inv_freq = np.power(F64(theta), -(2.0 * np.arange(half, dtype=F64)) / F64(dh))
    ang = np.arange(s, dtype=F64)[:, None] * inv_freq[None, :]
    c = np.cos(ang)[:, None, :]
    sn = np.sin(ang)[:, None, :]
    x = x.astype(F64)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * sn, x2 * c + x1 * sn], axis=-1)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, theta: float) -> np.ndarray:
    """softmax(rope(q) rope(k)^T / sqrt(dh), causal) v for one state.

    q[S, Hq, dh], k and v[S, Hkv, dh] hold fp32 values; query head h reads
    key/value head h // (Hq / Hkv).  All arithmetic in fp64; the result
    [S, Hq * dh] is rounded to fp32 once.
    """
    s, hq, dh = q.shape
    hkv = k.shape[1]
    group = hq // hkv
    qr = rope(q, theta)
    kr = rope(k, theta)
    v64 = v.astype(F64)
    out = np.empty((s, hq, dh), dtype=F64)
    mask = np.tril(np.ones((s, s), dtype=bool))
    scale = 1.0 / math.sqrt(dh)
    for h in range(hq):
        j = h // group
        sc = (qr[:, h, :] @ kr[:, j, :].T) * scale
        sc = np.where(mask, sc, -np.inf)
        sc = sc - sc.max(axis=-1, keepdims=True)
        p = np.exp(sc)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ v64[:, j, :]
    return out.reshape(s, hq * dh).astype(F32)


# --------------------------------------------------------------------------
# Encoder
# --------------------------------------------------------------------------

@dataclass
class LayerWeights:
    attn_norm_g: np.ndarray   # [d]
    wq: TernaryLinear         # [Hq*dh, d]
    wk: TernaryLinear         # [Hkv*dh, d]
    wv: TernaryLinear         # [Hkv*dh, d]
    attn_subln_g: np.ndarray  # [Hq*dh]
    wo: TernaryLinear         # [d, Hq*dh]
    ffn: FFNWeights


@dataclass
class EncoderConfig:
    n_layers: int
    d: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    f: int
    vocab: int
    rope_theta: float
    eps_norm: float = 1e-5
    eps_quant: float = 1e-5


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the same values as fp32 (exact)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(F32)


def attention_block_forward(x: np.ndarray, lw: LayerWeights, cfg: EncoderConfig,
                            taps: Optional[dict] = None) -> np.ndarray:
    """x + o(subLN(attention(q(n), k(n), v(n)))), n = RMSNorm(x), one state x[S, d]."""
    s = x.shape[0]
    n = rmsnorm(x, lw.attn_norm_g, cfg.eps_norm)
    qn, a_c = act_quant(n, cfg.eps_quant)
    q = dequant(ternary_matmul(qn, lw.wq.codes), a_c, lw.wq.beta)
    k = dequant(ternary_matmul(qn, lw.wk.codes), a_c, lw.wk.beta)
    v = dequant(ternary_matmul(qn, lw.wv.codes), a_c, lw.wv.beta)
    att = causal_gqa_attention(q.reshape(s, cfg.n_heads, cfg.head_dim),
                               k.reshape(s, cfg.n_kv_heads, cfg.head_dim),
                               v.reshape(s, cfg.n_kv_heads, cfg.head_dim), cfg.rope_theta)
    m = rmsnorm(att, lw.attn_subln_g, cfg.eps_norm)
    if taps is not None:
        taps.update(q=q, k=k, v=v, att=att)
    return bitlinear_forward(m, lw.wo.codes, lw.wo.beta, cfg.eps_quant, residual=x)


def encoder_forward(ids: np.ndarray, emb_bf16_bits: np.ndarray, layers: Sequence[LayerWeights],
                    final_norm_g: np.ndarray, cfg: EncoderConfig,
                    lengths: Optional[np.ndarray] = None, layer_taps: Optional[list] = None) -> np.ndarray:
    """h[b] = mean over the state's positions of RMSNorm_final(x_L[b, s]) (Sec. 3.1, Eq. 3).

    ids[B, S] int32; the embedding table holds bf16 values (given as bit
    patterns, widened exactly).  States are independent.  With `lengths`, the
    mean runs over the first lengths[b] positions (causality already keeps
    them blind to the padding behind them).  The mean is an fp64 sum divided
    by the count, rounded to fp32 once.
    """
    ids = np.asarray(ids)
    b_states, s = ids.shape
    h = np.empty((b_states, cfg.d), dtype=F32)
    for b in range(b_states):
        x = widen_bf16(emb_bf16_bits[ids[b]])
        for li, lw in enumerate(layers):
            x = attention_block_forward(x, lw, cfg)
            x = ffn_block_forward(x, lw.ffn, cfg.eps_quant, cfg.eps_norm)
            if layer_taps is not None and b == 0:
                layer_taps.append(x.copy())
        xf = rmsnorm(x, final_norm_g, cfg.eps_norm)
        n_b = s if lengths is None else int(lengths[b])
        h[b] = (np.sum(xf[:n_b].astype(F64), axis=0) / float(n_b)).astype(F32)
    return h


# --------------------------------------------------------------------------
# Heads (Sec. 3.1, Eq. 3; Appendix hyper-parameter table: fp32 heads)
# --------------------------------------------------------------------------

@dataclass
class MLP:
    """Fully connected head: hidden layers with an activation, linear output."""
    weights: List[np.ndarray]   # weights[i] is [out_i, in_i], fp32
    biases: List[np.ndarray]    # biases[i] is [out_i], fp32
    act: str = "tanh"           # "tanh" or "relu"


def mlp_forward(h: np.ndarray, mlp: MLP) -> np.ndarray:
    """Plain definition in fp64 on the fp32 parameters; rounded to fp32 once."""
    z = np.asarray(h, dtype=F32).astype(F64)
    n = len(mlp.weights)
    for i, (w, b) in enumerate(zip(mlp.weights, mlp.biases)):
        z = z @ np.asarray(w, dtype=F32).astype(F64).T + np.asarray(b, dtype=F32).astype(F64)
        if i + 1 < n:
            if mlp.act == "tanh":
                z = np.tanh(z)
            elif mlp.act == "relu":
                z = np.maximum(z, 0.0)
            else:
                raise ValueError(mlp.act)
    return z.astype(F32)


def policy_value_head(h: np.ndarray, policy: MLP, value: MLP) -> Tuple[np.ndarray, np.ndarray]:
    """logits[B, A] = g(h), value[B] = v(h); separate parameters for each head."""
    logits = mlp_forward(h, policy)
    val = mlp_forward(h, value)
    return logits, val.reshape(val.shape[0])


def softmax(logits: np.ndarray) -> np.ndarray:
    """pi(a|s) = softmax(g(h)) (Sec. 3.1, Eq. 3); applied by callers, kept here for checks."""
    z = np.asarray(logits, dtype=F64)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)
