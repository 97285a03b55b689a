"""Seeded synthetic inputs for the ternary-encoder hot path.

This module only draws numbers: it holds none of the method's arithmetic and
is the one piece of code that both the CPU oracle's tests and the GPU
library's tests feed from.  Every tensor comes from its own counter-based
Philox stream keyed by (seed, stream id), so any tensor can be regenerated
alone, in any order, on any machine.

The shapes and distributions stand in for a pretrained BitNet-b1.58 style
backbone and tokenised RL states: weights ~ N(0, 0.02^2) (about 31 % zeros
after ternarisation), activations ~ N(0, 1), norm gains 1 + 0.1 N(0, 1) (so a
dropped gain is visible), token ids uniform over the vocabulary.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def normal(seed: int, stream: int, shape, scale: float = 1.0, shift: float = 0.0) -> np.ndarray:
    """fp32 tensor of shift + scale * N(0, 1)."""
    x = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    if shift != 0.0:
        x += np.float32(shift)
    return x


def token_ids(seed: int, stream: int, shape, vocab: int) -> np.ndarray:
    """int32 token ids uniform on [0, vocab)."""
    return _rng(seed, stream).integers(0, vocab, size=shape, dtype=np.int32)


def state_lengths(seed: int, stream: int, n: int, lo: int, hi: int) -> np.ndarray:
    """int32 state lengths uniform on [lo, hi]."""
    return _rng(seed, stream).integers(lo, hi + 1, size=n, dtype=np.int32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """The fp32 values of bf16 bit patterns (exact widening)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- workloads

@dataclass(frozen=True)
class EncoderShape:
    name: str
    n_layers: int
    d: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    f: int
    vocab: int
    rope_theta: float
    n_actions: int = 18
    head_hidden: Tuple[int, ...] = (256,)


# 2B-parameter BitNet-b1.58 shape (the backbone size the paper freezes).
SHAPE_2B = EncoderShape("bitnet-2b", 30, 2560, 20, 5, 128, 6912, 128256, 500000.0)
# 3B shape used for the large-batch prefill regime.
SHAPE_3B = EncoderShape("bitnet-3b", 26, 3200, 32, 32, 100, 8640, 32000, 10000.0)


def tiny_shape(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=64, f=384, vocab=512,
               rope_theta=10000.0, n_actions=6, head_hidden=(32,)) -> EncoderShape:
    return EncoderShape("tiny", n_layers, d, n_heads, n_kv_heads, head_dim, f, vocab,
                        rope_theta, n_actions, tuple(head_hidden))


W_STD = 0.02


def bitlinear_case(seed: int, n: int, k: int, m: int) -> Dict[str, np.ndarray]:
    """One BitLinear layer: W[n, k] ~ N(0, .02^2), X[m, k] ~ N(0, 1)."""
    return {"W": normal(seed, 1, (n, k), W_STD), "X": normal(seed, 2, (m, k))}


def gemv_pair_case(seed: int, d: int = 2560, f: int = 6912, pair: int = 0) -> Dict[str, np.ndarray]:
    """Decode-shape pair: x[1, d] through W_up[f, d] then W_down[d, f]."""
    base = 16 * pair
    return {"x": normal(seed, 10, (1, d)),
            "W_up": normal(seed, 11 + base, (f, d), W_STD),
            "W_down": normal(seed, 12 + base, (d, f), W_STD)}


def ffn_case(seed: int, m: int, d: int = 2560, f: int = 6912) -> Dict[str, np.ndarray]:
    """One FFN block: bf16-valued input, gains 1 + 0.1 N, three weight matrices."""
    x_bits = to_bf16_bits(normal(seed, 20, (m, d)))
    return {"x_bf16": x_bits,
            "norm_g": normal(seed, 21, (d,), 0.1, 1.0),
            "W_gate": normal(seed, 22, (f, d), W_STD),
            "W_up": normal(seed, 23, (f, d), W_STD),
            "subln_g": normal(seed, 24, (f,), 0.1, 1.0),
            "W_down": normal(seed, 25, (d, f), W_STD)}


def _layer_stream(layer: int, j: int) -> int:
    return 1000 + 16 * layer + j


def encoder_layer(seed: int, shape: EncoderShape, layer: int) -> Dict[str, np.ndarray]:
    """fp32 master weights and gains of one transformer layer."""
    d, f = shape.d, shape.f
    dq = shape.n_heads * shape.head_dim
    dkv = shape.n_kv_heads * shape.head_dim
    st = lambda j: _layer_stream(layer, j)
    return {"attn_norm_g": normal(seed, st(0), (d,), 0.1, 1.0),
            "Wq": normal(seed, st(1), (dq, d), W_STD),
            "Wk": normal(seed, st(2), (dkv, d), W_STD),
            "Wv": normal(seed, st(3), (dkv, d), W_STD),
            "attn_subln_g": normal(seed, st(4), (dq,), 0.1, 1.0),
            "Wo": normal(seed, st(5), (d, dq), W_STD),
            "ffn_norm_g": normal(seed, st(6), (d,), 0.1, 1.0),
            "W_gate": normal(seed, st(7), (f, d), W_STD),
            "W_up": normal(seed, st(8), (f, d), W_STD),
            "ffn_subln_g": normal(seed, st(9), (f,), 0.1, 1.0),
            "W_down": normal(seed, st(10), (d, f), W_STD)}


def embedding_bf16(seed: int, shape: EncoderShape) -> np.ndarray:
    """Embedding table [vocab, d] as bf16 bit patterns, N(0, 1)."""
    g = _rng(seed, 100)
    out = np.empty((shape.vocab, shape.d), dtype=np.uint16)
    step = 8192
    for r0 in range(0, shape.vocab, step):
        r1 = min(shape.vocab, r0 + step)
        out[r0:r1] = to_bf16_bits(g.standard_normal(size=(r1 - r0, shape.d), dtype=np.float32))
    return out


def final_norm_gain(seed: int, shape: EncoderShape) -> np.ndarray:
    return normal(seed, 101, (shape.d,), 0.1, 1.0)


def head_params(seed: int, shape: EncoderShape, which: str) -> Tuple[list, list]:
    """fp32 MLP parameters: W ~ N(0, 1/fan_in), b ~ 0.1 N(0, 1)."""
    base = {"policy": 200, "value": 300}[which]
    out_dim = shape.n_actions if which == "policy" else 1
    dims = (shape.d,) + tuple(shape.head_hidden) + (out_dim,)
    ws, bs = [], []
    for i in range(len(dims) - 1):
        ws.append(normal(seed, base + 2 * i, (dims[i + 1], dims[i]), 1.0 / np.sqrt(dims[i])))
        bs.append(normal(seed, base + 2 * i + 1, (dims[i + 1],), 0.1))
    return ws, bs


def ppo_rollout_case(seed: int, T: int, d: int, n_actions: int, epochs: int, n_envs: int = 1) -> Dict[str, np.ndarray]:
    """A cached rollout for the head update: encoder outputs, actions, behaviour log-probabilities, rewards,
    value predictions, episode ends, bootstrap values and the mini-batch shuffles (one permutation per epoch)."""
    g = _rng(seed, 40)
    n = T * n_envs
    return {"h": normal(seed, 41, (n, d), 0.5),
            "actions": g.integers(0, n_actions, size=n, dtype=np.int32),
            "logp_old": (np.log(1.0 / n_actions) + 0.15 * normal(seed, 42, (n,))).astype(np.float32),
            "rewards": normal(seed, 43, (n_envs, T)),
            "values": normal(seed, 44, (n_envs, T), 0.7),
            "dones": (g.random(size=(n_envs, T)) < 0.03).astype(np.float32),
            "last_value": normal(seed, 45, (n_envs,), 0.7),
            "perm": np.stack([g.permutation(n) for _ in range(max(epochs, 1))]).astype(np.int32)[:epochs].reshape(epochs, n)}


def mlp_params(seed: int, stream: int, dims) -> Tuple[list, list]:
    """fp32 weights N(0, 1/fan_in) and biases 0.1 N(0, 1) for a layer list."""
    ws, bs = [], []
    for i in range(len(dims) - 1):
        ws.append(normal(seed, stream + 2 * i, (dims[i + 1], dims[i]), 1.0 / np.sqrt(dims[i])))
        bs.append(normal(seed, stream + 2 * i + 1, (dims[i + 1],), 0.1))
    return ws, bs
