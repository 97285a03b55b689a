"""ctypes binding of libbitrl.so: argument marshalling only.

Every function below has the name and the argument order of its C entry point
(include/bitrl.h).  Tensors are torch tensors on the GPU (torch is used for
device memory and streams, nothing else); every step of the computation runs
in the library's kernels.  A missing library is an error, never a fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libbitrl.so")

BRL_OK, BRL_EINVAL, BRL_ENOSPC, BRL_EHIP = 0, 1, 2, 3
BRL_F32, BRL_BF16 = 0, 1
BRL_ACT_TANH, BRL_ACT_RELU = 0, 1
BRL_ATTN_F32, BRL_ATTN_MFMA = 0, 1
BRL_W_TERNARY, BRL_W_INT8 = 0, 1

c_void_p, c_int, c_float, c_size_t = C.c_void_p, C.c_int, C.c_float, C.c_size_t


class brl_ffn_weights(C.Structure):
    _fields_ = [("norm_g", c_void_p), ("gate_packed", c_void_p), ("gate_beta", c_void_p),
                ("up_packed", c_void_p), ("up_beta", c_void_p), ("subln_g", c_void_p),
                ("down_packed", c_void_p), ("down_beta", c_void_p)]


class brl_layer_weights(C.Structure):
    _fields_ = [("attn_norm_g", c_void_p),
                ("wq_packed", c_void_p), ("wq_beta", c_void_p),
                ("wk_packed", c_void_p), ("wk_beta", c_void_p),
                ("wv_packed", c_void_p), ("wv_beta", c_void_p),
                ("attn_subln_g", c_void_p),
                ("wo_packed", c_void_p), ("wo_beta", c_void_p),
                ("ffn", brl_ffn_weights)]


class brl_encoder(C.Structure):
    _fields_ = [("n_layers", c_int), ("d", c_int), ("n_heads", c_int), ("n_kv_heads", c_int),
                ("head_dim", c_int), ("f", c_int), ("vocab", c_int),
                ("rope_theta", c_float), ("eps_norm", c_float), ("eps_act", c_float),
                ("attn_precision", c_int), ("weight_format", c_int),
                ("embedding", c_void_p), ("final_norm_g", c_void_p),
                ("layers", C.POINTER(brl_layer_weights))]


class brl_mlp(C.Structure):
    _fields_ = [("n_layers", c_int), ("dims", C.POINTER(c_int)),
                ("W", C.POINTER(c_void_p)), ("b", C.POINTER(c_void_p)), ("act", c_int)]


class brl_head(C.Structure):
    _fields_ = [("policy", brl_mlp), ("value", brl_mlp)]


class BitrlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("bitrl status %d: %s" % (status, message))
        self.status = status


_lib = None

class brl_ppo_config(C.Structure):
    _fields_ = [("policy_layers", c_int), ("policy_dims", C.POINTER(c_int)),
                ("value_layers", c_int), ("value_dims", C.POINTER(c_int)),
                ("act", c_int),
                ("clip_eps", c_float), ("ent_coef", c_float), ("max_grad_norm", c_float),
                ("lr_policy", c_float), ("lr_value", c_float),
                ("adam_b1", c_float), ("adam_b2", c_float), ("adam_eps", c_float), ("adv_eps", c_float),
                ("normalize_adv", c_int)]


_SIGNATURES = {
    "brl_last_error": (C.c_char_p, []),
    "brl_abi_version": (c_int, []),
    "brl_packed_bytes": (c_size_t, [c_int, c_int]),
    "brl_quantize_workspace_bytes": (c_size_t, [c_int, c_int]),
    "bitlinear_quantize_weights": (c_int, [c_void_p, c_int, c_int, c_float, c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_size_t, c_void_p]),
    "brl_unpack_codes": (c_int, [c_void_p, c_int, c_int, c_void_p, c_void_p]),
    "brl_bitlinear_workspace_bytes": (c_size_t, [c_int, c_int, c_int]),
    "bitlinear_forward": (c_int, [c_void_p, c_void_p, c_int, c_int, c_void_p, c_int, c_int, c_float,
                                  c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "bitlinear_forward_static": (c_int, [c_void_p, c_void_p, c_int, c_int, c_void_p, c_int, c_int, c_float,
                                         c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "brl_packed_int8_bytes": (c_size_t, [c_int, c_int]),
    "bitlinear_quantize_weights_int8": (c_int, [c_void_p, c_int, c_int, c_float, c_int, c_void_p, c_void_p, c_void_p,
                                                c_void_p, c_size_t, c_void_p]),
    "brl_unpack_codes_int8": (c_int, [c_void_p, c_int, c_int, c_void_p, c_void_p]),
    "bitlinear_int8_forward": (c_int, [c_void_p, c_void_p, c_int, c_int, c_void_p, c_int, c_int, c_float,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "brl_value_ensemble_workspace_bytes": (c_size_t, [C.POINTER(brl_mlp), c_int, c_int]),
    "value_ensemble_forward": (c_int, [C.POINTER(brl_mlp), c_int, c_void_p, c_int, c_void_p, c_void_p,
                                       c_void_p, c_size_t, c_void_p]),
    "bitlinear_forward_batch": (c_int, [c_void_p, c_void_p, c_int, c_int, c_void_p, c_int, c_int, c_float,
                                        c_void_p, c_int, c_void_p]),
    "brl_ffn_workspace_bytes": (c_size_t, [c_int, c_int, c_int]),
    "ffn_block_forward": (c_int, [C.POINTER(brl_ffn_weights), c_void_p, c_int, c_int, c_int, c_int, c_float, c_float,
                                  c_void_p, c_void_p, c_size_t, c_void_p]),
    "brl_encoder_workspace_bytes": (c_size_t, [C.POINTER(brl_encoder), c_int, c_int]),
    "encoder_forward": (c_int, [C.POINTER(brl_encoder), c_void_p, c_int, c_int, c_void_p, c_void_p,
                                c_void_p, c_size_t, c_void_p]),
    "brl_encoder_packed_workspace_bytes": (c_size_t, [C.POINTER(brl_encoder), c_int, c_int, c_int]),
    "encoder_forward_packed": (c_int, [C.POINTER(brl_encoder), c_void_p, c_void_p, c_void_p, c_int, c_int, c_void_p,
                                       c_void_p, c_size_t, c_void_p]),
    "brl_attention_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int, c_int]),
    "attention_forward": (c_int, [c_void_p, c_int, c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_float, c_int,
                                  c_void_p, c_void_p, c_size_t, c_void_p]),
    "brl_serialize_text": (c_size_t, [c_void_p, c_int, C.c_char_p, c_size_t]),
    "brl_tokenize": (c_int, [C.c_char_p, c_size_t, c_void_p, c_int, C.POINTER(c_int)]),
    "serialize_states": (c_int, [c_void_p, c_int, c_int, c_int, c_void_p, c_void_p]),
    "brl_head_workspace_bytes": (c_size_t, [C.POINTER(brl_head), c_int]),
    "policy_value_head": (c_int, [C.POINTER(brl_head), c_void_p, c_int, c_void_p, c_void_p,
                                  c_void_p, c_size_t, c_void_p]),
    "brl_ppo_param_count": (c_size_t, [C.POINTER(brl_ppo_config)]),
    "brl_ppo_param_offsets": (c_int, [C.POINTER(brl_ppo_config), C.POINTER(c_size_t), C.POINTER(c_size_t)]),
    "brl_ppo_workspace_bytes": (c_size_t, [C.POINTER(brl_ppo_config), c_int]),
    "ppo_gae": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_float, c_float, c_void_p, c_void_p,
                        c_void_p]),
    "ppo_head_update": (c_int, [C.POINTER(brl_ppo_config), c_void_p, c_void_p, c_void_p, C.POINTER(C.c_longlong),
                                c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_int, c_int,
                                c_void_p, c_void_p, c_size_t, c_void_p]),
    "brl_timing_enable": (c_int, [c_int]),
    "brl_timing_read": (c_int, [c_int, C.POINTER(C.c_longlong), C.POINTER(C.c_double)]),
    "brl_timing_read_ops": (c_int, [c_int, C.POINTER(C.c_longlong), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
}

EXPORTS = tuple(_SIGNATURES)


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: run `python -m paper_2604_24273_amd.build` (hipcc, gfx950) first" % LIB_PATH)
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(status: int) -> None:
    if status != BRL_OK:
        raise BitrlError(status, lib().brl_last_error().decode("utf-8", "replace"))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return BRL_F32
    if t.dtype == torch.bfloat16:
        return BRL_BF16
    raise ValueError("activations must be float32 or bfloat16")


# ---------------------------------------------------------------- entry points

def brl_abi_version() -> int:
    return lib().brl_abi_version()


def brl_packed_bytes(n_out: int, k_in: int) -> int:
    return lib().brl_packed_bytes(n_out, k_in)


def brl_quantize_workspace_bytes(n_out: int, k_in: int) -> int:
    return lib().brl_quantize_workspace_bytes(n_out, k_in)


def bitlinear_quantize_weights(W: torch.Tensor, eps: float, packed_out: torch.Tensor, beta_out: torch.Tensor,
                               codes_dbg: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    n, k = W.shape
    _check(lib().bitlinear_quantize_weights(_ptr(W), n, k, eps, _ptr(packed_out), _ptr(beta_out), _ptr(codes_dbg),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def brl_unpack_codes(packed: torch.Tensor, n_out: int, k_in: int, codes_out: torch.Tensor) -> None:
    _check(lib().brl_unpack_codes(_ptr(packed), n_out, k_in, _ptr(codes_out), _stream()))


def brl_bitlinear_workspace_bytes(M: int, N: int, K: int) -> int:
    return lib().brl_bitlinear_workspace_bytes(M, N, K)


def bitlinear_forward(packed: torch.Tensor, beta: torch.Tensor, N: int, K: int, x: torch.Tensor, M: int, eps_act: float,
                      y: torch.Tensor, residual: Optional[torch.Tensor], xq_dbg: Optional[torch.Tensor],
                      absmax_dbg: Optional[torch.Tensor], acc_dbg: Optional[torch.Tensor],
                      workspace: torch.Tensor) -> None:
    _check(lib().bitlinear_forward(_ptr(packed), _ptr(beta), N, K, _ptr(x), _dtype_code(x), M, eps_act, _ptr(y),
                                   _ptr(residual), _ptr(xq_dbg), _ptr(absmax_dbg), _ptr(acc_dbg), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))


BRL_STATIC_SCRATCH_BYTES = 16 << 20


def bitlinear_forward_static(packed: torch.Tensor, beta: torch.Tensor, N: int, K: int, x: torch.Tensor, M: int,
                             eps_act: float, y: torch.Tensor, residual: Optional[torch.Tensor],
                             xq_dbg: Optional[torch.Tensor], absmax_dbg: Optional[torch.Tensor],
                             acc_dbg: Optional[torch.Tensor]) -> None:
    _check(lib().bitlinear_forward_static(_ptr(packed), _ptr(beta), N, K, _ptr(x), _dtype_code(x), M, eps_act, _ptr(y),
                                          _ptr(residual), _ptr(xq_dbg), _ptr(absmax_dbg), _ptr(acc_dbg), _stream()))


def brl_packed_int8_bytes(n_out: int, k_in: int) -> int:
    return lib().brl_packed_int8_bytes(n_out, k_in)


def bitlinear_quantize_weights_int8(W: torch.Tensor, eps: float, qmax: int, packed_out: torch.Tensor,
                                    scale_out: torch.Tensor, codes_dbg: Optional[torch.Tensor],
                                    workspace: torch.Tensor) -> None:
    n, k = W.shape
    _check(lib().bitlinear_quantize_weights_int8(_ptr(W), n, k, eps, qmax, _ptr(packed_out), _ptr(scale_out), _ptr(codes_dbg),
                                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def brl_unpack_codes_int8(packed: torch.Tensor, n_out: int, k_in: int, codes_out: torch.Tensor) -> None:
    _check(lib().brl_unpack_codes_int8(_ptr(packed), n_out, k_in, _ptr(codes_out), _stream()))


def bitlinear_int8_forward(packed: torch.Tensor, scale: torch.Tensor, N: int, K: int, x: torch.Tensor, M: int,
                           eps_act: float, y: torch.Tensor, residual: Optional[torch.Tensor],
                           xq_dbg: Optional[torch.Tensor], absmax_dbg: Optional[torch.Tensor],
                           acc_dbg: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    _check(lib().bitlinear_int8_forward(_ptr(packed), _ptr(scale), N, K, _ptr(x), _dtype_code(x), M, eps_act, _ptr(y),
                                        _ptr(residual), _ptr(xq_dbg), _ptr(absmax_dbg), _ptr(acc_dbg), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()))


def bitlinear_forward_batch(packed_ptrs: torch.Tensor, beta_ptrs: torch.Tensor, N: int, K: int, x_ptrs: torch.Tensor,
                            x_dtype: int, M: int, eps_act: float, y_ptrs: torch.Tensor, count: int) -> None:
    """The four *_ptrs are int64 device tensors holding device addresses (tensor.data_ptr() values)."""
    _check(lib().bitlinear_forward_batch(_ptr(packed_ptrs), _ptr(beta_ptrs), N, K, _ptr(x_ptrs), x_dtype, M, eps_act,
                                         _ptr(y_ptrs), count, _stream()))


def brl_ffn_workspace_bytes(M: int, d: int, f: int) -> int:
    return lib().brl_ffn_workspace_bytes(M, d, f)


def ffn_block_forward(w: brl_ffn_weights, x: torch.Tensor, M: int, d: int, f: int, eps_norm: float, eps_act: float,
                      y: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(lib().ffn_block_forward(C.byref(w), _ptr(x), _dtype_code(x), M, d, f, eps_norm, eps_act, _ptr(y),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def brl_encoder_workspace_bytes(enc: brl_encoder, B: int, S: int) -> int:
    return lib().brl_encoder_workspace_bytes(C.byref(enc), B, S)


def encoder_forward(enc: brl_encoder, ids: torch.Tensor, B: int, S: int, lengths: Optional[torch.Tensor],
                    h: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(lib().encoder_forward(C.byref(enc), _ptr(ids), B, S, _ptr(lengths), _ptr(h), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()))


def brl_encoder_packed_workspace_bytes(enc: brl_encoder, B: int, T: int, max_len: int) -> int:
    return lib().brl_encoder_packed_workspace_bytes(C.byref(enc), B, T, max_len)


def encoder_forward_packed(enc: brl_encoder, ids: torch.Tensor, cu_seqlens: torch.Tensor, cu_seqlens_host,
                           B: int, max_len: int, h: torch.Tensor, workspace: torch.Tensor) -> None:
    """cu_seqlens: int32 device tensor [B+1]; cu_seqlens_host: contiguous int32 numpy array with the same values."""
    _check(lib().encoder_forward_packed(C.byref(enc), _ptr(ids), _ptr(cu_seqlens), cu_seqlens_host.ctypes.data, B, max_len,
                                        _ptr(h), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _stream()))


def brl_attention_workspace_bytes(B: int, S: int, n_heads: int, n_kv_heads: int, head_dim: int) -> int:
    return lib().brl_attention_workspace_bytes(B, S, n_heads, n_kv_heads, head_dim)


def attention_forward(qkv: torch.Tensor, B: int, S: int, cu_seqlens: Optional[torch.Tensor], cu_seqlens_host,
                      n_heads: int, n_kv_heads: int, head_dim: int, rope_theta: float, attn_precision: int,
                      out: torch.Tensor, workspace: torch.Tensor) -> None:
    """cu_seqlens: int32 device tensor [B+1] or None; cu_seqlens_host: int32 numpy array with the same values or None."""
    _check(lib().attention_forward(_ptr(qkv), B, S, _ptr(cu_seqlens),
                                   None if cu_seqlens_host is None else cu_seqlens_host.ctypes.data,
                                   n_heads, n_kv_heads, head_dim, rope_theta, attn_precision, _ptr(out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))


BRL_SERIALIZE_VOCAB = 457


def brl_serialize_text(state) -> str:
    """state: contiguous float32 numpy array [n_dims] on the host."""
    n = int(state.shape[0])
    need = lib().brl_serialize_text(state.ctypes.data, n, None, 0)
    buf = C.create_string_buffer(need + 1)
    lib().brl_serialize_text(state.ctypes.data, n, buf, need + 1)
    return buf.value.decode("ascii")


def brl_tokenize(text: bytes):
    """ids (list of int) of a byte string under the stand-in vocabulary."""
    import numpy as np
    cap = len(text) + 1
    ids = np.empty(cap, dtype=np.int32)
    n = c_int(0)
    _check(lib().brl_tokenize(text, len(text), ids.ctypes.data, cap, C.byref(n)))
    return [int(i) for i in ids[:n.value]]


def serialize_states(states, vocab: int):
    """states: contiguous float32 numpy array [B, n_dims] on the host -> (ids int32 [B * (n_dims + 2)], cu_seqlens int32 [B + 1])."""
    import numpy as np
    b, n = states.shape
    ids = np.empty(b * (n + 2), dtype=np.int32)
    cu = np.empty(b + 1, dtype=np.int32)
    _check(lib().serialize_states(states.ctypes.data, b, n, vocab, ids.ctypes.data, cu.ctypes.data))
    return ids, cu


def brl_head_workspace_bytes(head: brl_head, B: int) -> int:
    return lib().brl_head_workspace_bytes(C.byref(head), B)


def policy_value_head(head: brl_head, h: torch.Tensor, B: int, logits: torch.Tensor, value: torch.Tensor,
                      workspace: torch.Tensor) -> None:
    _check(lib().policy_value_head(C.byref(head), _ptr(h), B, _ptr(logits), _ptr(value), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))


def brl_value_ensemble_workspace_bytes(members, n_members: int, B: int) -> int:
    return lib().brl_value_ensemble_workspace_bytes(members, n_members, B)


def value_ensemble_forward(members, n_members: int, h: torch.Tensor, B: int, value_mean: torch.Tensor,
                           values_each: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    """members: a ctypes array of brl_mlp (see make_mlp_array)."""
    _check(lib().value_ensemble_forward(members, n_members, _ptr(h), B, _ptr(value_mean), _ptr(values_each),
                                        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def make_ppo_config(policy_dims: Sequence[int], value_dims: Sequence[int], act: int, clip_eps: float = 0.1,
                    ent_coef: float = 0.05, max_grad_norm: float = 0.5, lr_policy: float = 3e-4, lr_value: float = 1e-3,
                    adam_b1: float = 0.9, adam_b2: float = 0.999, adam_eps: float = 1e-8, adv_eps: float = 1e-8,
                    normalize_adv: bool = True):
    """Returns (brl_ppo_config, keepalive); defaults are the paper's hyper-parameter table."""
    pd = (c_int * len(policy_dims))(*policy_dims)
    vd = (c_int * len(value_dims))(*value_dims)
    cfg = brl_ppo_config(len(policy_dims) - 1, pd, len(value_dims) - 1, vd, act, clip_eps, ent_coef, max_grad_norm,
                         lr_policy, lr_value, adam_b1, adam_b2, adam_eps, adv_eps, 1 if normalize_adv else 0)
    return cfg, (pd, vd)


def brl_ppo_param_count(cfg: brl_ppo_config) -> int:
    return lib().brl_ppo_param_count(C.byref(cfg))


def brl_ppo_param_offsets(cfg: brl_ppo_config):
    n = cfg.policy_layers + cfg.value_layers
    w, b = (c_size_t * n)(), (c_size_t * n)()
    _check(lib().brl_ppo_param_offsets(C.byref(cfg), w, b))
    return list(w), list(b)


def brl_ppo_workspace_bytes(cfg: brl_ppo_config, batch: int) -> int:
    return lib().brl_ppo_workspace_bytes(C.byref(cfg), batch)


def ppo_gae(rewards: torch.Tensor, values: torch.Tensor, dones: torch.Tensor, last_value: torch.Tensor, n_envs: int,
            T: int, gamma: float, lam: float, adv: torch.Tensor, returns: torch.Tensor) -> None:
    _check(lib().ppo_gae(_ptr(rewards), _ptr(values), _ptr(dones), _ptr(last_value), n_envs, T, gamma, lam, _ptr(adv),
                         _ptr(returns), _stream()))


def ppo_head_update(cfg: brl_ppo_config, params: torch.Tensor, adam_m: torch.Tensor, adam_v: torch.Tensor, adam_step: int,
                    h: torch.Tensor, actions: torch.Tensor, logp_old: torch.Tensor, adv: torch.Tensor,
                    returns: torch.Tensor, T: int, perm: torch.Tensor, epochs: int, batch: int,
                    stats: Optional[torch.Tensor], workspace: torch.Tensor) -> int:
    """Returns the optimiser step count after the update."""
    step = C.c_longlong(adam_step)
    _check(lib().ppo_head_update(C.byref(cfg), _ptr(params), _ptr(adam_m), _ptr(adam_v), C.byref(step), _ptr(h),
                                 _ptr(actions), _ptr(logp_old), _ptr(adv), _ptr(returns), T, _ptr(perm), epochs, batch,
                                 _ptr(stats), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
    return step.value


BRL_KC_QUANTIZE_WEIGHTS, BRL_KC_ACT_QUANT, BRL_KC_GEMM, BRL_KC_GEMV, BRL_KC_ATTENTION, BRL_KC_OTHER, \
    BRL_KC_GEMM_NARROW, BRL_KC_GEMM_QKV_ATTN = range(8)
KERNEL_CLASSES = ("quantize_weights", "act_quant", "gemm", "gemv", "attention", "other", "gemm_narrow", "gemm_qkv_attn")


def brl_timing_enable(on: bool) -> None:
    _check(lib().brl_timing_enable(1 if on else 0))


def brl_timing_read(kernel_class: int):
    n, ms = C.c_longlong(0), C.c_double(0.0)
    _check(lib().brl_timing_read(kernel_class, C.byref(n), C.byref(ms)))
    return n.value, ms.value


def brl_timing_read_ops(kernel_class: int):
    n, ms, ops = C.c_longlong(0), C.c_double(0.0), C.c_double(0.0)
    _check(lib().brl_timing_read_ops(kernel_class, C.byref(n), C.byref(ms), C.byref(ops)))
    return n.value, ms.value, ops.value


# ------------------------------------------------ struct builders (marshalling)

def make_ffn_weights(norm_g, gate_packed, gate_beta, up_packed, up_beta, subln_g, down_packed, down_beta) -> brl_ffn_weights:
    return brl_ffn_weights(_ptr(norm_g), _ptr(gate_packed), _ptr(gate_beta), _ptr(up_packed), _ptr(up_beta),
                           _ptr(subln_g), _ptr(down_packed), _ptr(down_beta))


def make_mlp(weights: Sequence[torch.Tensor], biases: Sequence[torch.Tensor], act: int):
    """Returns (brl_mlp, keepalive): the ctypes arrays must outlive the struct."""
    n = len(weights)
    dims = (c_int * (n + 1))(*([weights[0].shape[1]] + [w.shape[0] for w in weights]))
    wp = (c_void_p * n)(*[_ptr(w) for w in weights])
    bp = (c_void_p * n)(*[_ptr(b) for b in biases])
    m = brl_mlp(n, C.cast(dims, C.POINTER(c_int)), C.cast(wp, C.POINTER(c_void_p)), C.cast(bp, C.POINTER(c_void_p)), act)
    return m, (dims, wp, bp, list(weights), list(biases))


def make_mlp_array(mlps: Sequence[brl_mlp]):
    """A contiguous ctypes array of brl_mlp structs (the member table of an ensemble)."""
    arr = (brl_mlp * len(mlps))(*mlps)
    return arr
