"""Convenience holders around the C ABI: device buffers, packed weights, encoder tables.

Nothing here computes anything of the method: tensors are allocated with
torch, filled by the library's kernels, and handed back to the library.
"""
from __future__ import annotations

import ctypes as C
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from . import synth

DEV = "cuda"


def device_bytes(n: int) -> torch.Tensor:
    return torch.empty(max(int(n), 16), dtype=torch.uint8, device=DEV)


class Workspace:
    """A caller-owned scratch buffer (no state is kept in it between calls)."""

    def __init__(self, nbytes: int):
        self.buf = device_bytes(nbytes)

    def ensure(self, nbytes: int) -> "Workspace":
        if self.buf.numel() < nbytes:
            self.buf = device_bytes(nbytes)
        return self


@dataclass
class PackedLinear:
    packed: torch.Tensor        # uint8 [brl_packed_bytes]
    beta: torch.Tensor          # float32 [1]
    n_out: int
    k_in: int
    codes: Optional[torch.Tensor] = None   # int8 [n_out, k_in] debug tap


_qws: Optional[torch.Tensor] = None


def quantize_linear(W, eps: float = 1e-5, want_codes: bool = False, int8: bool = False, qmax: int = 127) -> PackedLinear:
    """fp32 master weights (numpy or torch, host or device) -> packed ternary (or int8) weights on the GPU."""
    global _qws
    if isinstance(W, np.ndarray):
        W = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32))
    Wd = W.to(DEV, dtype=torch.float32).contiguous()
    n, k = Wd.shape
    packed = device_bytes(B.brl_packed_int8_bytes(n, k) if int8 else B.brl_packed_bytes(n, k))
    beta = torch.empty(1, dtype=torch.float32, device=DEV)
    codes = torch.empty((n, k), dtype=torch.int8, device=DEV) if want_codes else None
    need = B.brl_quantize_workspace_bytes(n, k)
    if _qws is None or _qws.numel() < need:
        _qws = device_bytes(need)
    if int8:
        B.bitlinear_quantize_weights_int8(Wd, eps, qmax, packed, beta, codes, _qws)
    else:
        B.bitlinear_quantize_weights(Wd, eps, packed, beta, codes, _qws)
    return PackedLinear(packed, beta, n, k, codes)


def dev(a: np.ndarray, dtype=None) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV).contiguous()


def bf16_from_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the GPU (a reinterpretation, no rounding)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV)
    return t.view(torch.bfloat16).contiguous()


class FFNHandle:
    def __init__(self, norm_g, W_gate, W_up, subln_g, W_down, eps: float = 1e-5):
        self.d, self.f = W_down.shape[0], W_gate.shape[0]
        self.norm_g = dev(norm_g)
        self.subln_g = dev(subln_g)
        self.gate = quantize_linear(W_gate, eps)
        self.up = quantize_linear(W_up, eps)
        self.down = quantize_linear(W_down, eps)
        self.struct = B.make_ffn_weights(self.norm_g, self.gate.packed, self.gate.beta, self.up.packed, self.up.beta,
                                         self.subln_g, self.down.packed, self.down.beta)


class EncoderHandle:
    """Device-resident packed encoder: embedding, per-layer packed weights, the ABI structs.

    int8_weights: every BitLinear matrix as an int8 blob (the higher-precision critic backbone).
    int8_twin: additionally build `self.int8_twin`, the int8-weight encoder of the same master weights
    (shares the embedding and the gains; the masters are drawn once)."""

    def __init__(self, shape: synth.EncoderShape, seed: int = 0, eps_norm: float = 1e-5, eps_act: float = 1e-5,
                 layer_sink=None, n_layers: Optional[int] = None,
                 attn_precision: int = B.BRL_ATTN_MFMA, int8_weights: bool = False, int8_twin: bool = False):
        self.shape = shape
        L = shape.n_layers if n_layers is None else n_layers
        self.keep: List[object] = []
        self.embedding = torch.from_numpy(synth.embedding_bf16(seed, shape).view(np.int16)).to(DEV)
        self.final_norm_g = dev(synth.final_norm_gain(seed, shape))
        self.layer_structs = (B.brl_layer_weights * max(L, 1))()
        twin_structs = (B.brl_layer_weights * max(L, 1))() if int8_twin else None
        with ThreadPoolExecutor(max_workers=2) as ex:
            fut = ex.submit(synth.encoder_layer, seed, shape, 0) if L > 0 else None
            for l in range(L):
                w = fut.result()
                fut = ex.submit(synth.encoder_layer, seed, shape, l + 1) if l + 1 < L else None
                if layer_sink is not None:
                    layer_sink(l, w)
                t = {k: (dev(v) if v.ndim == 1 else quantize_linear(v, eps_act, int8=int8_weights)) for k, v in w.items()}
                self.keep.append(t)
                self._fill(self.layer_structs[l], t)
                if int8_twin:
                    t8 = {k: (t[k] if v.ndim == 1 else quantize_linear(v, eps_act, int8=True)) for k, v in w.items()}
                    self.keep.append(t8)
                    self._fill(twin_structs[l], t8)

        def make(structs, fmt):
            return B.brl_encoder(L, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f, shape.vocab,
                                 shape.rope_theta, eps_norm, eps_act, attn_precision, fmt,
                                 self.embedding.data_ptr(), self.final_norm_g.data_ptr(),
                                 C.cast(structs, C.POINTER(B.brl_layer_weights)))

        self.struct = make(self.layer_structs, B.BRL_W_INT8 if int8_weights else B.BRL_W_TERNARY)
        self.ws: Optional[Workspace] = None
        self.int8_twin: Optional["EncoderHandle"] = None
        if int8_twin:
            twin = object.__new__(EncoderHandle)
            twin.shape, twin.keep, twin.embedding, twin.final_norm_g = shape, self.keep, self.embedding, self.final_norm_g
            twin.layer_structs = twin_structs
            twin.struct = make(twin_structs, B.BRL_W_INT8)
            twin.ws = None
            twin.int8_twin = None
            self.int8_twin = twin

    @staticmethod
    def _fill(s, t) -> None:
        s.attn_norm_g = t["attn_norm_g"].data_ptr()
        s.wq_packed, s.wq_beta = t["Wq"].packed.data_ptr(), t["Wq"].beta.data_ptr()
        s.wk_packed, s.wk_beta = t["Wk"].packed.data_ptr(), t["Wk"].beta.data_ptr()
        s.wv_packed, s.wv_beta = t["Wv"].packed.data_ptr(), t["Wv"].beta.data_ptr()
        s.attn_subln_g = t["attn_subln_g"].data_ptr()
        s.wo_packed, s.wo_beta = t["Wo"].packed.data_ptr(), t["Wo"].beta.data_ptr()
        s.ffn = B.make_ffn_weights(t["ffn_norm_g"], t["W_gate"].packed, t["W_gate"].beta, t["W_up"].packed,
                                   t["W_up"].beta, t["ffn_subln_g"], t["W_down"].packed, t["W_down"].beta)

    def forward(self, ids: torch.Tensor, lengths: Optional[torch.Tensor] = None) -> torch.Tensor:
        b, s = ids.shape
        need = B.brl_encoder_workspace_bytes(self.struct, b, s)
        self.ws = Workspace(need) if self.ws is None else self.ws.ensure(need)
        h = torch.empty((b, self.shape.d), dtype=torch.float32, device=DEV)
        B.encoder_forward(self.struct, ids, b, s, lengths, h, self.ws.buf)
        return h


    def forward_packed(self, ids_flat: torch.Tensor, cu_seqlens_host: np.ndarray, max_len: Optional[int] = None) -> torch.Tensor:
        """States of different lengths stored back to back: ids_flat [T] int32 on the GPU, cu_seqlens_host [B+1]."""
        cu = np.ascontiguousarray(cu_seqlens_host, dtype=np.int32)
        b = cu.shape[0] - 1
        if max_len is None:
            max_len = int(np.max(np.diff(cu)))
        need = B.brl_encoder_packed_workspace_bytes(self.struct, b, int(cu[-1]), max_len)
        self.ws = Workspace(need) if self.ws is None else self.ws.ensure(need)
        h = torch.empty((b, self.shape.d), dtype=torch.float32, device=DEV)
        cu_dev = torch.from_numpy(cu).to(DEV)
        B.encoder_forward_packed(self.struct, ids_flat, cu_dev, cu, b, max_len, h, self.ws.buf)
        return h


class HeadHandle:
    def __init__(self, shape: synth.EncoderShape, seed: int = 0, act: int = B.BRL_ACT_TANH):
        pw, pb = synth.head_params(seed, shape, "policy")
        vw, vb = synth.head_params(seed, shape, "value")
        self.host = {"policy": (pw, pb), "value": (vw, vb)}
        self.pol, self._k1 = B.make_mlp([dev(w) for w in pw], [dev(b) for b in pb], act)
        self.val, self._k2 = B.make_mlp([dev(w) for w in vw], [dev(b) for b in vb], act)
        self.struct = B.brl_head(self.pol, self.val)
        self.n_actions = shape.n_actions
        self.ws: Optional[Workspace] = None

    def forward(self, h: torch.Tensor):
        b = h.shape[0]
        need = B.brl_head_workspace_bytes(self.struct, b)
        self.ws = Workspace(need) if self.ws is None else self.ws.ensure(need)
        logits = torch.empty((b, self.n_actions), dtype=torch.float32, device=DEV)
        value = torch.empty((b,), dtype=torch.float32, device=DEV)
        B.policy_value_head(self.struct, h, b, logits, value, self.ws.buf)
        return logits, value


class ValueEnsemble:
    """n value heads of one shape evaluated together and averaged."""

    def __init__(self, members_wb, act: int = B.BRL_ACT_TANH):
        self._keep = []
        mlps = []
        for ws, bs in members_wb:
            m, k = B.make_mlp([dev(w) for w in ws], [dev(b) for b in bs], act)
            mlps.append(m)
            self._keep.append(k)
        self.n = len(mlps)
        self.members = B.make_mlp_array(mlps)
        self.ws: Optional[Workspace] = None

    def forward(self, h: torch.Tensor, want_each: bool = True):
        b = h.shape[0]
        need = B.brl_value_ensemble_workspace_bytes(self.members, self.n, b)
        self.ws = Workspace(need) if self.ws is None else self.ws.ensure(need)
        mean = torch.empty((b,), dtype=torch.float32, device=DEV)
        each = torch.empty((self.n, b), dtype=torch.float32, device=DEV) if want_each else None
        B.value_ensemble_forward(self.members, self.n, h, b, mean, each, self.ws.buf)
        return mean, each


class PPOTrainer:
    """The two trainable heads in one flat parameter buffer, their Adam state, and the update entry points."""

    def __init__(self, policy_wb, value_wb, act: int = B.BRL_ACT_TANH, **hyper):
        pw, pb = policy_wb
        vw, vb = value_wb
        pdims = [pw[0].shape[1]] + [w.shape[0] for w in pw]
        vdims = [vw[0].shape[1]] + [w.shape[0] for w in vw]
        self.cfg, self._keep = B.make_ppo_config(pdims, vdims, act, **hyper)
        n = B.brl_ppo_param_count(self.cfg)
        w_off, b_off = B.brl_ppo_param_offsets(self.cfg)
        flat = np.zeros(n, dtype=np.float32)
        self.slices = []
        for k, (w, b) in enumerate(list(zip(pw, pb)) + list(zip(vw, vb))):
            flat[w_off[k]:w_off[k] + w.size] = np.asarray(w, dtype=np.float32).reshape(-1)
            flat[b_off[k]:b_off[k] + b.size] = np.asarray(b, dtype=np.float32).reshape(-1)
            self.slices.append((w_off[k], w.shape, b_off[k], b.shape))
        self.params = dev(flat)
        self.adam_m = torch.zeros_like(self.params)
        self.adam_v = torch.zeros_like(self.params)
        self.step = 0
        self.n_policy_layers = len(pw)
        # a forward head whose tensors are views into the flat buffer
        views = [(self.params[wo:wo + int(np.prod(ws))].view(*ws), self.params[bo:bo + int(np.prod(bs))].view(*bs))
                 for wo, ws, bo, bs in self.slices]
        pol, self._k1 = B.make_mlp([v[0] for v in views[:len(pw)]], [v[1] for v in views[:len(pw)]], act)
        val, self._k2 = B.make_mlp([v[0] for v in views[len(pw):]], [v[1] for v in views[len(pw):]], act)
        self.head = B.brl_head(pol, val)
        self.ws: Optional[Workspace] = None

    def tensors(self):
        """Host copies of the parameters: (policy weights, policy biases, value weights, value biases)."""
        flat = self.params.cpu().numpy()
        out = [(flat[wo:wo + int(np.prod(ws))].reshape(ws).copy(), flat[bo:bo + int(np.prod(bs))].reshape(bs).copy())
               for wo, ws, bo, bs in self.slices]
        n = self.n_policy_layers
        return [o[0] for o in out[:n]], [o[1] for o in out[:n]], [o[0] for o in out[n:]], [o[1] for o in out[n:]]

    def update(self, h, actions, logp_old, adv, returns, perm, batch: int, want_stats: bool = True):
        epochs, T = perm.shape
        need = B.brl_ppo_workspace_bytes(self.cfg, batch)
        self.ws = Workspace(need) if self.ws is None else self.ws.ensure(need)
        stats = torch.zeros((epochs * (T // batch), 5), dtype=torch.float32, device=DEV) if want_stats else None
        self.step = B.ppo_head_update(self.cfg, self.params, self.adam_m, self.adam_v, self.step, h, actions, logp_old, adv,
                                      returns, T, perm, epochs, batch, stats, self.ws.buf)
        return stats


def gae(rewards: torch.Tensor, values: torch.Tensor, dones: torch.Tensor, last_value: torch.Tensor, gamma: float, lam: float):
    n_envs, T = rewards.shape
    adv = torch.empty_like(rewards)
    ret = torch.empty_like(rewards)
    B.ppo_gae(rewards, values, dones, last_value, n_envs, T, gamma, lam, adv, ret)
    return adv, ret
