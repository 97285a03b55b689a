"""CPU oracle for the critic variants of BitRL's ablation: an int8-weight BitLinear for a
higher-precision critic backbone, and an ensemble of value heads that is averaged.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: only the
test-suite does.  It shares no code with the HIP path; it builds on the plain definitions
of `oracle.bitrl_oracle` (integer matmul, rescale, fully connected head).

What the paper fixes and what it leaves open
--------------------------------------------
Sec. 5.3 (component ablations, hybrid-precision rows) names an "INT8 critic + 1-bit
policy" configuration and "3x / 5x 1-bit critics (avg)" ensembles, and reports returns and
memory for them; it defines neither the int8 quantiser nor what the ensemble averages.
Readings taken here (also listed in the design document):

* int8 critic weights: symmetric per-tensor absmax quantisation, the weight-side mirror of
  the per-token activation quantiser: a' = max(max|W|, eps); s = 127 / a' (fp32 divide);
  code = clamp(round_half_even(W * s), -127, 127); dequantisation scale a' / 127.
  Activations, accumulation and the rescale are those of the ternary BitLinear
  (W8A8, int32 accumulation, y = (float(acc) * (a_t / 127)) * scale).  The table's
  "INT4 critic" is taken as the same quantiser on the grid -7..7 (qmax = 7).
* ensemble: n value heads of identical shape read the same h_t; each member's value is the
  fp32 head output, and the ensemble value is their arithmetic mean (summed in member order
  in fp64, divided by n, rounded to fp32 once).

Parity pins: tests/test_critic_oracle_pins.py (hand-worked cases under tests/golden,
exact integer special cases, error bounds, symmetries, brute force).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

from . import bitrl_oracle as O

F32 = np.float32
F64 = np.float64
QB = 127


def int8_quantize(W: np.ndarray, eps: float = 1e-5, qmax: int = QB) -> Tuple[np.ndarray, np.float32]:
    """Per-tensor absmax integer code of W[N, K] (Sec. 5.3, hybrid-precision critic; reading above).

    qmax = 127 is the int8 critic; qmax = 7 is the grid of the table's int4 critic (codes in
    [-7, 7], here still one code per int8 element: the definition does not depend on storage).
    Returns (codes int8 [N, K] in [-qmax, qmax], scale float32 = a' / qmax).
    """
    if not 1 <= int(qmax) <= QB:
        raise ValueError("qmax must be in 1..127")
    W = np.asarray(W, dtype=F32)
    if W.ndim != 2:
        raise ValueError("W must be [N, K]")
    a = np.max(np.abs(W)) if W.size else F32(0)
    if not np.isfinite(a):
        raise ValueError("non-finite weights")
    a_c = np.maximum(F32(a), F32(eps)).astype(F32)
    s = F32(F32(qmax) / a_c)
    t = (W * s).astype(F32)
    codes = np.clip(np.rint(t), -qmax, qmax).astype(np.int8)
    scale = F32(a_c / F32(qmax))
    return codes, scale


@dataclass
class Int8Linear:
    """A frozen int8-weight BitLinear: codes [N, K] and the dequantisation scale.

    Field names match `bitrl_oracle.TernaryLinear`, so the block and encoder definitions
    there apply unchanged (they only need an integer code matrix and one scale)."""
    codes: np.ndarray
    beta: np.float32

    @staticmethod
    def from_fp32(W: np.ndarray, eps: float = 1e-5, qmax: int = QB) -> "Int8Linear":
        c, s = int8_quantize(W, eps, qmax)
        return Int8Linear(c, s)


def int8_bitlinear_forward(x: np.ndarray, codes: np.ndarray, scale, eps: float = 1e-5,
                           residual: Optional[np.ndarray] = None, taps: Optional[dict] = None) -> np.ndarray:
    """W8A8 BitLinear: per-token int8 activations, int8 x int8 -> int32 exactly, fp32 rescale."""
    q, a_c = O.act_quant(x, eps)
    acc = O.ternary_matmul(q, codes)          # the exact integer contraction; nothing ternary about it
    if taps is not None:
        taps.update(xq=q, absmax=a_c, acc=acc)
    return O.dequant(acc, a_c, scale, residual)


def value_ensemble(h: np.ndarray, members: Sequence[O.MLP]) -> Tuple[np.ndarray, np.ndarray]:
    """Ensemble critic (Sec. 5.3, ensemble rows; reading above).

    Returns (mean [B] float32, each [n, B] float32)."""
    if len(members) == 0:
        raise ValueError("empty ensemble")
    each = []
    for m in members:
        v = O.mlp_forward(h, m)
        if v.shape[-1] != 1:
            raise ValueError("a value head has one output")
        each.append(v.reshape(v.shape[0]))
    each = np.stack(each).astype(F32)
    total = np.zeros(each.shape[1], dtype=F64)
    for v in each:                              # member order
        total = total + v.astype(F64)
    mean = (total / float(len(members))).astype(F32)
    return mean, each
