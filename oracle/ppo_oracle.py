"""Plain fp64 NumPy definition of the PPO update of the trainable heads on cached encoder outputs.

TEST INFRASTRUCTURE ONLY: nothing in the product path may import this file.  It shares no code
with the HIP path.  Every function cites the passage of the paper it follows; where the paper is
silent the reading taken is stated in the docstring (and listed in the design notes).

What the paper fixes (Sec. 3.1 Eq. 1, Sec. 3.2, Appendix hyper-parameter table): the frozen
backbone is evaluated once per rollout step and only the policy head g_phi and the value head
v_psi are trained, with PPO's clipped surrogate (epsilon = 0.1), an entropy bonus (coefficient
0.05), gradient clipping at max norm 0.5, learning rates 3e-4 (policy head) and 1e-3 (value head),
generalised advantage estimation (lambda = 0.95, gamma = 0.99), rollouts of 2048 steps,
mini-batches of 64 and 4 epochs per update.

Pinned by tests/test_ppo_oracle_pins.py: GAE against its closed forms (lambda = 0, lambda = 1,
constant rewards, episode boundaries), every gradient against central finite differences of the
scalar losses, Adam against its first-step / constant-gradient closed forms, the clipping rule
and the entropy of a uniform policy.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np


@dataclass
class PPOHyper:
    """Appendix hyper-parameter table; Adam's own constants and the advantage normalisation are readings."""
    clip_eps: float = 0.1
    ent_coef: float = 0.05
    max_grad_norm: float = 0.5
    lr_policy: float = 3e-4
    lr_value: float = 1e-3
    gamma: float = 0.99
    lam: float = 0.95
    adam_b1: float = 0.9
    adam_b2: float = 0.999
    adam_eps: float = 1e-8
    normalize_adv: bool = True
    adv_eps: float = 1e-8


@dataclass
class MLPParams:
    """out = W_L act(... act(W_1 x + b_1) ...) + b_L; W_l is [out_l, in_l]."""
    weights: List[np.ndarray]
    biases: List[np.ndarray]
    act: str = "tanh"

    def copy64(self) -> "MLPParams":
        return MLPParams([np.array(w, dtype=np.float64) for w in self.weights],
                         [np.array(b, dtype=np.float64) for b in self.biases], self.act)


def gae(rewards: np.ndarray, values: np.ndarray, dones: np.ndarray, last_value: float, gamma: float, lam: float
        ) -> Tuple[np.ndarray, np.ndarray]:
    """Generalised advantage estimate over one rollout (Sec. 3.2: lambda = 0.95, gamma = 0.99).

    delta_t = r_t + gamma * V_{t+1} * (1 - done_t) - V_t,  A_t = delta_t + gamma * lambda * (1 - done_t) * A_{t+1},
    with V_T = last_value and A_T = 0; done_t = 1 when the episode ended with step t.  Returns (A, A + V).
    """
    r = np.asarray(rewards, dtype=np.float64)
    v = np.asarray(values, dtype=np.float64)
    d = np.asarray(dones, dtype=np.float64)
    T = r.shape[0]
    adv = np.zeros(T, dtype=np.float64)
    nxt_adv, nxt_val = 0.0, float(last_value)
    for t in range(T - 1, -1, -1):
        live = 1.0 - d[t]
        delta = r[t] + gamma * nxt_val * live - v[t]
        nxt_adv = delta + gamma * lam * live * nxt_adv
        adv[t] = nxt_adv
        nxt_val = v[t]
    return adv, adv + v


def _act(z: np.ndarray, kind: str) -> np.ndarray:
    return np.tanh(z) if kind == "tanh" else np.maximum(z, 0.0)


def _act_grad_from_output(a: np.ndarray, kind: str) -> np.ndarray:
    return 1.0 - a * a if kind == "tanh" else (a > 0.0).astype(np.float64)


def mlp_forward_cache(x: np.ndarray, p: MLPParams) -> List[np.ndarray]:
    """Layer inputs [x, a_1, ..., a_{L-1}] and the output as the last entry (fp64)."""
    acts = [np.asarray(x, dtype=np.float64)]
    n = len(p.weights)
    for l in range(n):
        z = acts[-1] @ np.asarray(p.weights[l], dtype=np.float64).T + np.asarray(p.biases[l], dtype=np.float64)
        acts.append(z if l == n - 1 else _act(z, p.act))
    return acts


def mlp_backward(acts: List[np.ndarray], p: MLPParams, dout: np.ndarray) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """Gradients of a scalar with d(scalar)/d(output) = dout, w.r.t. every W_l and b_l."""
    n = len(p.weights)
    dWs: List[np.ndarray] = [None] * n
    dbs: List[np.ndarray] = [None] * n
    delta = np.asarray(dout, dtype=np.float64)
    for l in range(n - 1, -1, -1):
        dWs[l] = delta.T @ acts[l]
        dbs[l] = delta.sum(axis=0)
        if l > 0:
            delta = (delta @ np.asarray(p.weights[l], dtype=np.float64)) * _act_grad_from_output(acts[l], p.act)
    return dWs, dbs


def log_softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def normalize_advantages(adv: np.ndarray, eps: float) -> np.ndarray:
    """Reading (the paper is silent): per mini-batch, (A - mean) / (std + eps) with the unbiased (n - 1) standard deviation."""
    a = np.asarray(adv, dtype=np.float64)
    return (a - a.mean()) / (a.std(ddof=1) + eps)


def policy_loss(logits: np.ndarray, actions: np.ndarray, logp_old: np.ndarray, adv: np.ndarray, clip_eps: float,
                ent_coef: float) -> Dict[str, np.ndarray]:
    """Clipped surrogate (Eq. 1) plus entropy bonus: L = -mean_t min(r_t A_t, clip(r_t, 1-eps, 1+eps) A_t) - beta * mean_t H_t,
    r_t = pi(a_t|s_t) / pi_old(a_t|s_t), H_t = -sum_a pi(a|s_t) log pi(a|s_t).  Also d L / d logits."""
    logits = np.asarray(logits, dtype=np.float64)
    n = logits.shape[0]
    lsm = log_softmax(logits)
    pi = np.exp(lsm)
    idx = np.arange(n)
    logp = lsm[idx, actions]
    ratio = np.exp(logp - np.asarray(logp_old, dtype=np.float64))
    a = np.asarray(adv, dtype=np.float64)
    surr1 = ratio * a
    surr2 = np.clip(ratio, 1.0 - clip_eps, 1.0 + clip_eps) * a
    ent = -(pi * lsm).sum(axis=1)
    loss = -np.minimum(surr1, surr2).mean() - ent_coef * ent.mean()
    # the unclipped branch carries the gradient wherever it is the minimum (inside the clip range both agree)
    active = (surr1 <= surr2).astype(np.float64)
    onehot = np.zeros_like(logits)
    onehot[idx, actions] = 1.0
    dlogits = (-(active * a * ratio)[:, None] * (onehot - pi) + ent_coef * pi * (lsm + ent[:, None])) / n
    return {"loss": loss, "dlogits": dlogits, "logp": logp, "ratio": ratio, "entropy": ent,
            "clip_fraction": 1.0 - active.mean()}


def value_loss(v: np.ndarray, returns: np.ndarray) -> Dict[str, np.ndarray]:
    """Reading (the paper names a value head but no loss): L_V = 0.5 * mean_t (V(s_t) - R_t)^2."""
    v = np.asarray(v, dtype=np.float64).reshape(-1)
    r = np.asarray(returns, dtype=np.float64).reshape(-1)
    diff = v - r
    return {"loss": 0.5 * np.mean(diff * diff), "dv": (diff / v.shape[0])[:, None]}


def minibatch_grads(h: np.ndarray, actions: np.ndarray, logp_old: np.ndarray, adv: np.ndarray, returns: np.ndarray,
                    policy: MLPParams, value: MLPParams, hp: PPOHyper) -> Dict[str, object]:
    """Losses and parameter gradients of one mini-batch (before clipping)."""
    a = normalize_advantages(adv, hp.adv_eps) if hp.normalize_adv else np.asarray(adv, dtype=np.float64)
    pc = mlp_forward_cache(h, policy)
    pl = policy_loss(pc[-1], actions, logp_old, a, hp.clip_eps, hp.ent_coef)
    dWp, dbp = mlp_backward(pc, policy, pl["dlogits"])
    vc = mlp_forward_cache(h, value)
    vl = value_loss(vc[-1], returns)
    dWv, dbv = mlp_backward(vc, value, vl["dv"])
    return {"policy_loss": pl["loss"], "value_loss": vl["loss"], "entropy": pl["entropy"].mean(),
            "clip_fraction": pl["clip_fraction"], "dWp": dWp, "dbp": dbp, "dWv": dWv, "dbv": dbv, "adv_used": a}


def global_norm(grads: Sequence[np.ndarray]) -> float:
    return float(np.sqrt(sum(float((g.astype(np.float64) ** 2).sum()) for g in grads)))


def clip_scale(norm: float, max_norm: float) -> float:
    """Gradient clipping at max norm 0.5 (Sec. 3.2).  Reading: one global L2 norm over the gradients of both heads;
    every gradient is multiplied by min(1, max_norm / (norm + 1e-6))."""
    return min(1.0, max_norm / (norm + 1e-6))


@dataclass
class AdamState:
    m: List[np.ndarray]
    v: List[np.ndarray]
    t: int = 0


def adam_init(params: Sequence[np.ndarray]) -> AdamState:
    return AdamState([np.zeros_like(p, dtype=np.float64) for p in params], [np.zeros_like(p, dtype=np.float64) for p in params])


def adam_step(params: List[np.ndarray], grads: Sequence[np.ndarray], st: AdamState, lrs: Sequence[float], b1: float,
              b2: float, eps: float) -> None:
    """Reading (the paper gives learning rates, not the optimiser): Adam with bias correction,
    p -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps); lrs gives the rate of each tensor."""
    st.t += 1
    c1, c2 = 1.0 - b1 ** st.t, 1.0 - b2 ** st.t
    for i, (p, g) in enumerate(zip(params, grads)):
        st.m[i] = b1 * st.m[i] + (1.0 - b1) * g
        st.v[i] = b2 * st.v[i] + (1.0 - b2) * g * g
        p -= lrs[i] * (st.m[i] / c1) / (np.sqrt(st.v[i] / c2) + eps)


def flat_params(policy: MLPParams, value: MLPParams) -> List[np.ndarray]:
    """Order used for the optimiser state: policy W_1, b_1, ..., W_L, b_L, then the value head likewise."""
    out: List[np.ndarray] = []
    for p in (policy, value):
        for w, b in zip(p.weights, p.biases):
            out.append(w)
            out.append(b)
    return out


def ppo_update(h: np.ndarray, actions: np.ndarray, logp_old: np.ndarray, adv: np.ndarray, returns: np.ndarray,
               policy: MLPParams, value: MLPParams, perm: np.ndarray, batch: int, hp: PPOHyper,
               state: AdamState = None) -> Dict[str, object]:
    """One PPO update on a cached rollout (Sec. 3.2): for every epoch e, the rollout indices in the order perm[e]
    are cut into mini-batches of `batch`; each mini-batch gives one clipped Adam step on both heads.
    perm [epochs, T] holds the shuffles (random draws are inputs).  Parameters are updated in place (fp64 copies
    expected); returns the per-step statistics and the optimiser state."""
    params = flat_params(policy, value)
    n_pol = 2 * len(policy.weights)
    lrs = [hp.lr_policy] * n_pol + [hp.lr_value] * (len(params) - n_pol)
    st = adam_init(params) if state is None else state
    stats = []
    epochs, T = perm.shape
    for e in range(epochs):
        for s0 in range(0, T - batch + 1, batch):
            idx = perm[e, s0:s0 + batch]
            g = minibatch_grads(h[idx], actions[idx], logp_old[idx], adv[idx], returns[idx], policy, value, hp)
            grads: List[np.ndarray] = []
            for dW, db in zip(g["dWp"], g["dbp"]):
                grads += [dW, db]
            for dW, db in zip(g["dWv"], g["dbv"]):
                grads += [dW, db]
            norm = global_norm(grads)
            sc = clip_scale(norm, hp.max_grad_norm)
            adam_step(params, [gr * sc for gr in grads], st, lrs, hp.adam_b1, hp.adam_b2, hp.adam_eps)
            stats.append({"policy_loss": float(g["policy_loss"]), "value_loss": float(g["value_loss"]),
                          "entropy": float(g["entropy"]), "clip_fraction": float(g["clip_fraction"]), "grad_norm": norm})
    return {"stats": stats, "adam": st}
