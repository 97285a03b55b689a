"""Pins for the PPO head-update oracle: closed forms, finite differences and invariants - nothing
here calls the oracle to check the oracle (no GPU needed)."""
import math

import numpy as np
import pytest

from oracle import ppo_oracle as P


def _rng(seed):
    return np.random.Generator(np.random.Philox(key=seed))


# ------------------------------------------------------------------ GAE (Sec. 3.2)

def test_gae_lambda_zero_is_the_td_residual():
    g = _rng(1)
    T = 37
    r, v = g.normal(size=T), g.normal(size=T)
    last = 0.7
    adv, ret = P.gae(r, v, np.zeros(T), last, 0.99, 0.0)
    v_next = np.concatenate([v[1:], [last]])
    assert np.allclose(adv, r + 0.99 * v_next - v, rtol=0, atol=1e-14)
    assert np.allclose(ret, adv + v, rtol=0, atol=0)


def test_gae_lambda_one_is_discounted_return_minus_value():
    g = _rng(2)
    T, gamma, last = 23, 0.9, -1.3
    r, v = g.normal(size=T), g.normal(size=T)
    adv, _ = P.gae(r, v, np.zeros(T), last, gamma, 1.0)
    for t in range(T):
        disc = sum(gamma ** k * r[t + k] for k in range(T - t)) + gamma ** (T - t) * last
        assert abs(adv[t] - (disc - v[t])) < 1e-12


def test_gae_constant_reward_zero_values_is_a_geometric_sum():
    T, gamma, lam, c = 50, 0.99, 0.95, 2.5
    adv, ret = P.gae(np.full(T, c), np.zeros(T), np.zeros(T), 0.0, gamma, lam)
    x = gamma * lam
    for t in range(T):
        n = T - t
        assert abs(adv[t] - c * (1 - x ** n) / (1 - x)) < 1e-12
    assert np.array_equal(adv, ret)


def test_gae_episode_boundary_cuts_the_future():
    g = _rng(3)
    T = 30
    r, v = g.normal(size=T), g.normal(size=T)
    d = np.zeros(T)
    d[11] = 1.0
    a0, _ = P.gae(r, v, d, 0.4, 0.99, 0.95)
    r2, v2 = r.copy(), v.copy()
    r2[12:] += 5.0
    v2[12:] -= 3.0
    a1, _ = P.gae(r2, v2, d, 9.0, 0.99, 0.95)
    assert np.array_equal(a0[:12], a1[:12])            # steps of the finished episode do not see the next one
    assert abs(a0[11] - (r[11] - v[11])) < 1e-14       # terminal step: no bootstrap
    assert not np.allclose(a0[12:], a1[12:])


# ------------------------------------------------------------------ losses and their gradients (Eq. 1)

def _heads(g, d=12, hid=7, A=5, two_hidden=False):
    dims_p = [d, hid, 6, A] if two_hidden else [d, hid, A]
    dims_v = [d, hid, 6, 1] if two_hidden else [d, hid, 1]

    def mk(dims):
        return P.MLPParams([g.normal(size=(dims[i + 1], dims[i])) / math.sqrt(dims[i]) for i in range(len(dims) - 1)],
                           [0.1 * g.normal(size=dims[i + 1]) for i in range(len(dims) - 1)])
    return mk(dims_p), mk(dims_v)


def _batch(g, n=9, d=12, A=5):
    h = g.normal(size=(n, d))
    actions = g.integers(0, A, size=n)
    logp_old = np.log(np.full(n, 1.0 / A)) + 0.3 * g.normal(size=n)
    adv = g.normal(size=n)
    returns = g.normal(size=n)
    return h, actions, logp_old, adv, returns


def _scalar_losses(h, actions, logp_old, adv, returns, pol, val, hp):
    a = P.normalize_advantages(adv, hp.adv_eps) if hp.normalize_adv else adv
    logits = P.mlp_forward_cache(h, pol)[-1]
    lp = P.policy_loss(logits, actions, logp_old, a, hp.clip_eps, hp.ent_coef)["loss"]
    lv = P.value_loss(P.mlp_forward_cache(h, val)[-1], returns)["loss"]
    return lp, lv


@pytest.mark.parametrize("two_hidden,act", [(False, "tanh"), (True, "tanh"), (False, "relu")])
def test_gradients_match_central_finite_differences(two_hidden, act):
    g = _rng(4)
    pol, val = _heads(g, two_hidden=two_hidden)
    pol.act = val.act = act
    h, actions, logp_old, adv, returns = _batch(g)
    hp = P.PPOHyper(clip_eps=0.2)
    out = P.minibatch_grads(h, actions, logp_old, adv, returns, pol, val, hp)
    eps = 1e-6
    checked = 0
    for which, mlp, dWs, dbs in (("p", pol, out["dWp"], out["dbp"]), ("v", val, out["dWv"], out["dbv"])):
        for l in range(len(mlp.weights)):
            for arr, grad in ((mlp.weights[l], dWs[l]), (mlp.biases[l], dbs[l])):
                flat = arr.reshape(-1)
                for k in g.choice(flat.shape[0], size=min(6, flat.shape[0]), replace=False):
                    old = flat[k]
                    flat[k] = old + eps
                    up = _scalar_losses(h, actions, logp_old, adv, returns, pol, val, hp)
                    flat[k] = old - eps
                    dn = _scalar_losses(h, actions, logp_old, adv, returns, pol, val, hp)
                    flat[k] = old
                    num = ((up[0] - dn[0]) if which == "p" else (up[1] - dn[1])) / (2 * eps)
                    ana = grad.reshape(-1)[k]
                    assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (which, l, k, num, ana)
                    checked += 1
    assert checked >= 20


def test_surrogate_at_ratio_one_is_the_plain_policy_gradient():
    g = _rng(5)
    n, A = 6, 4
    logits = g.normal(size=(n, A))
    actions = g.integers(0, A, size=n)
    lsm = logits - np.log(np.exp(logits).sum(axis=1, keepdims=True))
    logp_old = lsm[np.arange(n), actions]              # pi == pi_old  =>  r == 1
    adv = g.normal(size=n)
    out = P.policy_loss(logits, actions, logp_old, adv, 0.1, 0.0)
    assert np.allclose(out["ratio"], 1.0)
    assert abs(out["loss"] + adv.mean()) < 1e-14       # L = -mean(A)
    onehot = np.eye(A)[actions]
    assert np.allclose(out["dlogits"], -(adv[:, None] * (onehot - np.exp(lsm))) / n, atol=1e-14)


def test_clipping_removes_the_gradient_of_samples_that_moved_too_far():
    A, eps = 3, 0.1
    logits = np.zeros((4, A))
    actions = np.array([0, 0, 1, 1])
    base = math.log(1.0 / A)
    # ratios 1.25, 0.8, 1.25, 0.8 with advantages +, +, -, -
    logp_old = np.array([base - math.log(1.25), base - math.log(0.8), base - math.log(1.25), base - math.log(0.8)])
    adv = np.array([1.0, 1.0, -1.0, -1.0])
    out = P.policy_loss(logits, actions, logp_old, adv, eps, 0.0)
    d = out["dlogits"]
    assert np.all(d[0] == 0.0)         # A > 0, r > 1 + eps: clipped
    assert np.any(d[1] != 0.0)         # A > 0, r < 1 - eps: the unclipped term is the minimum
    assert np.any(d[2] != 0.0)         # A < 0, r > 1 + eps: unclipped term is the minimum
    assert np.all(d[3] == 0.0)         # A < 0, r < 1 - eps: clipped
    assert out["clip_fraction"] == 0.5
    expect = -(min(1.25, 1.1) * 1 + min(0.8, 0.9) * 1 + min(-1.25, -1.1) + min(-0.8, -0.9)) / 4
    assert abs(out["loss"] - expect) < 1e-14


def test_entropy_of_uniform_policy():
    A = 18
    out = P.policy_loss(np.zeros((3, A)), np.array([0, 5, 17]), np.full(3, math.log(1 / A)), np.zeros(3), 0.1, 0.05)
    assert np.allclose(out["entropy"], math.log(A))
    assert abs(out["loss"] + 0.05 * math.log(A)) < 1e-14
    assert np.allclose(out["dlogits"], 0.0, atol=1e-17)         # the uniform policy maximises the entropy


def test_advantage_normalisation_and_value_loss_closed_forms():
    a = np.array([1.0, 2.0, 3.0, 6.0])
    n = P.normalize_advantages(a, 0.0)
    assert abs(n.mean()) < 1e-15 and abs(n.std(ddof=1) - 1.0) < 1e-15
    assert np.allclose(n, (a - 3.0) / math.sqrt(14.0 / 3.0))
    out = P.value_loss(np.array([[1.0], [3.0]]), np.array([0.0, 5.0]))
    assert out["loss"] == 0.5 * (1.0 + 4.0) / 2
    assert np.array_equal(out["dv"], np.array([[0.5], [-1.0]]))


# ------------------------------------------------------------------ clipping and Adam (Sec. 3.2)

def test_clip_scale_bounds_the_norm_and_keeps_the_direction():
    g = _rng(6)
    grads = [g.normal(size=(5, 3)), g.normal(size=4)]
    norm = P.global_norm(grads)
    assert abs(norm - math.sqrt(sum((x ** 2).sum() for x in grads))) < 1e-12
    sc = P.clip_scale(norm, 0.5)
    assert sc < 1.0 and P.global_norm([x * sc for x in grads]) <= 0.5
    assert abs(P.global_norm([x * sc for x in grads]) - 0.5) < 1e-5
    assert P.clip_scale(0.3, 0.5) == 1.0


def test_adam_first_step_and_constant_gradient():
    p = [np.array([1.0, -2.0, 3.0])]
    gvec = np.array([0.3, -4.0, 1e-3])
    st = P.adam_init(p)
    P.adam_step(p, [gvec], st, [1e-3], 0.9, 0.999, 1e-8)
    # after bias correction m_hat = g and v_hat = g^2: the step is lr * g / (|g| + eps)
    assert np.allclose(p[0], np.array([1.0, -2.0, 3.0]) - 1e-3 * gvec / (np.abs(gvec) + 1e-8), rtol=0, atol=1e-15)
    for _ in range(9):
        P.adam_step(p, [gvec], st, [1e-3], 0.9, 0.999, 1e-8)
    # a constant gradient keeps m_hat = g and v_hat = g^2 at every step
    assert np.allclose(p[0], np.array([1.0, -2.0, 3.0]) - 10 * 1e-3 * gvec / (np.abs(gvec) + 1e-8), rtol=0, atol=1e-12)
    assert st.t == 10


def test_update_uses_the_two_learning_rates_and_the_given_order():
    g = _rng(7)
    pol, val = _heads(g)
    pol, val = pol.copy64(), val.copy64()
    T, batch = 32, 8
    h, actions, logp_old, adv, returns = _batch(g, n=T)
    perm = np.stack([g.permutation(T) for _ in range(2)])
    before = [x.copy() for x in P.flat_params(pol, val)]
    hp = P.PPOHyper()
    out = P.ppo_update(h, actions, logp_old, adv, returns, pol, val, perm, batch, hp)
    assert len(out["stats"]) == 2 * (T // batch) and out["adam"].t == 8
    after = P.flat_params(pol, val)
    n_pol = 2 * len(pol.weights)
    # Adam moves every coordinate by at most about lr per step (|m_hat| / sqrt(v_hat) <= ~1 early on, 1 / sqrt(1 - b2) at worst)
    for i, (b, a) in enumerate(zip(before, after)):
        lr = hp.lr_policy if i < n_pol else hp.lr_value
        step = np.abs(a - b).max()
        assert 0 < step <= 8 * lr * 3.2, (i, step)
    # the first step alone: direction is minus the sign of the clipped gradient
    pol2, val2 = _heads(_rng(7))
    pol2, val2 = pol2.copy64(), val2.copy64()
    idx = perm[0, :batch]
    gr = P.minibatch_grads(h[idx], actions[idx], logp_old[idx], adv[idx], returns[idx], pol2, val2, hp)
    one = P.ppo_update(h, actions, logp_old, adv, returns, pol2, val2, perm[:1, :batch], batch, hp)
    assert len(one["stats"]) == 1
    w_before = before[0]
    moved = pol2.weights[0] - w_before
    big = np.abs(gr["dWp"][0]) > 1e-3
    assert np.array_equal(np.sign(moved[big]), -np.sign(gr["dWp"][0][big]))
    assert np.allclose(np.abs(moved[big]), hp.lr_policy, rtol=1e-3)
