"""GPU parity of the PPO head update (through the C ABI) against the fp64 oracle.

Tolerances: the GPU keeps parameters and Adam state in fp32 (rounded after every step) and sums in fp64;
the oracle is fp64 throughout.  One step therefore agrees to about 1e-7 of a parameter's size; the bound
used on the parameter change after a whole update is 2e-4 of the largest change of that tensor."""
import numpy as np
import pytest

from oracle import ppo_oracle as P
from paper_2604_24273_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _mods():
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    B.lib()
    return B, R


def test_gae_matches_oracle():
    B, R = _mods()
    c = synth.ppo_rollout_case(3, 300, 8, 4, 0, n_envs=5)
    c["dones"][2, 299] = 1.0                      # an episode that ends with the rollout: no bootstrap
    adv, ret = R.gae(R.dev(c["rewards"]), R.dev(c["values"]), R.dev(c["dones"]), R.dev(c["last_value"]), 0.99, 0.95)
    for e in range(5):
        a_ref, r_ref = P.gae(c["rewards"][e], c["values"][e], c["dones"][e], c["last_value"][e], 0.99, 0.95)
        scale = np.abs(a_ref).max()
        assert np.abs(adv[e].cpu().numpy() - a_ref).max() <= 2e-7 * scale + 1e-7
        assert np.abs(ret[e].cpu().numpy() - r_ref).max() <= 2e-7 * np.abs(r_ref).max() + 1e-7


def _run_case(B, R, dims_p, dims_v, act, T, batch, epochs, seed, **hyper):
    d, A = dims_p[0], dims_p[-1]
    c = synth.ppo_rollout_case(seed, T, d, A, epochs)
    pw, pb = synth.mlp_params(seed, 60, dims_p)
    vw, vb = synth.mlp_params(seed, 80, dims_v)
    adv_ref, ret_ref = P.gae(c["rewards"][0], c["values"][0], c["dones"][0], c["last_value"][0], 0.99, 0.95)
    adv32, ret32 = adv_ref.astype(np.float32), ret_ref.astype(np.float32)
    tr = R.PPOTrainer((pw, pb), (vw, vb), act=B.BRL_ACT_TANH if act == "tanh" else B.BRL_ACT_RELU, **hyper)
    stats = tr.update(R.dev(c["h"]), R.dev(c["actions"]), R.dev(c["logp_old"]), R.dev(adv32), R.dev(ret32),
                      R.dev(c["perm"]), batch)
    hp = P.PPOHyper(**hyper)
    pol = P.MLPParams([w.astype(np.float64) for w in pw], [b.astype(np.float64) for b in pb], act)
    val = P.MLPParams([w.astype(np.float64) for w in vw], [b.astype(np.float64) for b in vb], act)
    out = P.ppo_update(c["h"].astype(np.float64), c["actions"], c["logp_old"].astype(np.float64), adv32.astype(np.float64),
                       ret32.astype(np.float64), pol, val, c["perm"], batch, hp)
    return tr, stats, pol, val, out, (pw, pb, vw, vb), c


@pytest.mark.parametrize("dims_p,dims_v,act,T,batch,epochs", [
    ([2560, 256, 18], [2560, 256, 1], "tanh", 256, 64, 2),       # the measured head shape
    ([96, 32, 16, 5], [96, 32, 16, 1], "relu", 200, 48, 3),      # two hidden layers, ragged rollout (8 steps dropped per epoch)
    ([64, 7], [64, 1], "tanh", 40, 40, 1),                        # single layer, one step
    ([96, 32, 16, 5], [96, 24, 1], "tanh", 128, 32, 2),           # heads of unequal depth: the deeper one's extra level runs alone
    ([64, 7], [64, 16, 8, 1], "relu", 96, 32, 2),
])
def test_head_update_matches_oracle(dims_p, dims_v, act, T, batch, epochs):
    B, R = _mods()
    tr, stats, pol, val, out, init, c = _run_case(B, R, dims_p, dims_v, act, T, batch, epochs, seed=11)
    n_steps = epochs * (T // batch)
    assert tr.step == n_steps == len(out["stats"])
    st = stats.cpu().numpy()
    ref = np.array([[s["policy_loss"], s["value_loss"], s["entropy"], s["clip_fraction"], s["grad_norm"]] for s in out["stats"]])
    # the first step starts from identical parameters: tight; later steps inherit the fp32 parameter rounding
    assert np.allclose(st[0], ref[0], rtol=2e-6, atol=1e-7), (st[0], ref[0])
    assert np.allclose(st[:, [0, 1, 2, 4]], ref[:, [0, 1, 2, 4]], rtol=2e-4, atol=1e-6)
    assert np.abs(st[:, 3] - ref[:, 3]).max() <= 1.0 / batch + 1e-6          # at most one sample on the clip boundary
    pw, pb, vw, vb = tr.tensors()
    got = list(pw) + list(pb) + list(vw) + list(vb)
    want = list(pol.weights) + list(pol.biases) + list(val.weights) + list(val.biases)
    start = list(init[0]) + list(init[1]) + list(init[2]) + list(init[3])
    for g, w, s0 in zip(got, want, start):
        change = np.abs(w - s0.astype(np.float64)).max()
        assert change > 0
        assert np.abs(g.astype(np.float64) - w).max() <= 2e-4 * change + 1e-7, (g.shape, np.abs(g - w).max(), change)
    # the forward entry point reads the same flat buffer: its outputs match the oracle's updated heads
    h_eval = R.dev(c["h"][:16])
    logits = torch.empty((16, dims_p[-1]), dtype=torch.float32, device="cuda")
    value = torch.empty((16,), dtype=torch.float32, device="cuda")
    ws = R.Workspace(B.brl_head_workspace_bytes(tr.head, 16))
    B.policy_value_head(tr.head, h_eval, 16, logits, value, ws.buf)
    l_ref = P.mlp_forward_cache(c["h"][:16], pol)[-1]
    v_ref = P.mlp_forward_cache(c["h"][:16], val)[-1][:, 0]
    assert np.abs(logits.cpu().numpy() - l_ref).max() <= 1e-4 * np.abs(l_ref).max()
    assert np.abs(value.cpu().numpy() - v_ref).max() <= 1e-4 * max(np.abs(v_ref).max(), 1.0)


def test_head_update_is_deterministic_and_resumable():
    B, R = _mods()
    dims_p, dims_v = [128, 32, 6], [128, 32, 1]
    c = synth.ppo_rollout_case(5, 128, 128, 6, 2)
    pw, pb = synth.mlp_params(5, 60, dims_p)
    vw, vb = synth.mlp_params(5, 80, dims_v)
    adv = R.dev(synth.normal(5, 90, (128,)))
    ret = R.dev(synth.normal(5, 91, (128,)))
    args = (R.dev(c["h"]), R.dev(c["actions"]), R.dev(c["logp_old"]), adv, ret)
    a = R.PPOTrainer((pw, pb), (vw, vb))
    a.update(*args, R.dev(c["perm"]), 32)
    b = R.PPOTrainer((pw, pb), (vw, vb))
    b.update(*args, R.dev(c["perm"][:1]), 32)           # the same update as two calls: the step counter carries over
    b.update(*args, R.dev(c["perm"][1:]), 32)
    assert a.step == b.step == 8
    assert torch.equal(a.params, b.params) and torch.equal(a.adam_m, b.adam_m) and torch.equal(a.adam_v, b.adam_v)
    before = a.params.clone()
    step = B.ppo_head_update(a.cfg, a.params, a.adam_m, a.adam_v, a.step, *args, 128, R.dev(c["perm"]), 0, 32, None,
                             a.ws.buf)                  # no epochs: nothing changes
    assert torch.equal(before, a.params) and step == 8


def test_no_normalisation_and_paper_hyperparameters_defaults():
    B, R = _mods()
    tr, stats, pol, val, out, init, c = _run_case(B, R, [64, 16, 3], [64, 16, 1], "tanh", 64, 16, 1, seed=13,
                                                  normalize_adv=False, clip_eps=0.2, ent_coef=0.0)
    ref = np.array([[s["policy_loss"], s["value_loss"], s["entropy"], s["clip_fraction"], s["grad_norm"]] for s in out["stats"]])
    assert np.allclose(stats.cpu().numpy()[:, [0, 1, 2, 4]], ref[:, [0, 1, 2, 4]], rtol=2e-4, atol=1e-6)
    cfg, _ = B.make_ppo_config([8, 4, 2], [8, 4, 1], B.BRL_ACT_TANH)
    assert abs(cfg.clip_eps - 0.1) < 1e-7 and abs(cfg.ent_coef - 0.05) < 1e-7 and abs(cfg.max_grad_norm - 0.5) < 1e-7
    assert abs(cfg.lr_policy - 3e-4) < 1e-7 and abs(cfg.lr_value - 1e-3) < 1e-7
