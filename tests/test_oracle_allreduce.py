"""Pins of the oracle's synchronous-A2C comparator (agents average their gradients before
every update; Sec. 5 "Experimental setup" and its footnote, Eq. (5)) against facts that do
not come from that function: the single agent with all simulators it must equal, PyTorch's
reverse-mode gradient of the batched loss, and the update written out in numpy."""
import numpy as np
import torch

import gala_synth as gs
from oracle import gala_oracle as orc
from test_oracle_learner import HP, MID, _torch_loss_and_grad


def _merge_agents(ro):
    """Rollouts of N agents with B simulators each -> one agent with N*B simulators
    (simulator i*B + b of the merged agent is simulator b of agent i)."""
    N, T, B = ro["actions"].shape

    def tb(a):                                  # [N, T, B, ...] -> [T, N*B, ...]
        return np.ascontiguousarray(np.moveaxis(a, 0, 1).reshape((T, N * B) + a.shape[3:]))
    return dict(obs=tb(ro["obs"]), actions=tb(ro["actions"]), rewards=tb(ro["rewards"]), dones=tb(ro["dones"]),
                boot_obs=np.ascontiguousarray(ro["boot_obs"].reshape((N * B,) + ro["boot_obs"].shape[2:])))


def test_allreduce_equals_one_agent_with_all_simulators():
    """n agents with b simulators each are one agent with n*b simulators (footnote in Sec. 5):
    the averaged gradient is the gradient of the batched loss Eq. (5), here taken both by the
    oracle's single-agent routine on the merged rollout and by autograd."""
    torch.set_num_threads(4)
    net, N, T, B = MID, 3, 3, 2
    hp = dict(HP, ent_coef=0.05)
    X = gs.init_params(net, N, seed=61, shared=True, bias_scale=0.1)
    ro = gs.rollout(net, N, T, B, 61)
    ro["dones"][1, 1, 0] = 1                    # an episode end inside one agent's rollout
    o = orc.OracleGala(net, N, T, B, hp, "ring")
    o.set_params(X)
    o.a2c_allreduce_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    merged = _merge_agents(ro)
    x = X[0].astype(np.float64)
    g1, terms1 = orc.agent_gradient(net, T, N * B, hp, x, merged["obs"], merged["actions"], merged["rewards"],
                                    merged["dones"], merged["boot_obs"])
    scale = np.abs(g1).max()
    assert np.abs(o.gbar - g1).max() <= 1e-12 * scale
    np.testing.assert_allclose(o.stats[:, :3].mean(0), terms1, rtol=1e-12)
    _, tg, _, _ = _torch_loss_and_grad(net, T, N * B, hp, x, merged)
    assert np.abs(o.gbar - tg).max() <= 1e-10 * scale
    # a sum instead of a mean, or one agent left out, would be off by far more than this
    assert np.abs(o.gbar * N - g1).max() > 0.5 * scale


def test_allreduce_update_is_clip_then_rmsprop_of_the_mean_and_keeps_replicas_identical():
    net, N, T, B = MID, 4, 2, 2
    hp = dict(HP, max_grad_norm=0.02)
    X = gs.init_params(net, N, seed=62, shared=True, bias_scale=0.1)
    ro = gs.rollout(net, N, T, B, 62)
    o = orc.OracleGala(net, N, T, B, hp, "ring")
    o.set_params(X)
    V0 = np.tile(np.abs(np.random.default_rng(1).normal(size=o.d)) * 1e-3, (N, 1))
    o.set_opt_state(V0)
    o.a2c_allreduce_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    own = [orc.agent_gradient(net, T, B, hp, X[i].astype(np.float64), ro["obs"][i], ro["actions"][i],
                              ro["rewards"][i], ro["dones"][i], ro["boot_obs"][i])[0] for i in range(N)]
    np.testing.assert_array_equal(o.grads, np.stack(own))
    gbar = np.mean(np.stack(own), axis=0)
    np.testing.assert_allclose(o.gbar, gbar, rtol=1e-13, atol=1e-18)
    n = np.linalg.norm(gbar)
    c = min(1.0, hp["max_grad_norm"] / (n + 1e-6))
    assert c < 1.0
    g = gbar * c
    v = hp["rms_alpha"] * V0[0] + (1 - hp["rms_alpha"]) * g * g
    x = X[0].astype(np.float64) - hp["lr"] * g / (np.sqrt(v) + hp["rms_eps"])
    for i in range(N):
        np.testing.assert_allclose(o.V[i], v, rtol=1e-13, atol=0)
        np.testing.assert_allclose(o.X[i], x, rtol=1e-13, atol=1e-16)
        np.testing.assert_array_equal(o.X[i], o.X[0])
        assert abs(o.stats[i, 3] - n) <= 1e-12 * n and abs(o.stats[i, 4] - c) <= 1e-13


def test_allreduce_uses_each_agents_own_parameters_and_state():
    """With different replicas the average is over gradients taken at each agent's own
    parameters, and each agent's own RMSprop state is updated."""
    net, N, T, B = MID, 2, 2, 2
    X = gs.init_params(net, N, seed=63, bias_scale=0.1)
    ro = gs.rollout(net, N, T, B, 63)
    o = orc.OracleGala(net, N, T, B, HP, "ring")
    o.set_params(X)
    V0 = np.abs(np.random.default_rng(2).normal(size=o.V.shape)) * 1e-3
    o.set_opt_state(V0)
    o.a2c_allreduce_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    own = [orc.agent_gradient(net, T, B, HP, X[i].astype(np.float64), ro["obs"][i], ro["actions"][i],
                              ro["rewards"][i], ro["dones"][i], ro["boot_obs"][i])[0] for i in range(N)]
    gbar = 0.5 * (own[0] + own[1])
    c = min(1.0, HP["max_grad_norm"] / (np.linalg.norm(gbar) + 1e-6))
    for i in range(N):
        v = HP["rms_alpha"] * V0[i] + (1 - HP["rms_alpha"]) * (c * gbar) ** 2
        np.testing.assert_allclose(o.V[i], v, rtol=1e-13, atol=0)
        np.testing.assert_allclose(o.X[i], X[i] - HP["lr"] * c * gbar / (np.sqrt(v) + HP["rms_eps"]), rtol=1e-13, atol=1e-16)


def test_allreduce_with_one_agent_is_the_learner_step():
    net, T, B = MID, 3, 2
    X = gs.init_params(net, 1, seed=64, bias_scale=0.1)
    ro = gs.rollout(net, 1, T, B, 64)
    a = orc.OracleGala(net, 1, T, B, HP, "ring")
    b = orc.OracleGala(net, 1, T, B, HP, "ring")
    a.set_params(X)
    b.set_params(X)
    a.a2c_allreduce_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    b.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    np.testing.assert_array_equal(a.X, b.X)
    np.testing.assert_array_equal(a.V, b.V)
    np.testing.assert_array_equal(a.stats, b.stats)
