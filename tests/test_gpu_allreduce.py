"""GPU parity of gala_a2c_allreduce_step (synchronous A2C with gradient averaging, the
method the paper compares GALA-A2C with) against the oracle, and against the single agent
with all simulators that it must equal for identical replicas."""
import numpy as np
import pytest

import gala_synth as gs
from oracle import gala_oracle as orc
from parity_util import RTOL, grad_scale, pg_scale, rel_err, relu_gates, upload

pytestmark = pytest.mark.gpu

HP = gs.HPARAMS


def _compare(gpu, om, net, tag, ro=None, X_before=None):
    sl = gs.segment_slices(net)
    g = gpu.get_grads()
    gbar = gpu.get_mean_grad()
    st = gpu.get_step_stats()
    x, v = gpu.get_params(), gpu.get_opt_state()
    for name, s in sl.items():
        assert rel_err(gbar[s], om.gbar[s], grad_scale(om.gbar, sl, name)) <= RTOL, f"{tag} mean grad {name}"
    for i in range(gpu.N):
        for name, s in sl.items():
            assert rel_err(g[i, s], om.grads[i, s], grad_scale(om.grads[i], sl, name)) <= RTOL, f"{tag} grad {name} agent {i}"
            assert rel_err(x[i, s], om.X[i, s]) <= RTOL, f"{tag} param {name} agent {i}"
            assert rel_err(v[i, s], om.V[i, s], grad_scale(om.V[i], sl, name)) <= 2 * RTOL, f"{tag} rmsprop {name} agent {i}"
        for k in range(5):
            ref = om.stats[i, k]
            scale = max(abs(ref), 1e-2 if k < 3 else 1e-30)
            if k == 0 and ro is not None:
                scale = max(scale, pg_scale(net, om.hp, X_before[i], ro, i))
            assert abs(st[i, k] - ref) <= RTOL * scale, f"{tag} stat {k} agent {i}"


def _both(gpu, om, net, ro):
    """Returns the pre-step parameters."""
    X = gpu.get_params()
    om.set_params(X)
    om.set_opt_state(gpu.get_opt_state())
    dev = upload(ro)
    gpu.a2c_allreduce_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
    gates, marked = relu_gates(gpu, net, X, ro)
    om.a2c_allreduce_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"],
                          gates=gates if marked else None)
    return X


@pytest.mark.parametrize("shared", [True, False])
def test_allreduce_lockstep_against_oracle(shared):
    """Four agents, 18 actions, 5 x 16 rollouts, three updates; with identical replicas and
    with replicas that differ (each gradient is taken at the agent's own parameters)."""
    from paper_1906_04585_amd import Gala
    cfg = gs.CONFIGS[2]
    N, A, T, B = cfg["n_agents"], cfg["n_actions"], cfg["T"], cfg["B"]
    net = gs.make_net(A)
    hp = dict(HP, max_grad_norm=0.5 if shared else 0.05)     # the second run clips
    gpu = Gala(N, A, T, B, hp, "ring")
    om = orc.OracleGala(net, N, T, B, hp, "ring")
    gpu.set_params(gs.init_params(net, N, seed=91, shared=shared, bias_scale=0.05))
    for r in range(3):
        ro = gs.rollout(net, N, T, B, gs.round_seed(2, 200 + r))
        X = _both(gpu, om, net, ro)
        _compare(gpu, om, net, f"shared={shared} update {r}", ro, X)
    if shared:
        x = gpu.get_params()
        for i in range(1, N):
            np.testing.assert_array_equal(x[i], x[0])        # replicas stay identical bit for bit
    else:
        assert gpu.get_step_stats()[0, 4] < 1.0


def test_allreduce_equals_one_agent_with_all_simulators():
    """n agents with b simulators each against one agent with n*b simulators on the merged
    rollout (footnote in Sec. 5), both on the GPU."""
    from paper_1906_04585_amd import Gala
    N, A, T, B = 4, 6, 5, 4
    net = gs.make_net(A)
    sl = gs.segment_slices(net)
    X0 = gs.init_params(net, N, seed=92, shared=True, bias_scale=0.05)
    ro = gs.rollout(net, N, T, B, 4321)
    many = Gala(N, A, T, B, HP, "ring")
    one = Gala(1, A, T, N * B, HP, "ring")
    many.set_params(X0)
    one.set_params(X0[:1])
    dev = upload(ro)
    many.a2c_allreduce_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])

    def tb(a):                                               # [N, T, B, ...] -> [1, T, N*B, ...]
        return np.ascontiguousarray(np.moveaxis(a, 0, 1).reshape((1, T, N * B) + a.shape[3:]))
    merged = dict(obs=tb(ro["obs"]), actions=tb(ro["actions"]), rewards=tb(ro["rewards"]), dones=tb(ro["dones"]),
                  boot_obs=np.ascontiguousarray(ro["boot_obs"].reshape((1, N * B) + ro["boot_obs"].shape[2:])))
    dm = upload(merged)
    one.learner_step(dm["obs"], dm["actions"], dm["rewards"], dm["dones"], dm["boot_obs"])
    gbar, g1 = many.get_mean_grad(), one.get_grads()[0]
    x, x1 = many.get_params(), one.get_params()[0]
    for name, s in sl.items():
        assert rel_err(gbar[s], g1[s], grad_scale(g1.astype(np.float64), sl, name)) <= RTOL, name
        for i in range(N):
            assert rel_err(x[i, s], x1[s]) <= RTOL, name
    assert abs(many.get_step_stats()[0, 3] - one.get_step_stats()[0, 3]) <= RTOL * one.get_step_stats()[0, 3]


def test_allreduce_full_size_32_agents():
    """The 32-agent, 5 x 16 shape the benchmark times: one update, every agent's gradient
    from the oracle."""
    from paper_1906_04585_amd import Gala
    cfg = gs.CONFIGS[4]
    N, A, T, B = cfg["n_agents"], cfg["n_actions"], cfg["T"], cfg["B"]
    net = gs.make_net(A)
    gpu = Gala(N, A, T, B, HP, cfg["topology"])
    om = orc.OracleGala(net, N, T, B, HP, cfg["topology"])
    gpu.set_params(gs.init_params(net, N, seed=93, shared=True, bias_scale=0.05))
    ro = gs.rollout(net, N, T, B, gs.round_seed(4, 300))
    X = _both(gpu, om, net, ro)
    _compare(gpu, om, net, "32 agents", ro, X)
