"""GPU-side behaviour of the boundary's error paths and options: call order, the opt-in action
validation, and the reversed exponential graph."""
import numpy as np
import pytest

import gala_synth as gs
from oracle import gala_oracle as orc
from parity_util import upload

pytestmark = pytest.mark.gpu

HP = gs.HPARAMS


def test_learner_step_before_set_params_is_a_state_error():
    from paper_1906_04585_amd import Gala
    from paper_1906_04585_amd.gala import GalaError
    net = gs.make_net(6)
    gpu = Gala(2, 6, 1, 2, HP, "ring")
    dev = upload(gs.rollout(net, 2, 1, 2, 5))
    import torch
    acts = torch.empty((2, 2), dtype=torch.int32, device="cuda")
    for call in (lambda: gpu.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"]),
                 lambda: gpu.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], 0),
                 lambda: gpu.a2c_allreduce_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"]),
                 lambda: gpu.act(dev["boot_obs"], 1, 0, acts)):
        with pytest.raises(GalaError) as ei:
            call()
        assert ei.value.code == -4 and "gala_set_params" in str(ei.value)
    gpu.set_params(gs.init_params(net, 2, seed=1))
    gpu.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])


def test_action_range_check_is_opt_in(monkeypatch):
    """With GALA_CHECK_ACTIONS set at creation a step whose action buffer holds a value outside
    [0, A) is refused with GALA_EINVAL before anything is computed; valid actions give the bits of
    an unchecked context."""
    from paper_1906_04585_amd import Gala
    from paper_1906_04585_amd.gala import GalaError
    N, A, T, B = 2, 6, 2, 3
    net = gs.make_net(A)
    X0 = gs.init_params(net, N, seed=12, bias_scale=0.05)
    ro = gs.rollout(net, N, T, B, 77)
    plain = Gala(N, A, T, B, HP, "ring")
    monkeypatch.setenv("GALA_CHECK_ACTIONS", "1")
    checked = Gala(N, A, T, B, HP, "ring")
    monkeypatch.delenv("GALA_CHECK_ACTIONS")
    for g in (plain, checked):
        g.set_params(X0)
    dev = upload(ro)
    for bad_value in (A, -1, 1 << 20):
        bad = ro["actions"].copy()
        bad[1, 1, 2] = bad_value
        dbad = upload(dict(ro, actions=bad))
        with pytest.raises(GalaError) as ei:
            checked.learner_step(dbad["obs"], dbad["actions"], dbad["rewards"], dbad["dones"], dbad["boot_obs"])
        assert ei.value.code == -1 and "outside [0, 6)" in str(ei.value)
        np.testing.assert_array_equal(checked.get_params(), X0)          # nothing was applied
    for g in (plain, checked):
        g.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], 0)
    np.testing.assert_array_equal(checked.get_params(), plain.get_params())


@pytest.mark.parametrize("N,tau", [(4, 0), (8, 0), (8, 2), (32, 0)])
def test_reverse_exponential_graph(N, tau):
    """Tables bit-exact against the oracle, mixing against the oracle, both mixing paths."""
    from paper_1906_04585_amd import Gala
    net = gs.make_net(6)
    gpu = Gala(N, 6, 1, 1, HP, "exp_reverse", max_delay=tau, delay_seed=19)
    fwd = Gala(N, 6, 1, 1, HP, "exp", max_delay=tau, delay_seed=19)
    om = orc.OracleGala(net, N, 1, 1, HP, "exp_reverse", max_delay=tau, delay_seed=19)
    X0 = gs.init_params(net, N, seed=8, bias_scale=0.1)
    gpu.set_params(X0)
    om.set_params(X0)
    m = N.bit_length() - 1
    for r in range(2 * m + 1):
        peer, delay = gpu.get_peer_table(r)
        opeer, odelay = orc.peer_table("exp_reverse", N, r, tau, 19)
        np.testing.assert_array_equal(peer[:, 0], opeer)
        np.testing.assert_array_equal(delay[:, 0], odelay)
        fpeer = fwd.get_peer_table(r)[0][:, 0]
        assert all(peer[fpeer[i], 0] == i for i in range(N))      # the inverse permutation of the forward graph
        gpu.gossip(r)
        om.gossip(r)
        x = gpu.get_params()
        assert np.abs(x - om.X).max() <= 2.0 ** -22 * np.abs(om.X).max(), f"round {r}"
    if tau == 0:     # log2 N rounds of either direction reach the exact average
        mean = X0.astype(np.float64).mean(0)
        assert np.abs(x - mean).max() <= 1e-6 * np.abs(mean).max() + 1e-9


def test_reverse_exponential_graph_fused_round_is_bit_identical():
    from paper_1906_04585_amd import Gala
    N, A, T, B = 8, 6, 2, 3
    net = gs.make_net(A)
    fused, split = Gala(N, A, T, B, HP, "exp_reverse"), Gala(N, A, T, B, HP, "exp_reverse")
    X0 = gs.init_params(net, N, seed=4, bias_scale=0.05)
    fused.set_params(X0)
    split.set_params(X0)
    for r in range(4):
        dev = upload(gs.rollout(net, N, T, B, 600 + r))
        fused.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        split.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
        split.gossip(r)
        np.testing.assert_array_equal(fused.get_params(), split.get_params())
