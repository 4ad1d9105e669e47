"""GPU parity of gala_round: the whole round of Algorithm 1 in one call, with clipping, RMSprop
and the mixing step fused into one kernel.  Checked against the oracle (learner step, then
gossip) and against the library's own two-call sequence, which the other parity tests cover."""
import numpy as np
import pytest

import gala_synth as gs
from oracle import gala_oracle as orc
from parity_util import RTOL, compare_params, grad_scale, rel_err, relu_gates, upload

pytestmark = pytest.mark.gpu

HP = gs.HPARAMS


def _pair(N, A, T, B, topology, tau=0, seed=21, **kw):
    from paper_1906_04585_amd import Gala
    net = gs.make_net(A)
    a = Gala(N, A, T, B, HP, topology, max_delay=tau, delay_seed=seed, **kw)
    b = Gala(N, A, T, B, HP, topology, max_delay=tau, delay_seed=seed, **kw)
    X0 = gs.init_params(net, N, seed=seed, bias_scale=0.05)
    a.set_params(X0)
    b.set_params(X0)
    return net, a, b, X0


def _explicit_two_peer_tables(N, phases):
    """Every agent averages two in-peers per phase with unequal weights (row-stochastic)."""
    peers = np.zeros((phases, N, 2), dtype=np.int32)
    weights = np.zeros((phases, N, 3), dtype=np.float32)
    for p in range(phases):
        for i in range(N):
            peers[p, i] = [(i + 1 + p) % N, (i + N - 2 - p) % N]
            weights[p, i] = [0.5, 0.3, 0.2]
    peers[0, 1, 1] = -1                      # one unused slot: its weight goes back to the agent
    weights[0, 1] = [0.7, 0.3, 0.0]
    return peers, weights


def _explicit_one_peer_tables(N, phases, permutation):
    """One in-peer per agent and phase with unequal weights.  permutation: every agent is the
    in-peer of exactly one agent (a random permutation: cycles of different lengths);
    otherwise two agents listen to the same peer and one agent to nobody."""
    rng = np.random.default_rng(5 + N)
    peers = np.zeros((phases, N, 1), dtype=np.int32)
    weights = np.zeros((phases, N, 2), dtype=np.float32)
    for p in range(phases):
        perm = rng.permutation(N)
        peers[p, :, 0] = perm
        w_self = rng.uniform(0.2, 0.8, size=N).astype(np.float32)
        weights[p, :, 0] = w_self
        weights[p, :, 1] = np.float32(1.0) - w_self
    if not permutation:
        peers[0, 0, 0] = peers[0, 1, 0]
        peers[1, 2, 0] = -1
        weights[1, 2] = [1.0, 0.0]
    return peers, weights


@pytest.mark.parametrize("N,topology,tau", [(4, "exp", 0), (8, "exp", 2), (3, "ring", 1), (5, "explicit", 0),
                                            (6, "explicit", 2), (5, "ring", 0), (16, "exp", 0), (1, "ring", 0),
                                            (9, "one_peer_permutation", 0), (9, "one_peer_shared", 0),
                                            (6, "one_peer_permutation", 1)])
def test_round_equals_learner_step_then_gossip(N, topology, tau):
    """Same arithmetic in the same order: the fused call must give the parameters and the
    RMSprop state of the two-call sequence to the last bit, round after round.  One-peer
    topologies without delays whose peers form a permutation take the cycle-walking kernel
    (ring, exponential graph, explicit permutations); the others the general fused kernel."""
    kw = {}
    if topology == "explicit":
        kw["peers"], kw["weights"] = _explicit_two_peer_tables(N, 3)
    elif topology.startswith("one_peer"):
        kw["peers"], kw["weights"] = _explicit_one_peer_tables(N, 2, topology.endswith("permutation"))
        topology = "explicit"
    net, fused, split, X0 = _pair(N, 6, 2, 3, topology, tau, **kw)
    for r in range(5):
        dev = upload(gs.rollout(net, N, 2, 3, 900 + r))
        fused.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        split.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
        split.gossip(r)
        np.testing.assert_array_equal(fused.get_grads(), split.get_grads())
        np.testing.assert_array_equal(fused.get_step_stats(), split.get_step_stats())
        np.testing.assert_array_equal(fused.get_opt_state(), split.get_opt_state(), err_msg=f"round {r}")
        np.testing.assert_array_equal(fused.get_params(), split.get_params(), err_msg=f"round {r}")


@pytest.mark.parametrize("cfg_id,rounds", [(2, 3), (3, 5)])
def test_round_lockstep_against_oracle(cfg_id, rounds):
    """Configurations with 4 agents (no delay) and 8 agents (delays 0..2): the oracle is put
    in the GPU's pre-round state, runs learner step + gossip, and must agree on the gradients,
    the optimizer state and the post-round parameters.  Delayed messages come from the
    oracle's own history of earlier rounds, which matches the GPU's within the tolerance."""
    from paper_1906_04585_amd import Gala
    cfg = gs.CONFIGS[cfg_id]
    N, A, T, B, tau = cfg["n_agents"], cfg["n_actions"], cfg["T"], cfg["B"], cfg["max_delay"]
    net = gs.make_net(A)
    sl = gs.segment_slices(net)
    gpu = Gala(N, A, T, B, HP, cfg["topology"], max_delay=tau, delay_seed=31)
    om = orc.OracleGala(net, N, T, B, HP, cfg["topology"], max_delay=tau, delay_seed=31)
    X0 = gs.init_params(net, N, seed=77, bias_scale=0.05)
    gpu.set_params(X0)
    for r in range(rounds):
        X, V = gpu.get_params(), gpu.get_opt_state()
        om.set_params(X)
        om.set_opt_state(V)
        ro = gs.rollout(net, N, T, B, gs.round_seed(cfg_id, 50 + r))
        dev = upload(ro)
        gpu.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        gates, marked = relu_gates(gpu, net, X, ro)
        om.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"],
                        gates=gates if marked else None)
        g = gpu.get_grads()
        for i in range(N):
            for name, s in sl.items():
                assert rel_err(g[i, s], om.grads[i, s], grad_scale(om.grads[i], sl, name)) <= RTOL
        v = gpu.get_opt_state()
        for i in range(N):
            for name, s in sl.items():
                assert rel_err(v[i, s], om.V[i, s], grad_scale(om.V[i], sl, name)) <= 2 * RTOL
        om.gossip(r)
        compare_params(gpu, om, net, f"cfg{cfg_id} fused round {r}")


def test_round_full_size_32_agents():
    """The benchmark's launch shape (32 agents, 5 x 16, exponential graph): two rounds of the
    fused call against the two-call sequence bit for bit, and the mixing against the oracle
    from the broadcast parameters."""
    cfg = gs.CONFIGS[4]
    N, A, T, B = cfg["n_agents"], cfg["n_actions"], cfg["T"], cfg["B"]
    net, fused, split, X0 = _pair(N, A, T, B, cfg["topology"], cfg["max_delay"], seed=41)
    om = orc.OracleGala(net, N, T, B, HP, cfg["topology"], max_delay=cfg["max_delay"], delay_seed=41)
    for r in range(2):
        dev = upload(gs.rollout(net, N, T, B, gs.round_seed(4, 70 + r)))
        fused.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        split.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
        om.set_params(split.get_params())
        split.gossip(r)
        om.gossip(r)
        Z = fused.get_params()
        np.testing.assert_array_equal(Z, split.get_params())
        np.testing.assert_array_equal(fused.get_opt_state(), split.get_opt_state())
        assert np.abs(Z - om.X).max() <= 2.0 ** -22 * np.abs(om.X).max()


def test_round_rejects_what_gossip_rejects():
    from paper_1906_04585_amd import Gala
    from paper_1906_04585_amd.gala import GalaError
    net = gs.make_net(6)
    gpu = Gala(2, 6, 1, 2, HP, "ring", max_delay=1)
    gpu.set_params(gs.init_params(net, 2, seed=1))
    dev = upload(gs.rollout(net, 2, 1, 2, 5))
    with pytest.raises(GalaError):
        gpu.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], 3)   # not consecutive
    with pytest.raises(GalaError):
        gpu.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], -1)
    gpu.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], 0)


@pytest.mark.parametrize("N,tau", [(72, 1), (130, 1), (72, 0), (130, 0)])
def test_round_many_agents(N, tau):
    """With delays the general fused kernel runs, and above 64 agents its column block narrows
    (32, then 16 float4 columns) so that its LDS tile still fits; without delays the ring takes
    the cycle-walking kernel (one cycle of N agents).  Either way the result stays that of the
    two-call sequence."""
    net, fused, split, X0 = _pair(N, 6, 1, 2, "ring", tau, seed=5)
    for r in range(3):
        dev = upload(gs.rollout(net, N, 1, 2, 300 + r))
        fused.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        split.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
        split.gossip(r)
        np.testing.assert_array_equal(fused.get_opt_state(), split.get_opt_state())
        np.testing.assert_array_equal(fused.get_params(), split.get_params())


def test_single_stream_and_event_timing_give_the_same_bits(monkeypatch):
    """The weight gradients normally run on an internal second stream; GALA_SINGLE_STREAM=1 at
    creation and the per-kernel event timing both put everything on one stream.  Same kernels,
    same order of arithmetic: identical gradients, statistics, optimizer state and parameters."""
    from paper_1906_04585_amd import Gala
    N, A, T, B = 4, 6, 3, 4
    net = gs.make_net(A)
    X0 = gs.init_params(net, N, seed=33, bias_scale=0.05)
    two = Gala(N, A, T, B, HP, "exp")
    timed = Gala(N, A, T, B, HP, "exp")
    timed.set_profiling(True)
    monkeypatch.setenv("GALA_SINGLE_STREAM", "1")
    one = Gala(N, A, T, B, HP, "exp")
    monkeypatch.delenv("GALA_SINGLE_STREAM")
    for g in (two, timed, one):
        g.set_params(X0)
    for r in range(3):
        dev = upload(gs.rollout(net, N, T, B, 700 + r))
        for g in (two, timed, one):
            g.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        for other in (timed, one):
            np.testing.assert_array_equal(other.get_grads(), two.get_grads())
            np.testing.assert_array_equal(other.get_step_stats(), two.get_step_stats())
            np.testing.assert_array_equal(other.get_opt_state(), two.get_opt_state())
            np.testing.assert_array_equal(other.get_params(), two.get_params())
    assert set(timed.get_phase_times()) >= {"conv1_fwd", "loss_heads_dgrad", "clip_rmsprop_mix"}


@pytest.mark.parametrize("N,topology", [(4, "exp"), (5, "ring"), (32, "exp")])
def test_overlapped_optimizer_share_gives_the_same_bits(monkeypatch, N, topology):
    """GALA_OVERLAP_OPTIMIZER at creation: the hidden layer's share of the fused optimizer + mixing pass
    runs on the internal stream next to the following round's convolutions.  Same kernels on the same
    values: gradients, statistics, RMSprop state and parameters of every round are those of the plain
    context, also when other entry points (which must wait for the pending share) come in between."""
    from paper_1906_04585_amd import Gala
    A, T, B = 6, 2, 3
    net = gs.make_net(A)
    X0 = gs.init_params(net, N, seed=35, bias_scale=0.05)
    plain = Gala(N, A, T, B, HP, topology)
    monkeypatch.setenv("GALA_OVERLAP_OPTIMIZER", "1")
    over = Gala(N, A, T, B, HP, topology)
    monkeypatch.delenv("GALA_OVERLAP_OPTIMIZER")
    for g in (plain, over):
        g.set_params(X0)
    for r in range(6):
        dev = upload(gs.rollout(net, N, T, B, 500 + r))
        for g in (plain, over):
            g.round(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"], r)
        if r % 2 == 1:            # every other round is followed directly by the next round (late wait)
            np.testing.assert_array_equal(over.get_grads(), plain.get_grads())
            np.testing.assert_array_equal(over.get_step_stats(), plain.get_step_stats())
            np.testing.assert_array_equal(over.get_opt_state(), plain.get_opt_state(), err_msg=f"round {r}")
            np.testing.assert_array_equal(over.get_params(), plain.get_params(), err_msg=f"round {r}")
            assert over.consensus_distance() == plain.consensus_distance()
    # a split step and a gossip round after an overlapped round
    dev = upload(gs.rollout(net, N, T, B, 520))
    for g in (plain, over):
        g.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
        g.gossip(6)
    np.testing.assert_array_equal(over.get_params(), plain.get_params())
