"""GPU parity: the HIP path through the C ABI against the CPU oracle on identical seeded
inputs.  Integer work (action gather, peer and delay tables) bit-exact; floating point
within the norm-wise tolerance of parity_util.RTOL per tensor."""
import numpy as np
import pytest

import gala_synth as gs
from oracle import gala_oracle as orc
from parity_util import RTOL, compare_learner_step, compare_params, rel_err, step_both, upload

pytestmark = pytest.mark.gpu

HP = gs.HPARAMS


def _make(cfg_id, shared=False, rounds_seed=None, **over):
    from paper_1906_04585_amd import Gala
    cfg = dict(gs.CONFIGS[cfg_id], **over)
    net = gs.make_net(cfg["n_actions"])
    N, T, B = cfg["n_agents"], cfg["T"], cfg["B"]
    seed = 7 + cfg_id
    gpu = Gala(N, cfg["n_actions"], T, B, HP, cfg["topology"], max_delay=cfg["max_delay"], delay_seed=seed)
    om = orc.OracleGala(net, N, T, B, HP, cfg["topology"], max_delay=cfg["max_delay"], delay_seed=seed)
    X0 = gs.init_params(net, N, seed=gs.BASE_SEED + cfg_id, shared=shared, bias_scale=0.05)
    gpu.set_params(X0)
    om.set_params(X0)
    return cfg, net, gpu, om, X0


def test_set_get_roundtrip_is_bit_exact():
    cfg, net, gpu, om, X0 = _make(1)
    np.testing.assert_array_equal(gpu.get_params(), X0)
    V0 = np.abs(gs.init_params(net, cfg["n_agents"], seed=3)) * 1e-3
    gpu.set_opt_state(V0)
    np.testing.assert_array_equal(gpu.get_opt_state(), V0)
    import torch
    xd = torch.from_numpy(X0[::-1].copy()).cuda()
    gpu.set_params(xd)
    out = torch.empty_like(xd)
    gpu.get_params(out)
    assert torch.equal(out, xd)


def test_config1_forward_outputs_and_returns():
    cfg, net, gpu, om, X0 = _make(1)
    N, T, B = cfg["n_agents"], cfg["T"], cfg["B"]
    ro = gs.rollout(net, N, T, B, gs.round_seed(1, 0))
    step_both(gpu, om, ro)
    out = gpu.get_outputs()
    for i in range(N):
        g, terms, ex = orc.agent_gradient(net, T, B, HP, X0[i], ro["obs"][i], ro["actions"][i],
                                          ro["rewards"][i], ro["dones"][i], ro["boot_obs"][i], extras=True)
        assert rel_err(out["logits"][i], ex["logits"]) <= RTOL
        assert rel_err(out["values"][i], ex["values"]) <= RTOL
        assert rel_err(out["returns"][i], ex["G"]) <= RTOL
        assert np.abs(out["advantages"][i] - ex["Adv"]).max() <= RTOL * np.abs(ex["G"]).max()


def test_config1_one_round_ring():
    cfg, net, gpu, om, X0 = _make(1)
    ro = gs.rollout(net, cfg["n_agents"], cfg["T"], cfg["B"], gs.round_seed(1, 0))
    step_both(gpu, om, ro)
    worst = compare_learner_step(gpu, om, net, "cfg1")        # no rollout passed: the plain tolerance
    print("worst per-tensor gradient errors:", {k: f"{v:.2e}" for k, v in worst.items()})
    gpu.gossip(0)
    om.gossip(0)
    x = compare_params(gpu, om, net, "cfg1 after gossip")
    # two agents on a ring: one round is the exact average, both rows identical bits
    np.testing.assert_array_equal(x[0], x[1])
    mx, fr = gpu.consensus_distance()
    assert mx == 0.0 and fr == 0.0


def test_action_gather_is_exact():
    """The integer gather of the taken action, checked on the head gradients the loss kernel writes
    (read back through gala_get_head_grads).  With the entropy term switched off a sample's row is
    A_m (pi - onehot(a_m)) / M: every entry has the sign of A_m except the taken action's, which has
    the opposite sign, so the one odd-signed lane *is* the gathered index -- compared exactly with
    the action fed in.  Changing one action must then change, bit for bit, nothing but that sample's
    two lanes (old and new action), and the oracle must agree on both action sets."""
    from paper_1906_04585_amd import Gala
    A = 6
    net = gs.make_net(A)
    N, T, B = 2, 5, 4
    M = T * B
    hp = dict(HP, ent_coef=0.0)
    X0 = gs.init_params(net, N, seed=99, bias_scale=0.05)
    ro = gs.rollout(net, N, T, B, 1234)
    rows = {}
    for flip in (False, True):
        r2 = dict(ro)
        if flip:
            a = ro["actions"].copy()
            a[1, 3, 2] = (a[1, 3, 2] + 1) % A
            r2["actions"] = a
        gpu = Gala(N, A, T, B, hp, "ring")
        om = orc.OracleGala(net, N, T, B, hp, "ring")
        gpu.set_params(X0)
        om.set_params(X0)
        step_both(gpu, om, r2)
        compare_learner_step(gpu, om, net, f"flip={flip}")
        dlogits, dvalues = gpu.get_head_grads()
        adv = gpu.get_outputs()["advantages"]
        assert np.all(adv != 0.0) and np.all(dlogits != 0.0)
        odd = np.sign(dlogits) != np.sign(adv)[:, :, None]          # [N][M][A]
        assert np.all(odd.sum(axis=2) == 1)                         # exactly one lane per sample ...
        np.testing.assert_array_equal(odd.argmax(axis=2), r2["actions"].reshape(N, M))   # ... the action taken
        rows[flip] = (dlogits, dvalues, r2["actions"].reshape(N, M))
    (d0, v0, a0), (d1, v1, a1) = rows[False], rows[True]
    np.testing.assert_array_equal(v0, v1)                           # the value gradient does not see the action
    changed = np.argwhere(d0 != d1)
    m = 3 * B + 2
    assert {tuple(c) for c in changed} == {(1, m, int(a0[1, m])), (1, m, int(a1[1, m]))}


@pytest.mark.parametrize("topology,N", [("ring", 2), ("ring", 4), ("exp", 4), ("exp", 8), ("exp", 32)])
def test_peer_tables_bit_exact(topology, N):
    from paper_1906_04585_amd import Gala
    gpu = Gala(N, 6, 1, 1, HP, topology, max_delay=2, delay_seed=4242)
    for r in range(12):
        peer, delay = gpu.get_peer_table(r)
        opeer, odelay = orc.peer_table(topology, N, r, 2, 4242)
        np.testing.assert_array_equal(peer[:, 0], opeer)
        np.testing.assert_array_equal(delay[:, 0], odelay)


@pytest.mark.parametrize("topology,N,tau", [("ring", 4, 0), ("exp", 8, 0), ("exp", 32, 0), ("exp", 8, 2), ("ring", 4, 1)])
def test_gossip_only_matches_oracle(topology, N, tau):
    from paper_1906_04585_amd import Gala
    net = gs.make_net(6)
    gpu = Gala(N, 6, 1, 1, HP, topology, max_delay=tau, delay_seed=11)
    om = orc.OracleGala(net, N, 1, 1, HP, topology, max_delay=tau, delay_seed=11)
    X0 = gs.init_params(net, N, seed=5, bias_scale=0.1)
    gpu.set_params(X0)
    om.set_params(X0)
    for r in range(7):
        if tau:   # perturb between rounds so that stale and fresh messages differ
            X = gpu.get_params()
            X = (X * (1.0 + 0.01 * (r + 1))).astype(np.float32)
            gpu.set_params(X)
            om.set_params(X)
        gpu.gossip(r)
        om.gossip(r)
        x = gpu.get_params()
        assert np.abs(x - om.X).max() <= 2.0 ** -22 * np.abs(om.X).max(), f"round {r}"
        mx, fr = gpu.consensus_distance()
        omx, ofr = om.consensus_distance()
        # fp32 mixing leaves rounding noise of a few ulp of the parameters themselves
        floor = 4e-7 * float(np.linalg.norm(om.X))
        assert abs(mx - omx) <= 1e-4 * omx + floor and abs(fr - ofr) <= 1e-4 * ofr + floor


def test_exponential_graph_exact_average_after_log2_rounds():
    from paper_1906_04585_amd import Gala
    N = 8
    gpu = Gala(N, 6, 1, 1, HP, "exp")
    X0 = gs.init_params(gs.make_net(6), N, seed=6, bias_scale=0.1)
    gpu.set_params(X0)
    for r in range(3):
        gpu.gossip(r)
    x = gpu.get_params()
    mean = X0.astype(np.float64).mean(0)
    assert np.abs(x - mean).max() <= 4e-7 * np.abs(mean).max() + 1e-9
    mx, _ = gpu.consensus_distance()
    assert mx <= 1e-4 * np.linalg.norm(mean)


def _all_agents_full_size(cfg_id, rounds):
    """A full-size configuration in the launch shape the benchmark times, every agent checked:
    each round the oracle restarts from the GPU's parameters and RMSprop state, both sides take one
    learner step (gradients, loss terms, norm, clip factor, post-update parameters and state of all
    agents compared) and one gossip round, and the distance from consensus is compared."""
    cfg, net, gpu, om, X0 = _make(cfg_id, shared=True)
    N, T, B = cfg["n_agents"], cfg["T"], cfg["B"]
    mx0, fr0 = gpu.consensus_distance()
    assert mx0 == 0.0 and fr0 == 0.0      # identical initialisation: exactly at consensus
    phases = set()
    for r in range(rounds):
        X = gpu.get_params()
        om.set_params(X)
        om.set_opt_state(gpu.get_opt_state())
        ro = gs.rollout(net, N, T, B, gs.round_seed(cfg_id, r))
        marked = step_both(gpu, om, ro)
        # every round is held to the plain tolerance: the conditioning factors are printed, not applied
        w = compare_learner_step(gpu, om, net, f"cfg{cfg_id} round {r}", ro=ro, X_before=X, plain=True)
        om.set_params(gpu.get_params())       # gossip for every agent, from the parameters the GPU broadcasts
        gpu.gossip(r)
        om.gossip(r)
        Z = gpu.get_params()
        assert np.abs(Z - om.X).max() <= 2.0 ** -22 * np.abs(om.X).max()
        phases.add(int(gpu.get_peer_table(r)[0][0, 0]))
        mx, fr = gpu.consensus_distance()     # distance from consensus, logged per round
        omx, ofr = orc.consensus_distance(Z)
        assert abs(mx - omx) <= 1e-4 * omx + 4e-7 * np.linalg.norm(Z)
        assert abs(fr - ofr) <= 1e-4 * ofr + 4e-7 * np.linalg.norm(Z)
        assert omx > 0.0                      # the agents saw different data: they have drifted apart
        print(f"cfg{cfg_id} round {r}: consensus max {mx:.4e} frob {fr:.4e}, {marked} ReLU units at rounding distance, "
              f"worst gradient error {max(v for k, v in w.items() if '.' in k):.2e}", flush=True)
    return phases


@pytest.mark.timeout(600)
def test_config4_full_size_all_agents_all_phases():
    """32 agents, 5 x 16 rollouts: all 32 agents, five rounds = all log2 32 phases of the exponential graph."""
    phases = _all_agents_full_size(4, rounds=5)
    assert phases == {1, 2, 4, 8, 16}         # agent 0's in-peer went through every hop length


@pytest.mark.timeout(600)
def test_config5_full_size_all_agents():
    """64 agents, 5 x 32 rollouts (fp32 path): all 64 agents, one round."""
    _all_agents_full_size(5, rounds=1)


# ---- bf16 matrix-instruction variant (fp32 parameters, activations and accumulation) -------------
# Tolerance 2e-2 relative on the loss terms, as the 64-agent configuration specifies.  The policy
# term is a mean of signed products and may cancel, so its error is measured against the
# magnitude it is made of (mean |log pi * A|), which is not smaller than |pg| itself.
BF16_RTOL = 2e-2


def _bf16_losses(cfg_id, agents, over=None):
    from paper_1906_04585_amd import Gala
    cfg = dict(gs.CONFIGS[cfg_id], **(over or {}))
    net = gs.make_net(cfg["n_actions"])
    N, T, B = cfg["n_agents"], cfg["T"], cfg["B"]
    gpu = Gala(N, cfg["n_actions"], T, B, dict(HP, compute_dtype=1), cfg["topology"])
    X0 = gs.init_params(net, N, seed=gs.BASE_SEED + 50 + cfg_id, bias_scale=0.05)
    gpu.set_params(X0)
    ro = gs.rollout(net, N, T, B, gs.round_seed(cfg_id, 0))
    dev = upload(ro)
    gpu.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
    st = gpu.get_step_stats()
    out = gpu.get_outputs()
    assert np.isfinite(gpu.get_params()).all()
    for i in agents:
        g, terms, ex = orc.agent_gradient(net, T, B, HP, X0[i], ro["obs"][i], ro["actions"][i], ro["rewards"][i],
                                          ro["dones"][i], ro["boot_obs"][i], extras=True)
        logp = ex["logits"] - np.log(np.exp(ex["logits"]).sum(1, keepdims=True))
        pg_scale = np.abs(logp[np.arange(T * B), ro["actions"][i].ravel()] * ex["Adv"]).mean()
        assert abs(st[i, 0] - terms[0]) <= BF16_RTOL * max(abs(terms[0]), pg_scale), (i, st[i, 0], terms[0])
        assert abs(st[i, 1] - terms[1]) <= BF16_RTOL * abs(terms[1]), (i, st[i, 1], terms[1])
        assert abs(st[i, 2] - terms[2]) <= BF16_RTOL * abs(terms[2]), (i, st[i, 2], terms[2])
        total_gpu = st[i, 0] + HP["vf_coef"] * st[i, 1] - HP["ent_coef"] * st[i, 2]
        total_ref = orc.total_loss(terms, HP)
        assert abs(total_gpu - total_ref) <= BF16_RTOL * max(abs(total_ref), pg_scale)
        assert rel_err(out["logits"][i], ex["logits"]) <= BF16_RTOL
        assert rel_err(out["values"][i], ex["values"]) <= BF16_RTOL
        # a different matrix path really ran: not bit-identical to what fp32 would give
        assert rel_err(out["values"][i], ex["values"]) > 1e-6


def test_bf16_variant_losses_small():
    _bf16_losses(2, range(4))


def test_config5_bf16_variant_losses_sampled():
    """64 agents, 5 x 32 rollouts, bf16 matrix instructions: loss terms of two sampled agents."""
    _bf16_losses(5, [11, 60])


# ---- ragged and degenerate shapes -------------------------------------------------------------------
@pytest.mark.parametrize("N,T,B,A,topology,tweak", [
    (1, 1, 1, 1, "ring", None),              # one agent, one sample, one action: every tile is an edge tile
    (3, 3, 5, 7, "ring", None),              # nothing a multiple of a tile: M = 15, F = 20, odd agent count
    (2, 2, 3, 64, "ring", None),             # the largest action set the loss kernel maps to lanes
    (2, 4, 2, 6, "exp", "all_done"),         # every transition terminal: returns are the rewards themselves
    (2, 4, 2, 6, "exp", "no_reward"),        # zero rewards and no terminals: returns are discounted bootstraps
    (5, 1, 7, 18, "ring", "same_action"),    # horizon 1, every sample takes the same action
])
def test_edge_shapes_one_round(N, T, B, A, topology, tweak):
    from paper_1906_04585_amd import Gala
    net = gs.make_net(A)
    gpu = Gala(N, A, T, B, HP, topology)
    om = orc.OracleGala(net, N, T, B, HP, topology)
    X0 = gs.init_params(net, N, seed=900 + N * 7 + T, bias_scale=0.05)
    gpu.set_params(X0)
    om.set_params(X0)
    ro = gs.rollout(net, N, T, B, 4000 + N + 10 * T + 100 * B)
    if tweak == "all_done":
        ro["dones"][:] = 1
    elif tweak == "no_reward":
        ro["rewards"][:] = 0.0
        ro["dones"][:] = 0
    elif tweak == "same_action":
        ro["actions"][:] = A - 1
    step_both(gpu, om, ro)
    compare_learner_step(gpu, om, net, f"edge {N},{T},{B},{A},{tweak}")   # the plain tolerance
    out = gpu.get_outputs()
    if tweak == "all_done":
        np.testing.assert_array_equal(out["returns"], ro["rewards"].reshape(N, T * B))
    if A == 1:                                # a single action: log pi = 0, entropy 0, no policy gradient
        st = gpu.get_step_stats()
        assert np.all(st[:, 0] == 0.0) and np.all(st[:, 2] == 0.0)
    gpu.gossip(0)
    om.gossip(0)
    compare_params(gpu, om, net, "edge after gossip")


def test_conv1_split_precision_is_fp32_level():
    """The first convolution multiplies byte images (exact in bf16) with fp32 operands cut into
    three bf16 pieces.  Its activations and its weight gradient must agree with the fp64 oracle as
    closely as single-precision accumulation allows (1e-5 of the largest entry), far below what one
    bf16 rounding (4e-3) would leave."""
    cfg, net, gpu, om, X0 = _make(2)
    N, T, B = cfg["n_agents"], cfg["T"], cfg["B"]
    ro = gs.rollout(net, N, T, B, gs.round_seed(2, 77))
    step_both(gpu, om, ro)
    a1 = gpu.get_activations(1).transpose(0, 1, 4, 2, 3).reshape(N, T * B + B, -1)
    off, shape = orc.act_offsets(net)["conv1"]
    n = int(np.prod(shape))
    sl = gs.segment_slices(net)
    g = gpu.get_grads()
    worst_a = worst_g = 0.0
    for i in range(N):
        obs = ro["obs"][i].reshape((T * B,) + ro["obs"].shape[3:])
        _, _, acts = orc.forward_acts(net, X0[i].astype(np.float64), obs)
        worst_a = max(worst_a, rel_err(a1[i, :T * B], acts[:, off:off + n]))
        worst_g = max(worst_g, rel_err(g[i, sl["conv1.w"]], om.grads[i, sl["conv1.w"]]))
    print(f"conv1 activation err {worst_a:.2e}, conv1.w gradient err {worst_g:.2e}")
    assert worst_a <= 1e-5 and worst_g <= 1e-5


def test_six_product_split_precision_is_fp32_level():
    """The second and third convolutions and the hidden layer (forward), and the data gradients of
    the hidden layer and the third convolution, multiply three bf16 pieces of both operands (six
    piece products).  Their activations and the gradients that flow through them must agree with
    the fp64 oracle as closely as single-precision accumulation allows (1e-5 of the largest
    entry), two orders below what one bf16 rounding of an operand (4e-3) would leave."""
    cfg, net, gpu, om, X0 = _make(2)
    N, T, B = cfg["n_agents"], cfg["T"], cfg["B"]
    ro = gs.rollout(net, N, T, B, gs.round_seed(2, 78))
    step_both(gpu, om, ro)
    offs = orc.act_offsets(net)
    sl = gs.segment_slices(net)
    g = gpu.get_grads()
    worst = {}
    for layer, key in ((2, "conv2"), (3, "conv3"), (4, "fc")):
        a = gpu.get_activations(layer)
        a = a.reshape(N, T * B + B, -1) if layer == 4 else a.transpose(0, 1, 4, 2, 3).reshape(N, T * B + B, -1)
        off, shape = offs[key]
        n = int(np.prod(shape))
        for i in range(N):
            obs = ro["obs"][i].reshape((T * B,) + ro["obs"].shape[3:])
            _, _, acts = orc.forward_acts(net, X0[i].astype(np.float64), obs)
            worst[key] = max(worst.get(key, 0.0), rel_err(a[i, :T * B], acts[:, off:off + n]))
    # weight gradients downstream of the split data-gradient kernels (fc dgrad feeds conv3.w, conv3 dgrad feeds conv2.w)
    for name in ("conv3.w", "conv2.w", "conv1.w"):
        for i in range(N):
            worst[name] = max(worst.get(name, 0.0), rel_err(g[i, sl[name]], om.grads[i, sl[name]]))
    print("six-product split errors:", {k: f"{v:.2e}" for k, v in worst.items()})
    assert max(worst.values()) <= 1e-5
