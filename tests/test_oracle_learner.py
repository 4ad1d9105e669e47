"""Pins of the CPU oracle's learner step against things fixed by the paper and
by mathematics, none of which come from the oracle itself: hand-worked returns,
closed forms, finite differences, and PyTorch's double-precision convolution
with reverse-mode differentiation as an independent library routine."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import gala_synth as gs
from oracle import gala_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))
HP = gs.HPARAMS

TINY = dict(in_c=1, in_h=12, in_w=12, conv=[(2, 4, 2), (3, 2, 1), (3, 2, 1)], fc=8, n_actions=3)
MID = dict(in_c=2, in_h=28, in_w=28, conv=[(4, 8, 4), (5, 4, 2), (6, 2, 1)], fc=16, n_actions=4)


# ---- n-step returns (Sec. 2; Algorithm 1, "Compute returns") ------------------

def _golden_cases():
    cases = {}
    with open(os.path.join(HERE, "golden", "nstep_returns.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, t, r, dn, G, A = line.split()
            cases.setdefault(name, []).append((int(t), float(r), int(dn), float(G), float(A)))
    return cases


@pytest.mark.parametrize("name", ["no_done", "done_at_1"])
def test_returns_hand_worked(name):
    rows = sorted(_golden_cases()[name])
    r = np.array([[x[1]] for x in rows])
    dn = np.array([[x[2]] for x in rows], dtype=np.uint8)
    G, A = orc.nstep_returns(r, dn, np.array([2.0]), np.full((3, 1), 0.5), 0.99)
    np.testing.assert_allclose(G[:, 0], [x[3] for x in rows], rtol=0, atol=1e-12)
    np.testing.assert_allclose(A[:, 0], [x[4] for x in rows], rtol=0, atol=1e-12)


def test_returns_closed_form_brute_force():
    rng = np.random.default_rng(5)
    T, B, gamma = 5, 7, 0.99
    r = rng.normal(size=(T, B))
    vb = rng.normal(size=B)
    v = rng.normal(size=(T, B))
    G, A = orc.nstep_returns(r, np.zeros((T, B), np.uint8), vb, v, gamma)
    for b in range(B):
        for t in range(T):
            n = T - t
            want = sum(gamma ** i * r[t + i, b] for i in range(n)) + gamma ** n * vb[b]
            assert abs(G[t, b] - want) < 1e-12
            assert abs(A[t, b] - (want - v[t, b])) < 1e-12


def test_returns_done_cuts_everything_after():
    rng = np.random.default_rng(6)
    T, B, gamma = 5, 4, 0.9
    r = rng.normal(size=(T, B))
    dn = np.zeros((T, B), np.uint8)
    dn[2, 1] = 1
    dn[4, 3] = 1
    vb = rng.normal(size=B)
    G, _ = orc.nstep_returns(r, dn, vb, np.zeros((T, B)), gamma)
    # env 1: samples 0..2 see rewards up to t=2 only
    for t in range(3):
        want = sum(gamma ** i * r[t + i, 1] for i in range(3 - t))
        assert abs(G[t, 1] - want) < 1e-12
    # env 1 after the cut is a fresh episode that still bootstraps
    assert abs(G[3, 1] - (r[3, 1] + gamma * r[4, 1] + gamma ** 2 * vb[1])) < 1e-12
    # env 3: terminal at the last step removes the bootstrap value altogether
    assert abs(G[4, 3] - r[4, 3]) < 1e-12


# ---- loss closed forms (Eq. (1), Eq. (4)) ---------------------------------------

@pytest.mark.parametrize("A", [6, 18])
def test_loss_uniform_logits(A):
    M = 5
    rng = np.random.default_rng(1)
    logits = np.full((M, A), 0.37)
    values = rng.normal(size=M)
    G = rng.normal(size=M)
    Adv = rng.normal(size=M)
    actions = rng.integers(0, A, size=M)
    terms, dlogits, dvalues = orc.a2c_loss(logits, values, actions, G, Adv, 0.5, 0.01)
    assert abs(terms[2] - np.log(A)) < 1e-12                     # entropy of the uniform policy
    assert abs(terms[0] - np.mean(np.log(A) * Adv)) < 1e-12      # -log(1/A) * A_t
    assert abs(terms[1] - np.mean((G - values) ** 2)) < 1e-12
    # the entropy is stationary at the uniform policy: only the pg part remains
    want = Adv[:, None] * (1.0 / A - np.eye(A)[actions]) / M
    np.testing.assert_allclose(dlogits, want, atol=1e-14)
    np.testing.assert_allclose(dvalues, -2 * 0.5 * (G - values) / M, atol=1e-14)


def test_loss_zero_advantage_zero_entropy_coef_has_no_policy_gradient():
    rng = np.random.default_rng(2)
    M, A = 4, 6
    logits = rng.normal(size=(M, A))
    _, dlogits, _ = orc.a2c_loss(logits, np.zeros(M), rng.integers(0, A, M), np.zeros(M), np.zeros(M), 0.5, 0.0)
    assert np.all(dlogits == 0.0)


def test_loss_near_deterministic_policy_has_vanishing_entropy():
    logits = np.array([[60.0, 0.0, 0.0, 0.0]])
    terms, _, _ = orc.a2c_loss(logits, np.zeros(1), np.array([0]), np.zeros(1), np.ones(1), 0.5, 0.01)
    assert 0.0 <= terms[2] < 1e-20
    assert abs(terms[0]) < 1e-15      # log pi(a) ~ 0 for the certain action


def test_loss_head_gradients_by_finite_differences():
    rng = np.random.default_rng(3)
    M, A = 6, 5
    logits = rng.normal(size=(M, A))
    values = rng.normal(size=M)
    G = rng.normal(size=M)
    Adv = rng.normal(size=M)
    actions = rng.integers(0, A, size=M)
    cv, eta = 0.5, 0.3

    def L(lg, v):
        t, _, _ = orc.a2c_loss(lg, v, actions, G, Adv, cv, eta)
        return t[0] + cv * t[1] - eta * t[2]

    _, dlogits, dvalues = orc.a2c_loss(logits, values, actions, G, Adv, cv, eta)
    h = 1e-6
    for m in range(M):
        for a in range(A):
            lp, lm = logits.copy(), logits.copy()
            lp[m, a] += h
            lm[m, a] -= h
            fd = (L(lp, values) - L(lm, values)) / (2 * h)
            assert abs(fd - dlogits[m, a]) < 1e-8
        vp, vm = values.copy(), values.copy()
        vp[m] += h
        vm[m] -= h
        fd = (L(logits, vp) - L(logits, vm)) / (2 * h)
        assert abs(fd - dvalues[m]) < 1e-8


def test_entropy_enters_as_a_bonus():
    # Raising the entropy coefficient must push logits towards uniform: the
    # entropy part of dL/dz has the sign of p (log p + H), i.e. it lowers the loss
    # to move probability from likely to unlikely actions.
    logits = np.array([[2.0, 0.0, 0.0]])
    _, d0, _ = orc.a2c_loss(logits, np.zeros(1), np.array([1]), np.zeros(1), np.zeros(1), 0.5, 0.0)
    _, d1, _ = orc.a2c_loss(logits, np.zeros(1), np.array([1]), np.zeros(1), np.zeros(1), 0.5, 1.0)
    assert np.all(d0 == 0)
    assert d1[0, 0] > 0 and d1[0, 1] < 0 and d1[0, 2] < 0     # gradient descent lowers z_0


# ---- network: special cases and an independent library routine -------------------

def _tiny_problem(net, T, B, seed, bias_scale=0.1):
    x = gs.init_params(net, 1, seed=seed, bias_scale=bias_scale)[0].astype(np.float64)
    ro = gs.rollout(net, 1, T, B, seed)
    return x, {k: v[0] for k, v in ro.items()}


def test_conv_with_full_size_kernel_is_a_dot_product():
    # one conv layer whose kernel covers the whole input -> 1x1 output -> plain dot product
    net = dict(in_c=2, in_h=5, in_w=5, conv=[(3, 5, 1)], fc=4, n_actions=2)
    x = gs.init_params(net, 1, seed=11, bias_scale=0.2)[0].astype(np.float64)
    obs = gs.rollout(net, 1, 1, 3, 11)["obs"][0, 0]
    _, _, acts = orc.forward_acts(net, x, obs)
    sl = gs.segment_slices(net)
    w = x[sl["conv1.w"]].reshape(3, 50)
    b = x[sl["conv1.b"]]
    s = obs.reshape(3, 50).astype(np.float64) / 255.0
    want = np.maximum(s @ w.T + b, 0.0)
    np.testing.assert_allclose(acts[:, 50:53], want, atol=1e-13)
    # and the dense layers on top of it
    h = np.maximum(want @ x[sl["fc.w"]].reshape(4, 3).T + x[sl["fc.b"]], 0.0)
    logits, values = orc.forward(net, x, obs)
    np.testing.assert_allclose(logits, h @ x[sl["pi.w"]].reshape(2, 4).T + x[sl["pi.b"]], atol=1e-13)
    np.testing.assert_allclose(values, h @ x[sl["v.w"]] + x[sl["v.b"]], atol=1e-13)


def _torch_loss_and_grad(net, T, B, hp, x, ro):
    """The same loss written with PyTorch double ops and differentiated by autograd."""
    sl = gs.segment_slices(net)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    shapes = {name: shape for name, shape, _ in gs.param_segments(net)}
    P = {k: xt[sl[k]].reshape(shapes[k]) for k in sl}

    def fwd(obs_u8):
        a = torch.tensor(obs_u8.astype(np.float64) / 255.0)
        for li, (o, k, s) in enumerate(net["conv"], start=1):
            a = F.relu(F.conv2d(a, P[f"conv{li}.w"], P[f"conv{li}.b"], stride=s))
        hdn = F.relu(F.linear(a.flatten(1), P["fc.w"], P["fc.b"]))
        return F.linear(hdn, P["pi.w"], P["pi.b"]), F.linear(hdn, P["v.w"], P["v.b"])[:, 0]

    M = T * B
    logits, values = fwd(ro["obs"].reshape((M,) + ro["obs"].shape[2:]))
    _, vboot = fwd(ro["boot_obs"])
    G = torch.zeros(T, B, dtype=torch.float64)
    nxt = vboot.detach()
    r = torch.tensor(ro["rewards"].astype(np.float64))
    dn = torch.tensor(ro["dones"].astype(np.float64))
    for t in reversed(range(T)):
        nxt = r[t] + hp["gamma"] * (1 - dn[t]) * nxt
        G[t] = nxt
    G = G.reshape(M)
    adv = (G - values).detach()
    logp = torch.log_softmax(logits, dim=1)
    act = torch.tensor(ro["actions"].reshape(M).astype(np.int64))
    pg = -(logp[torch.arange(M), act] * adv).mean()
    td = ((G - values) ** 2).mean()
    ent = -(logp.exp() * logp).sum(1).mean()
    loss = pg + hp["vf_coef"] * td - hp["ent_coef"] * ent
    loss.backward()
    return np.array([pg.item(), td.item(), ent.item()]), xt.grad.numpy().copy(), logits.detach().numpy(), values.detach().numpy()


@pytest.mark.parametrize("net,T,B", [(MID, 3, 2), (gs.make_net(6), 2, 2)])
def test_gradient_matches_autograd_double(net, T, B):
    torch.set_num_threads(4)
    x, ro = _tiny_problem(net, T, B, seed=21)
    hp = dict(HP, ent_coef=0.05)
    g, terms, ex = orc.agent_gradient(net, T, B, hp, x, ro["obs"], ro["actions"],
                                      ro["rewards"], ro["dones"], ro["boot_obs"], extras=True)
    tterms, tg, tlogits, tvalues = _torch_loss_and_grad(net, T, B, hp, x, ro)
    np.testing.assert_allclose(ex["logits"], tlogits, rtol=0, atol=1e-11)
    np.testing.assert_allclose(ex["values"][:T * B], tvalues, rtol=0, atol=1e-11)
    np.testing.assert_allclose(terms, tterms, rtol=1e-11, atol=1e-13)
    sl = gs.segment_slices(net)
    for name, s in sl.items():
        scale = np.abs(tg[s]).max()
        assert scale > 0, name
        assert np.abs(g[s] - tg[s]).max() <= 1e-10 * scale, name


def test_gradient_by_finite_differences_and_stop_gradient():
    net, T, B = TINY, 2, 2
    x, ro = _tiny_problem(net, T, B, seed=31)
    hp = dict(HP, ent_coef=0.05)
    args = (ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    g, terms, ex = orc.agent_gradient(net, T, B, hp, x, *args, extras=True)
    fixed = (ex["G"], ex["Adv"])
    h = 1e-6
    fd_fixed = np.empty_like(x)
    fd_free = np.empty_like(x)
    for i in range(x.size):
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        fd_fixed[i] = (orc.total_loss(orc.agent_loss(net, T, B, hp, xp, *args, fixed=fixed), hp) -
                       orc.total_loss(orc.agent_loss(net, T, B, hp, xm, *args, fixed=fixed), hp)) / (2 * h)
        fd_free[i] = (orc.total_loss(orc.agent_loss(net, T, B, hp, xp, *args), hp) -
                      orc.total_loss(orc.agent_loss(net, T, B, hp, xm, *args), hp)) / (2 * h)
    scale = np.abs(g).max()
    assert np.abs(g - fd_fixed).max() < 1e-6 * scale
    # differentiating through the returns/advantages gives a different vector:
    # the oracle really treats them as constants
    assert np.abs(g - fd_free).max() > 1e-3 * scale


def test_agents_are_independent_in_the_learner_step():
    net = MID
    N, T, B = 3, 2, 2
    X = gs.init_params(net, N, seed=41, bias_scale=0.1)
    ro = gs.rollout(net, N, T, B, 41)
    o = orc.OracleGala(net, N, T, B, HP, "ring")
    o.set_params(X)
    o.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    for i in range(N):
        g, _ = orc.agent_gradient(net, T, B, HP, X[i], ro["obs"][i], ro["actions"][i],
                                  ro["rewards"][i], ro["dones"][i], ro["boot_obs"][i])
        np.testing.assert_array_equal(o.grads[i], g)


# ---- clip and RMSprop (Table 2) ------------------------------------------------

def test_clip_below_threshold_is_identity():
    g = np.array([0.1, -0.2, 0.05])
    g0 = g.copy()
    norm, scale = orc.clip_grad_norm(g, 0.5)
    assert scale == 1.0 and np.array_equal(g, g0)
    assert abs(norm - np.sqrt(0.01 + 0.04 + 0.0025)) < 1e-15


def test_clip_above_threshold_rescales_to_the_bound():
    g = np.array([3.0, -4.0])
    norm, scale = orc.clip_grad_norm(g, 0.5)
    assert norm == 5.0
    assert abs(scale - 0.5 / (5.0 + 1e-6)) < 1e-16
    assert abs(np.linalg.norm(g) - 0.5 * 5.0 / (5.0 + 1e-6)) < 1e-15
    np.testing.assert_allclose(g / np.linalg.norm(g), [0.6, -0.8], atol=1e-15)


def test_rmsprop_first_step_and_constant_gradient():
    lr, alpha, eps = 7e-4, 0.99, 1e-5
    g = np.array([1e3, -1e3, 0.0, 2.0])
    x = np.zeros(4)
    v = np.zeros(4)
    orc.rmsprop(x, v, g, lr, alpha, eps)
    np.testing.assert_allclose(v, (1 - alpha) * g ** 2, rtol=1e-15)
    # first step from v = 0: -lr g / (sqrt(1-alpha) |g| + eps) -> -lr sign(g) / sqrt(1 - alpha)
    np.testing.assert_allclose(x[:2], [-7e-3, 7e-3], rtol=1e-6)
    assert x[2] == 0.0
    assert abs(x[3] + lr * 2.0 / (np.sqrt(0.01 * 4.0) + eps)) < 1e-17
    for k in range(2, 6):
        orc.rmsprop(x, v, g, lr, alpha, eps)
        np.testing.assert_allclose(v, (1 - alpha ** k) * g ** 2, rtol=1e-13)


def test_learner_step_composes_gradient_clip_and_rmsprop():
    net, N, T, B = MID, 2, 2, 2
    X = gs.init_params(net, N, seed=51, bias_scale=0.1)
    ro = gs.rollout(net, N, T, B, 51)
    hp = dict(HP, max_grad_norm=0.05)
    o = orc.OracleGala(net, N, T, B, hp, "ring")
    o.set_params(X)
    V0 = np.abs(np.random.default_rng(0).normal(size=o.V.shape)) * 1e-3
    o.set_opt_state(V0)
    o.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    clipped = 0
    for i in range(N):
        g = o.grads[i].copy()
        n = np.linalg.norm(g)
        c = min(1.0, hp["max_grad_norm"] / (n + 1e-6))
        clipped += c < 1.0
        g *= c
        v = hp["rms_alpha"] * V0[i] + (1 - hp["rms_alpha"]) * g * g
        x = X[i].astype(np.float64) - hp["lr"] * g / (np.sqrt(v) + hp["rms_eps"])
        np.testing.assert_allclose(o.V[i], v, rtol=1e-14, atol=0)
        np.testing.assert_allclose(o.X[i], x, rtol=1e-13, atol=1e-16)
        assert abs(o.stats[i, 3] - n) < 1e-12 * n and abs(o.stats[i, 4] - c) < 1e-14
    assert clipped > 0


def test_relu_marks_only_change_the_marked_unit():
    """Marks equal to the natural decisions change nothing; blocking one active unit
    changes the gradient, and only for parameters at or below that unit's layer."""
    net, T, B = MID, 2, 2
    x, ro = _tiny_problem(net, T, B, seed=61)
    args = (ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    g0, _ = orc.agent_gradient(net, T, B, HP, x, *args)
    M = T * B
    obs = ro["obs"].reshape((M,) + ro["obs"].shape[2:])
    _, _, acts = orc.forward_acts(net, x, obs)
    natural = np.where(acts > 0, 1, 2).astype(np.uint8)
    g1, _ = orc.agent_gradient(net, T, B, HP, x, *args, gate=natural)
    np.testing.assert_array_equal(g0, g1)
    off, shape = orc.act_offsets(net)["conv2"]
    frame = 1
    idx = off + int(np.argmax(acts[frame, off:off + int(np.prod(shape))]))
    gate = np.zeros_like(natural)
    gate[frame, idx] = 2
    g2, _ = orc.agent_gradient(net, T, B, HP, x, *args, gate=gate)
    assert np.abs(g2 - g0).max() > 1e-6 * np.abs(g0).max()
    # blocking a unit only affects parameters at or below its layer
    sl = gs.segment_slices(net)
    for name in ("conv3.w", "conv3.b", "fc.w", "fc.b", "pi.w", "pi.b", "v.w", "v.b"):
        np.testing.assert_array_equal(g2[sl[name]], g0[sl[name]])
