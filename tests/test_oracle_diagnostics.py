"""Pins of the oracle's diagnostics (Sec. 5 "Effects of gossip"): the gradient
cosine-similarity matrix of Fig. 2b, the size of a round's local updates, and the bound of
Prop. 1, which is then checked as an inequality on the oracle's own training rounds."""
import numpy as np

import gala_synth as gs
from oracle import gala_oracle as orc
from test_oracle_learner import HP, MID


def test_cosine_hand_worked_vectors():
    G = np.array([[1.0, 0.0, 0.0], [0.0, 2.0, 0.0], [3.0, 3.0, 0.0], [-2.0, 0.0, 0.0], [0.0, 0.0, 0.0]])
    c = orc.cosine_matrix(G)
    r = np.sqrt(0.5)
    want = np.array([[1, 0, r, -1, 0], [0, 1, r, 0, 0], [r, r, 1, -r, 0], [-1, 0, -r, 1, 0], [0, 0, 0, 0, 0]])
    np.testing.assert_allclose(c, want, atol=1e-15)


def test_cosine_matches_normalised_gram_and_is_scale_invariant():
    rng = np.random.default_rng(0)
    G = rng.normal(size=(6, 1000))
    c = orc.cosine_matrix(G)
    Gn = G / np.linalg.norm(G, axis=1, keepdims=True)
    np.testing.assert_allclose(c, Gn @ Gn.T, atol=1e-13)
    np.testing.assert_allclose(np.diag(c), 1.0, atol=1e-15)
    np.testing.assert_array_equal(c, c.T)
    assert np.abs(c).max() <= 1.0 + 1e-15
    scale = np.array([1.0, 10.0, 1e-3, 5.0, 2.0, 7.0])[:, None]
    np.testing.assert_allclose(orc.cosine_matrix(G * scale), c, atol=1e-13)


def test_update_norm_hand_worked_and_rmsprop_displacement():
    a = np.array([[1.0, 2.0, 3.0], [0.0, 0.0, 0.0]])
    b = np.array([[1.0, 5.0, 7.0], [1.0, 0.0, 0.0]])
    fr, rows = orc.update_norm(a, b)
    np.testing.assert_allclose(rows, [5.0, 1.0])
    assert abs(fr - np.sqrt(26.0)) < 1e-15
    # one learner step: the displacement is lr * c * g / (sqrt(v) + eps)
    net, N, T, B = MID, 3, 2, 2
    X = gs.init_params(net, N, seed=71, bias_scale=0.1)
    ro = gs.rollout(net, N, T, B, 71)
    o = orc.OracleGala(net, N, T, B, HP, "ring")
    o.set_params(X)
    o.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
    fr, rows = orc.update_norm(X, o.X)
    for i in range(N):
        g = o.grads[i] * o.stats[i, 4]
        disp = HP["lr"] * g / (np.sqrt(o.V[i]) + HP["rms_eps"])
        assert abs(rows[i] - np.linalg.norm(disp)) <= 1e-9 * rows[i]
    assert abs(fr - np.linalg.norm(rows)) <= 1e-12 * fr


def test_prop1_bound_closed_forms():
    u = np.array([0.3, 1.1, 0.7, 2.0])
    # written out: beta^4 u0 + beta^3 u1 + beta^2 u2 + beta u3
    beta = 0.8
    assert abs(orc.prop1_bound(beta, u) - (beta ** 4 * 0.3 + beta ** 3 * 1.1 + beta ** 2 * 0.7 + beta * 2.0)) < 1e-15
    # recursion B_{k+1} = beta (B_k + u_k)
    bound = 0.0
    for k in range(u.size):
        bound = beta * (bound + u[k])
        assert abs(orc.prop1_bound(beta, u[:k + 1]) - bound) < 1e-14
    # constant updates: geometric series
    n, c = 30, 0.25
    assert abs(orc.prop1_bound(beta, np.full(n, c)) - c * beta * (1 - beta ** n) / (1 - beta)) < 1e-13
    assert orc.prop1_bound(0.0, u) == 0.0
    assert abs(orc.prop1_bound(1.0, u) - u.sum()) < 1e-15


def test_prop1_holds_on_the_ring_and_fails_for_a_smaller_beta():
    """Agents start identical, train on different data and gossip over the directed ring with
    weights 1/2: the mixing matrix is normal with second singular value cos(pi/n), so the
    distance from consensus must stay below the bound with that beta in every round.  With a
    beta that is too small the bound is violated, so the inequality is a real constraint on
    the mixing and update code."""
    net, N, T, B = MID, 4, 2, 2
    o = orc.OracleGala(net, N, T, B, dict(HP, lr=5e-3), "ring")
    o.set_params(gs.init_params(net, N, seed=72, shared=True, bias_scale=0.1))
    P = 0.5 * (np.eye(N) + np.roll(np.eye(N), -1, axis=1))
    sv = np.linalg.svd(P, compute_uv=False)
    beta = np.cos(np.pi / N)
    assert abs(sv[0] - 1.0) < 1e-12 and abs(sv[1] - beta) < 1e-12
    norms, violated_small = [], False
    for k in range(10):
        ro = gs.rollout(net, N, T, B, 7200 + k)
        before = o.X.copy()
        o.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
        norms.append(orc.update_norm(before, o.X)[0])
        o.gossip(k)
        _, frob = o.consensus_distance()
        assert frob > 0.0
        assert frob <= orc.prop1_bound(beta, norms) * (1 + 1e-12), f"round {k}"
        violated_small |= frob > orc.prop1_bound(0.25 * beta, norms)
    assert violated_small
