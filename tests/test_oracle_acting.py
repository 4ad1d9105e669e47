"""Pins of the oracle's acting step (Algorithm 1: take actions according to pi): the
counter-based uniform generator against splitmix64's published outputs, and the categorical
draw against hand-worked cases, numpy's searchsorted on the same distribution, and the
frequencies it must reproduce."""
import numpy as np

import gala_synth as gs
from oracle import gala_oracle as orc

GOLDEN = 0x9E3779B97F4A7C15


def test_uniform24_is_the_top_24_bits_of_splitmix64():
    # first three outputs of splitmix64 started from state 0 (reference implementation's vector)
    outs = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    for n, z in enumerate(outs):
        # output n+1 mixes the state (n+1) * golden; uniform24 adds one golden itself
        assert orc.uniform24(0, (n * GOLDEN) % 2 ** 64) == (z >> 40) / 2.0 ** 24
    assert orc.uniform24(12345, 678) == orc.uniform24(12345 + 678, 0)        # keyed by seed + counter only


def test_uniform24_range_grid_and_moments():
    u = np.array([orc.uniform24(99, c) for c in range(40000)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))                      # multiples of 2^-24
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / u.size)
    assert abs(u.var() - 1 / 12) < 0.002
    assert len(np.unique(u)) > 0.99 * u.size


def test_categorical_hand_worked():
    p = np.array([0.2, 0.5, 0.3])
    z = np.log(p) + 3.7                                                       # any shift of the logits
    for u, want in [(0.0, 0), (0.19, 0), (0.21, 1), (0.69, 1), (0.71, 2), (0.999999, 2)]:
        a, lp, cdf = orc.categorical_sample(z, u)
        assert a == want, (u, a)
        assert abs(lp - np.log(p[want])) < 1e-12
        np.testing.assert_allclose(cdf, [0.2, 0.7, 1.0], rtol=1e-12)


def test_categorical_degenerate_cases():
    assert orc.categorical_sample([0.3], 0.9)[0] == 0                         # a single action
    for u in (0.0, 0.5, 0.999):
        a, lp, _ = orc.categorical_sample([0.0, 800.0, -5.0], u)              # exp would overflow unshifted
        assert a == 1 and abs(lp) < 1e-12
    # equal logits: uniform, boundaries at k / A
    for k in range(4):
        assert orc.categorical_sample(np.zeros(4), (k + 0.5) / 4)[0] == k


def test_categorical_matches_searchsorted_and_frequencies():
    rng = np.random.default_rng(3)
    for A in (2, 6, 18, 64):
        z = rng.normal(scale=2.0, size=A)
        p = np.exp(z - z.max())
        p /= p.sum()
        cdf = np.cumsum(p)
        counts = np.zeros(A)
        n = 6000
        for c in range(n):
            u = orc.uniform24(A, c)
            a, lp, _ = orc.categorical_sample(z, u)
            assert a == min(int(np.searchsorted(cdf, u, side="right")), A - 1)
            counts[a] += 1
        sigma = np.sqrt(n * p * (1 - p)) + 1.0
        assert np.all(np.abs(counts - n * p) <= 4.5 * sigma)


def test_act_uses_each_agents_parameters_and_distinct_draws():
    net = dict(in_c=1, in_h=12, in_w=12, conv=[(2, 4, 2), (3, 2, 1), (3, 2, 1)], fc=8, n_actions=3)
    N, B = 3, 4
    X = gs.init_params(net, N, seed=8, bias_scale=0.2).astype(np.float64)
    obs = gs.rollout(net, N, 1, B, 17)["obs"][:, 0]
    actions, values, logp, us, cdfs = orc.act(net, X, obs, seed=5, step=2)
    assert actions.shape == (N, B) and actions.dtype == np.int32
    for i in range(N):
        logits, v = orc.forward(net, X[i], obs[i])
        np.testing.assert_array_equal(values[i], v)
        for b in range(B):
            assert us[i, b] == orc.uniform24(5, (2 * N + i) * B + b)
            lsm = logits[b] - np.log(np.exp(logits[b] - logits[b].max()).sum()) - logits[b].max()
            assert abs(logp[i, b] - lsm[actions[i, b]]) < 1e-12
            k = actions[i, b]
            assert cdfs[i, b, k] > us[i, b] and (k == 0 or cdfs[i, b, k - 1] <= us[i, b])
    assert len(np.unique(us)) == N * B
    assert not np.array_equal(us, orc.act(net, X, obs, seed=5, step=3)[3])
