"""Pins of the oracle's gossip side: integer topology tables by brute force,
and the invariants that Sec. 2 ("Gossip algorithms"), Algorithm 1 and App. B of
the paper attach to row- / doubly-stochastic mixing."""
import numpy as np
import pytest

import gala_synth as gs
from oracle import gala_oracle as orc

NET = dict(in_c=1, in_h=12, in_w=12, conv=[(2, 4, 2), (3, 2, 1), (3, 2, 1)], fc=8, n_actions=3)


def _gossip_only(N, topology, X0, rounds, max_delay=0, seed=0):
    o = orc.OracleGala(NET, N, 1, 1, gs.HPARAMS, topology, max_delay=max_delay, delay_seed=seed)
    o.d = X0.shape[1]
    o.set_params(X0)
    out = []
    for r in range(rounds):
        o.gossip(r)
        out.append(o.X.copy())
    return out


def _mixing_matrix(topology, N, rnd):
    P = np.zeros((N, N))
    for i in range(N):
        P[i, i] += 0.5
        P[i, orc.in_peer(topology, N, rnd, i)] += 0.5
    return P


# ---- integer tables ---------------------------------------------------------------

@pytest.mark.parametrize("N", [2, 4, 8, 32, 64])
def test_ring_table(N):
    # v_1 -> v_2 -> ... -> v_n -> v_1: the sender into i is its predecessor
    for r in (0, 1, 7):
        assert [orc.in_peer("ring", N, r, i) for i in range(N)] == [(i - 1) % N for i in range(N)]


@pytest.mark.parametrize("N", [2, 4, 8, 32, 64])
def test_exponential_table(N):
    m = N.bit_length() - 1
    assert orc.n_phases("exp", N) == m
    for r in range(3 * m):
        want = [(i + 2 ** (r % m)) % N for i in range(N)]
        got = [orc.in_peer("exp", N, r, i) for i in range(N)]
        assert got == want
        assert sorted(got) == list(range(N))         # a permutation: P is doubly stochastic
        P = _mixing_matrix("exp", N, r)
        np.testing.assert_array_equal(P.sum(0), np.ones(N))
        np.testing.assert_array_equal(P.sum(1), np.ones(N))


@pytest.mark.parametrize("N", [2, 4, 8, 32, 64])
def test_reverse_exponential_table_is_the_transposed_graph(N):
    """Every edge of the exponential graph turned round: the mixing matrix is the transpose of the
    forward one (sender and receiver swap), itself doubly stochastic, and log2 N rounds still
    give the exact average."""
    m = N.bit_length() - 1
    assert orc.n_phases("exp_reverse", N) == m
    for r in range(2 * m):
        fwd = [orc.in_peer("exp", N, r, i) for i in range(N)]
        rev = [orc.in_peer("exp_reverse", N, r, i) for i in range(N)]
        assert rev == [(i - 2 ** (r % m)) % N for i in range(N)]
        assert all(rev[fwd[i]] == i for i in range(N))            # the inverse permutation
        np.testing.assert_array_equal(_mixing_matrix("exp_reverse", N, r), _mixing_matrix("exp", N, r).T)
    X0 = np.random.default_rng(3).normal(size=(N, 17))
    Xs = _gossip_only(N, "exp_reverse", X0, m)
    np.testing.assert_allclose(Xs[-1], np.tile(X0.mean(0), (N, 1)), atol=1e-14)
    if N > 2:    # and it is a different graph: one round differs from the forward direction
        assert np.abs(Xs[0] - _gossip_only(N, "exp", X0, 1)[0]).max() > 1e-3


def test_edge_delay_is_splitmix64_of_the_edge_key():
    # independent restatement with Python integers of the published splitmix64 step
    def sm64(z):
        z = (z + 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & (2 ** 64 - 1)
        return z ^ (z >> 31)
    # first outputs of the reference generator seeded with 0 (published test vector)
    assert sm64(0) == 0xE220A8397B1DCDAF
    N, seed = 8, 77
    seen = set()
    for k in range(3):
        for i in range(N):
            want = sm64(seed + k * N + i) % 3
            assert orc.edge_delay(seed, N, k, i, 2) == want
            seen.add(want)
            assert orc.edge_delay(seed, N, k, i, 0) == 0
    assert seen == {0, 1, 2}


# ---- mixing invariants ----------------------------------------------------------------

def test_two_agent_ring_averages_exactly_in_one_round():
    X0 = np.random.default_rng(0).normal(size=(2, 50))
    X1 = _gossip_only(2, "ring", X0, 1)[0]
    np.testing.assert_allclose(X1[0], X0.mean(0), rtol=0, atol=1e-16)
    np.testing.assert_array_equal(X1[0], X1[1])


@pytest.mark.parametrize("topology,N", [("ring", 4), ("ring", 8), ("exp", 4), ("exp", 32)])
def test_mean_preserved_and_consensus_is_fixed_point(topology, N):
    rng = np.random.default_rng(1)
    X0 = rng.normal(size=(N, 40))
    Xs = _gossip_only(N, topology, X0, 6)
    for X in Xs:                                        # doubly stochastic: column means stay
        np.testing.assert_allclose(X.mean(0), X0.mean(0), rtol=0, atol=1e-15)
    c = rng.normal(size=40)
    Xc = np.tile(c, (N, 1))
    for X in _gossip_only(N, topology, Xc, 3):           # row stochastic: 1 c^T is fixed
        np.testing.assert_array_equal(X, Xc)


@pytest.mark.parametrize("N", [2, 4, 8, 32, 64])
def test_exponential_graph_reaches_exact_average_in_log2_rounds(N):
    m = N.bit_length() - 1
    X0 = np.random.default_rng(2).normal(size=(N, 30))
    Xs = _gossip_only(N, "exp", X0, m)
    mx, fr = orc.consensus_distance(Xs[-1])
    assert mx < 1e-14 and fr < 1e-13
    np.testing.assert_allclose(Xs[-1], np.tile(X0.mean(0), (N, 1)), atol=1e-14)
    if m > 1:
        assert orc.consensus_distance(Xs[-2])[0] > 1e-3   # not before


@pytest.mark.parametrize("N", [4, 8, 16])
def test_ring_contracts_by_cos_pi_over_n(N):
    # P = (I + shift)/2 is circulant, singular values |cos(pi j / N)|: away from the
    # consensus direction one round shrinks the Frobenius distance by at most cos(pi/N)
    X = np.random.default_rng(3).normal(size=(N, 25))
    prev = orc.consensus_distance(X)[1]
    for Xn in _gossip_only(N, "ring", X, 10):
        cur = orc.consensus_distance(Xn)[1]
        assert cur <= np.cos(np.pi / N) * prev * (1 + 1e-12)
        prev = cur
    # the bound is attained by the slowest mode
    j = np.arange(N)
    mode = np.stack([np.cos(2 * np.pi * j / N), np.sin(2 * np.pi * j / N)], axis=1)
    d0 = orc.consensus_distance(mode)[1]
    d1 = orc.consensus_distance(_gossip_only(N, "ring", mode, 1)[0])[1]
    assert abs(d1 / d0 - np.cos(np.pi / N)) < 1e-12


def test_consensus_distance_definition():
    X = np.array([[1.0, 2.0], [3.0, 6.0], [2.0, 1.0]])
    mean = np.array([2.0, 3.0])
    rows = np.sqrt(((X - mean) ** 2).sum(1))
    mx, fr = orc.consensus_distance(X)
    assert abs(mx - rows.max()) < 1e-15 and abs(fr - np.sqrt((rows ** 2).sum())) < 1e-15


def test_mix_matches_dense_matrix_product():
    N = 8
    X0 = np.random.default_rng(4).normal(size=(N, 12))
    Xs = _gossip_only(N, "exp", X0, 5)
    X = X0
    for r in range(5):
        X = _mixing_matrix("exp", N, r) @ X
        np.testing.assert_allclose(Xs[r], X, rtol=0, atol=1e-15)


def test_weighted_mix_is_a_row_of_P_times_X():
    rng = np.random.default_rng(5)
    X = rng.normal(size=(4, 9))
    w = np.array([0.1, 0.2, 0.3, 0.4])
    out = orc.mix_weighted(X[2], w[2], [X[0], X[1], X[3]], [w[0], w[1], w[3]])
    np.testing.assert_allclose(out, w @ X, atol=1e-15)
    out = orc.mix_uniform(X[0], [X[1], X[2]])
    np.testing.assert_allclose(out, X[:3].mean(0), atol=1e-15)


# ---- delayed messages (Eq. (6), augmented graph of App. B) -----------------------

def test_zero_delay_bound_reduces_to_plain_mixing():
    N = 8
    X0 = np.random.default_rng(6).normal(size=(N, 20))
    a = _gossip_only(N, "exp", X0, 7)
    b = _gossip_only(N, "exp", X0, 7, max_delay=0, seed=123)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_delayed_mix_equals_augmented_matrix_iteration():
    """n (tau + 1) virtual nodes: block s of the augmented state holds the
    parameters broadcast s rounds ago.  One gossip-only round is then a single
    row-stochastic matrix applied to the stacked state."""
    N, tau, d, seed = 4, 2, 3, 99
    rng = np.random.default_rng(7)
    X0 = rng.normal(size=(N, d))
    rounds = 9
    got = _gossip_only(N, "exp", X0, rounds, max_delay=tau, seed=seed)
    delays_seen = set()

    Z = np.zeros((N * (tau + 1), d))        # [age][agent]
    Z[:N] = X0
    for r in range(rounds):
        peer, delay = orc.peer_table("exp", N, r, tau, seed)
        Pt = np.zeros((N * (tau + 1),) * 2)
        for i in range(N):
            dl = int(delay[i])
            delays_seen.add(dl)
            if r - dl < 0:                   # message not sent yet: agent keeps its value
                Pt[i, i] = 1.0
            else:
                Pt[i, i] += 0.5
                Pt[i, dl * N + peer[i]] += 0.5
        for s in range(1, tau + 1):          # age the history
            for i in range(N):
                Pt[s * N + i, (s - 1) * N + i] = 1.0
        np.testing.assert_allclose(Pt.sum(1), 1.0)       # row stochastic
        # Z's block 0 must hold the parameters *broadcast* this round, i.e. the
        # pre-mix values, when older blocks are read; the mix reads delayed blocks
        # of the previous state and its own current block.
        Z = Pt @ Z
        np.testing.assert_allclose(got[r], Z[:N], rtol=0, atol=1e-15)
    assert delays_seen == {0, 1, 2}
