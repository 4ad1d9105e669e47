"""ctypes front end of the CPU oracle (gala_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
module.  It shares nothing with the GPU library.  `OracleGala` strings the C
pieces together in the order of Algorithm 1 of the paper: learner step for
every agent, then one gossip round over the peer-to-peer topology, with the
message history kept as a plain dict {round: parameters sent that round}.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gala_oracle.c")
_LIB = os.path.join(_HERE, "libgala_oracle.so")

MAX_CONV = 4


def build(force: bool = False) -> str:
    """Compile gala_oracle.c with gcc into libgala_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Net(C.Structure):
    _fields_ = [("in_c", C.c_int), ("in_h", C.c_int), ("in_w", C.c_int), ("n_conv", C.c_int),
                ("conv_out", C.c_int * MAX_CONV), ("conv_k", C.c_int * MAX_CONV),
                ("conv_stride", C.c_int * MAX_CONV), ("fc", C.c_int), ("n_actions", C.c_int)]


class _HParams(C.Structure):
    _fields_ = [("T", C.c_int), ("B", C.c_int), ("gamma", C.c_double), ("vf_coef", C.c_double),
                ("ent_coef", C.c_double), ("lr", C.c_double), ("rms_alpha", C.c_double),
                ("rms_eps", C.c_double), ("max_grad_norm", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_param_count.restype = C.c_long
        L.orc_act_size.restype = C.c_long
        L.orc_clip_grad_norm.restype = C.c_double
        L.orc_clip_grad_norm.argtypes = [C.c_void_p, C.c_long, C.c_double, C.c_void_p]
        L.orc_rmsprop.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_long,
                                  C.c_double, C.c_double, C.c_double]
        L.orc_in_peer.argtypes = [C.c_int, C.c_int, C.c_long, C.c_int]
        L.orc_edge_delay.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_nstep_returns.argtypes = [C.c_int, C.c_int, C.c_double] + [C.c_void_p] * 6
        L.orc_a2c_loss.argtypes = ([C.c_int, C.c_int] + [C.c_void_p] * 5 +
                                   [C.c_double, C.c_double] + [C.c_void_p] * 3)
        L.orc_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int] + [C.c_void_p] * 4
        L.orc_agent_gradient.argtypes = [C.c_void_p] * 15
        L.orc_agent_loss.argtypes = [C.c_void_p] * 11
        L.orc_learner_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int] + [C.c_void_p] * 10
        L.orc_a2c_allreduce_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int] + [C.c_void_p] * 11
        L.orc_uniform24.restype = C.c_double
        L.orc_uniform24.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_categorical_sample.argtypes = [C.c_int, C.c_void_p, C.c_double, C.c_void_p, C.c_void_p]
        L.orc_mix_uniform.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_long, C.c_void_p]
        L.orc_mix_weighted.argtypes = [C.c_void_p, C.c_double, C.c_void_p, C.c_void_p,
                                       C.c_int, C.c_long, C.c_void_p]
        L.orc_consensus_distance.argtypes = [C.c_void_p, C.c_int, C.c_long, C.c_void_p, C.c_void_p]
        L.orc_cosine_matrix.argtypes = [C.c_void_p, C.c_int, C.c_long, C.c_void_p]
        L.orc_update_norm.restype = C.c_double
        L.orc_update_norm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_long, C.c_void_p]
        L.orc_prop1_bound.restype = C.c_double
        L.orc_prop1_bound.argtypes = [C.c_double, C.c_void_p, C.c_int]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def c_net(net: dict) -> _Net:
    n = _Net()
    n.in_c, n.in_h, n.in_w = net["in_c"], net["in_h"], net["in_w"]
    n.n_conv = len(net["conv"])
    for i, (o, k, s) in enumerate(net["conv"]):
        n.conv_out[i], n.conv_k[i], n.conv_stride[i] = o, k, s
    n.fc, n.n_actions = net["fc"], net["n_actions"]
    return n


def c_hparams(T: int, B: int, hp: dict) -> _HParams:
    h = _HParams()
    h.T, h.B = T, B
    for k in ("gamma", "vf_coef", "ent_coef", "lr", "rms_alpha", "rms_eps", "max_grad_norm"):
        setattr(h, k, float(hp[k]))
    return h


# ---- thin numpy wrappers of the C pieces -----------------------------------

def param_count(net: dict) -> int:
    n = c_net(net)
    return int(lib().orc_param_count(C.byref(n)))


def forward(net: dict, x: np.ndarray, obs: np.ndarray):
    """obs uint8 [F, C, H, W]; returns logits [F, A], values [F]."""
    n = c_net(net)
    x = np.ascontiguousarray(x, dtype=np.float64)
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    F = obs.shape[0]
    logits = np.empty((F, net["n_actions"]))
    values = np.empty(F)
    lib().orc_forward(C.byref(n), _p(x), _p(obs), F, _p(logits), _p(values), None, None)
    return logits, values


def forward_acts(net: dict, x: np.ndarray, obs: np.ndarray, with_pre: bool = False):
    """As forward(), also returning the per-frame record [F, act_size]
    (scaled input, each conv output after ReLU, hidden after ReLU) and, with
    with_pre=True, the values before each ReLU at the same offsets."""
    n = c_net(net)
    x = np.ascontiguousarray(x, dtype=np.float64)
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    F = obs.shape[0]
    logits = np.empty((F, net["n_actions"]))
    values = np.empty(F)
    acts = np.empty((F, int(lib().orc_act_size(C.byref(n)))))
    pre = np.zeros_like(acts) if with_pre else None
    lib().orc_forward(C.byref(n), _p(x), _p(obs), F, _p(logits), _p(values), _p(acts), _p(pre))
    if with_pre:
        return logits, values, acts, pre
    return logits, values, acts


def act_offsets(net: dict) -> dict:
    """Offsets and CHW shapes of each layer's output inside a per-frame record."""
    c, h, w = net["in_c"], net["in_h"], net["in_w"]
    off = c * h * w
    out = {}
    for li, (o, k, s) in enumerate(net["conv"], start=1):
        h = (h - k) // s + 1
        w = (w - k) // s + 1
        out[f"conv{li}"] = (off, (o, h, w))
        off += o * h * w
    out["fc"] = (off, (net["fc"],))
    return out


def nstep_returns(rewards, dones, v_boot, values, gamma):
    rewards = np.ascontiguousarray(rewards, dtype=np.float64)
    dones = np.ascontiguousarray(dones, dtype=np.uint8)
    v_boot = np.ascontiguousarray(v_boot, dtype=np.float64)
    values = np.ascontiguousarray(values, dtype=np.float64)
    T, B = rewards.shape
    G = np.empty((T, B))
    Adv = np.empty((T, B))
    lib().orc_nstep_returns(T, B, float(gamma), _p(rewards), _p(dones), _p(v_boot), _p(values),
                            _p(G), _p(Adv))
    return G, Adv


def a2c_loss(logits, values, actions, G, Adv, vf_coef, ent_coef):
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    values = np.ascontiguousarray(values, dtype=np.float64).ravel()
    actions = np.ascontiguousarray(actions, dtype=np.int32).ravel()
    G = np.ascontiguousarray(G, dtype=np.float64).ravel()
    Adv = np.ascontiguousarray(Adv, dtype=np.float64).ravel()
    M, A = logits.shape
    terms = np.empty(3)
    dlogits = np.empty((M, A))
    dvalues = np.empty(M)
    lib().orc_a2c_loss(M, A, _p(logits), _p(values), _p(actions), _p(G), _p(Adv),
                       float(vf_coef), float(ent_coef), _p(terms), _p(dlogits), _p(dvalues))
    return terms, dlogits, dvalues


def agent_gradient(net, T, B, hp, x, obs, actions, rewards, dones, boot_obs, extras=False, gate=None):
    """Gradient of one agent's loss.  Returns (grads[d], terms[3]) and, with
    extras=True, also a dict with G, Adv, logits, values (rollout then bootstrap)."""
    n, h = c_net(net), c_hparams(T, B, hp)
    x = np.ascontiguousarray(x, dtype=np.float64)
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    boot_obs = np.ascontiguousarray(boot_obs, dtype=np.uint8)
    actions = np.ascontiguousarray(actions, dtype=np.int32)
    rewards = np.ascontiguousarray(rewards, dtype=np.float64)
    dones = np.ascontiguousarray(dones, dtype=np.uint8)
    M, A = T * B, net["n_actions"]
    g = np.empty(x.shape[0])
    terms = np.empty(3)
    G = np.empty(M); Adv = np.empty(M); lg = np.empty((M, A)); vals = np.empty(M + B)
    lib().orc_agent_gradient(C.byref(n), C.byref(h), _p(x), _p(obs), _p(actions), _p(rewards),
                             _p(dones), _p(boot_obs), _p(g), _p(terms),
                             _p(G), _p(Adv), _p(lg), _p(vals),
                             _p(None if gate is None else np.ascontiguousarray(gate, dtype=np.uint8)))
    if extras:
        return g, terms, dict(G=G, Adv=Adv, logits=lg, values=vals)
    return g, terms


def agent_loss(net, T, B, hp, x, obs, actions, rewards, dones, boot_obs, fixed=None):
    """The three loss terms; fixed=(G, Adv) holds returns/advantages constant."""
    n, h = c_net(net), c_hparams(T, B, hp)
    x = np.ascontiguousarray(x, dtype=np.float64)
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    boot_obs = np.ascontiguousarray(boot_obs, dtype=np.uint8)
    actions = np.ascontiguousarray(actions, dtype=np.int32)
    rewards = np.ascontiguousarray(rewards, dtype=np.float64)
    dones = np.ascontiguousarray(dones, dtype=np.uint8)
    terms = np.empty(3)
    fG = fA = None
    if fixed is not None:
        fG = np.ascontiguousarray(fixed[0], dtype=np.float64).ravel()
        fA = np.ascontiguousarray(fixed[1], dtype=np.float64).ravel()
    lib().orc_agent_loss(C.byref(n), C.byref(h), _p(x), _p(obs), _p(actions), _p(rewards),
                         _p(dones), _p(boot_obs), _p(fG), _p(fA), _p(terms))
    return terms


def total_loss(terms, hp):
    return terms[0] + hp["vf_coef"] * terms[1] - hp["ent_coef"] * terms[2]


def clip_grad_norm(g: np.ndarray, max_norm: float):
    """In place on a float64 vector; returns (pre-clip norm, scale)."""
    assert g.dtype == np.float64 and g.flags.c_contiguous
    scale = C.c_double(0.0)
    norm = lib().orc_clip_grad_norm(_p(g), g.size, float(max_norm), C.byref(scale))
    return float(norm), float(scale.value)


def rmsprop(x: np.ndarray, v: np.ndarray, g: np.ndarray, lr, alpha, eps):
    for a in (x, v, g):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    lib().orc_rmsprop(_p(x), _p(v), _p(g), x.size, float(lr), float(alpha), float(eps))


TOPOLOGY_KIND = {"ring": 0, "exp": 1, "exp_reverse": 2}


def in_peer(kind: str, N: int, rnd: int, i: int) -> int:
    return int(lib().orc_in_peer(TOPOLOGY_KIND[kind], N, rnd, i))


def n_phases(kind: str, N: int) -> int:
    return int(lib().orc_n_phases(TOPOLOGY_KIND[kind], N))


def edge_delay(seed: int, N: int, phase: int, i: int, max_delay: int) -> int:
    return int(lib().orc_edge_delay(seed, N, phase, i, max_delay))


def peer_table(kind: str, N: int, rnd: int, max_delay: int = 0, delay_seed: int = 0):
    """(peer[N], delay[N]) int32 tables for one round."""
    phase = rnd % n_phases(kind, N)
    peer = np.array([in_peer(kind, N, rnd, i) for i in range(N)], dtype=np.int32)
    delay = np.array([edge_delay(delay_seed, N, phase, i, max_delay) for i in range(N)], dtype=np.int32)
    return peer, delay


def uniform24(seed: int, counter: int) -> float:
    return float(lib().orc_uniform24(seed % 2 ** 64, counter % 2 ** 64))


def categorical_sample(logits, u: float):
    """(action, log pi(action), running sums of pi) for one draw with the uniform variate u."""
    z = np.ascontiguousarray(logits, dtype=np.float64)
    cdf = np.empty(z.size)
    lp = C.c_double()
    a = lib().orc_categorical_sample(z.size, _p(z), float(u), C.byref(lp), _p(cdf))
    return int(a), lp.value, cdf


def act_counter(step: int, n_agents: int, B: int, agent: int, env: int) -> int:
    """Index of the uniform variate of (acting step, agent, simulator)."""
    return (step * n_agents + agent) * B + env


def act(net: dict, X: np.ndarray, obs: np.ndarray, seed: int, step: int):
    """Acting step of Algorithm 1 for all agents: obs uint8 [N, B, C, H, W] -> sampled actions
    [N, B], values [N, B], log pi(a|s) [N, B], the uniform variates and running sums used."""
    N, B = obs.shape[:2]
    A = net["n_actions"]
    actions = np.empty((N, B), dtype=np.int32)
    values = np.empty((N, B))
    logp = np.empty((N, B))
    us = np.empty((N, B))
    cdfs = np.empty((N, B, A))
    for i in range(N):
        logits, values[i] = forward(net, np.asarray(X[i], dtype=np.float64), obs[i])
        for b in range(B):
            us[i, b] = uniform24(seed, act_counter(step, N, B, i, b))
            actions[i, b], logp[i, b], cdfs[i, b] = categorical_sample(logits[b], us[i, b])
    return actions, values, logp, us, cdfs


def mix_uniform(x: np.ndarray, msgs: list[np.ndarray]) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    msgs = [np.ascontiguousarray(m, dtype=np.float64) for m in msgs]
    out = np.empty_like(x)
    arr = (C.c_void_p * max(1, len(msgs)))(*[m.ctypes.data for m in msgs])
    lib().orc_mix_uniform(_p(x), arr, len(msgs), x.size, _p(out))
    return out


def mix_weighted(x: np.ndarray, w_self: float, msgs: list[np.ndarray], w: list[float]) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    msgs = [np.ascontiguousarray(m, dtype=np.float64) for m in msgs]
    wv = np.ascontiguousarray(w, dtype=np.float64)
    out = np.empty_like(x)
    arr = (C.c_void_p * max(1, len(msgs)))(*[m.ctypes.data for m in msgs])
    lib().orc_mix_weighted(_p(x), float(w_self), arr, _p(wv), len(msgs), x.size, _p(out))
    return out


def consensus_distance(X: np.ndarray):
    X = np.ascontiguousarray(X, dtype=np.float64)
    mx, fr = C.c_double(0.0), C.c_double(0.0)
    lib().orc_consensus_distance(_p(X), X.shape[0], X.shape[1], C.byref(mx), C.byref(fr))
    return float(mx.value), float(fr.value)


def cosine_matrix(G: np.ndarray) -> np.ndarray:
    """Pair-wise cosine similarity [N, N] of the rows of G (Fig. 2b)."""
    G = np.ascontiguousarray(G, dtype=np.float64)
    out = np.empty((G.shape[0], G.shape[0]))
    lib().orc_cosine_matrix(_p(G), G.shape[0], G.shape[1], _p(out))
    return out


def update_norm(X_before: np.ndarray, X_after: np.ndarray):
    """(||alpha G||_F, per-agent ||alpha g_i||_2) of one round's optimiser step (Prop. 1)."""
    a = np.ascontiguousarray(X_before, dtype=np.float64)
    b = np.ascontiguousarray(X_after, dtype=np.float64)
    rows = np.empty(a.shape[0])
    fr = lib().orc_update_norm(_p(a), _p(b), a.shape[0], a.shape[1], _p(rows))
    return float(fr), rows


def prop1_bound(beta: float, update_norms) -> float:
    u = np.ascontiguousarray(update_norms, dtype=np.float64)
    return float(lib().orc_prop1_bound(float(beta), _p(u), u.size))


# ---- Algorithm 1 for N agents ------------------------------------------------

class OracleGala:
    """N independent A2C actor-learners plus gossip, in double precision.

    State: X [N, d] parameters, V [N, d] RMSprop second-moment estimates, and the
    history {round: parameters broadcast in that round} needed for delayed
    messages (Eq. (6): a message carries the sender's parameters as of the time
    it was sent)."""

    def __init__(self, net: dict, n_agents: int, T: int, B: int, hp: dict, topology: str = "ring",
                 max_delay: int = 0, delay_seed: int = 0):
        self.net, self.N, self.T, self.B, self.hp = net, n_agents, T, B, dict(hp)
        self.topology, self.max_delay, self.delay_seed = topology, max_delay, delay_seed
        if topology in ("exp", "exp_reverse") and n_agents & (n_agents - 1):
            raise ValueError("the exponential graph needs a power-of-two number of agents")
        self.d = param_count(net)
        self.X = np.zeros((n_agents, self.d))
        self.V = np.zeros((n_agents, self.d))
        self.sent: dict[int, np.ndarray] = {}
        self.grads = None
        self.stats = None

    def set_params(self, X):
        self.X = np.array(X, dtype=np.float64).reshape(self.N, self.d)

    def set_opt_state(self, V):
        self.V = np.array(V, dtype=np.float64).reshape(self.N, self.d)

    def learner_step(self, obs, actions, rewards, dones, boot_obs, gates=None):
        n, h = c_net(self.net), c_hparams(self.T, self.B, self.hp)
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        boot_obs = np.ascontiguousarray(boot_obs, dtype=np.uint8)
        actions = np.ascontiguousarray(actions, dtype=np.int32)
        rewards = np.ascontiguousarray(rewards, dtype=np.float32)
        dones = np.ascontiguousarray(dones, dtype=np.uint8)
        self.grads = np.empty((self.N, self.d))
        self.stats = np.empty((self.N, 5))
        lib().orc_learner_step(C.byref(n), C.byref(h), self.N, _p(self.X), _p(self.V),
                               _p(obs), _p(actions), _p(rewards), _p(dones), _p(boot_obs),
                               _p(self.grads), _p(self.stats),
                               _p(None if gates is None else np.ascontiguousarray(gates, dtype=np.uint8)))

    def a2c_allreduce_step(self, obs, actions, rewards, dones, boot_obs, gates=None):
        """Synchronous A2C comparator: the agents' gradients are averaged, clipped once and
        applied by every agent (Sec. 5, "Experimental setup")."""
        n, h = c_net(self.net), c_hparams(self.T, self.B, self.hp)
        obs = np.ascontiguousarray(obs, dtype=np.uint8)
        boot_obs = np.ascontiguousarray(boot_obs, dtype=np.uint8)
        actions = np.ascontiguousarray(actions, dtype=np.int32)
        rewards = np.ascontiguousarray(rewards, dtype=np.float32)
        dones = np.ascontiguousarray(dones, dtype=np.uint8)
        self.grads = np.empty((self.N, self.d))
        self.gbar = np.empty(self.d)
        self.stats = np.empty((self.N, 5))
        lib().orc_a2c_allreduce_step(C.byref(n), C.byref(h), self.N, _p(self.X), _p(self.V),
                                     _p(obs), _p(actions), _p(rewards), _p(dones), _p(boot_obs),
                                     _p(self.grads), _p(self.gbar), _p(self.stats),
                                     _p(None if gates is None else np.ascontiguousarray(gates, dtype=np.uint8)))

    def gossip(self, rnd: int):
        """Broadcast the post-update parameters, then every agent that holds a
        message from its in-peer averages with it; an agent whose (delayed)
        message does not exist yet keeps its own parameters."""
        Y = self.X.copy()
        self.sent[rnd] = Y
        for old in [r for r in self.sent if r < rnd - self.max_delay]:
            del self.sent[old]
        peer, delay = peer_table(self.topology, self.N, rnd, self.max_delay, self.delay_seed)
        Xn = np.empty_like(Y)
        for i in range(self.N):
            src_round = rnd - int(delay[i])
            if src_round < 0 or src_round not in self.sent:
                Xn[i] = Y[i]
            else:
                Xn[i] = mix_uniform(Y[i], [self.sent[src_round][peer[i]]])
        self.X = Xn

    def consensus_distance(self):
        return consensus_distance(self.X)
