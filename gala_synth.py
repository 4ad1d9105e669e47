"""Seeded synthetic inputs for the GALA-A2C learner step and gossip round.

This module only *draws numbers*: Atari-shaped observations, actions, rewards,
episode-end flags and initial network parameters.  It contains none of the
method's arithmetic (no returns, losses, updates or mixing) and is the single
piece shared by the CPU oracle's tests and the GPU path's tests and benchmark,
so that both sides are fed byte-identical inputs.

The stream is a counter-based generator: element ``i`` of stream ``s`` is
``splitmix64(key(s) + i)``, where ``splitmix64`` is Steele/Lea/Flood's
published finaliser.  Nothing depends on a library's RNG state.

Workload shape (App. C.2 / Table 2 of the paper): 84x84 grayscale frames,
4-frame stack, horizon N=5, 16 simulators per learner, rewards clipped to
[-1, 1].  The emulator itself is replaced by iid draws:
  observations  uniform bytes 0..255
  actions       uniform integers in [0, A)
  rewards       -1 / 0 / +1 with probabilities 0.05 / 0.85 / 0.10
  dones         Bernoulli(0.01)
  weights       N(0, 1/fan_in), biases 0
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 190604585

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def splitmix64(z: np.ndarray) -> np.ndarray:
    """The splitmix64 output function applied to (already incremented) states."""
    with np.errstate(over="ignore"):
        z = z.astype(np.uint64, copy=True)
        z ^= z >> np.uint64(30)
        z *= _C1
        z ^= z >> np.uint64(27)
        z *= _C2
        z ^= z >> np.uint64(31)
    return z


def _stream(seed: int, stream: int, n: int, start: int = 0) -> np.ndarray:
    """n consecutive 64-bit words of stream `stream` under `seed`."""
    with np.errstate(over="ignore"):
        key = splitmix64(np.array([(seed * 0x100000001B3 + stream) & 0xFFFFFFFFFFFFFFFF],
                                  dtype=np.uint64))[0]
        ctr = (np.arange(start, start + n, dtype=np.uint64) + np.uint64(1)) * _GOLDEN + key
    return splitmix64(ctr)


def _uniform01(seed: int, stream: int, n: int) -> np.ndarray:
    """n doubles in [0, 1) with 53 random bits each."""
    return (_stream(seed, stream, n) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def _bytes(seed: int, stream: int, n: int) -> np.ndarray:
    words = _stream(seed, stream, (n + 7) // 8)
    return words.view(np.uint8)[:n].copy()


def _normal(seed: int, stream: int, n: int) -> np.ndarray:
    """n standard normals (Box-Muller on two uniform streams)."""
    m = (n + 1) // 2
    u1 = 1.0 - _uniform01(seed, 2 * stream, m)          # (0, 1]
    u2 = _uniform01(seed, 2 * stream + 1, m)
    r = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(2.0 * np.pi * u2)
    out[1::2] = r * np.sin(2.0 * np.pi * u2)
    return out[:n]


# --------------------------------------------------------------------------
# network shape bookkeeping (shapes only)
# --------------------------------------------------------------------------

NATURE_CNN = dict(in_c=4, in_h=84, in_w=84,
                  conv=[(32, 8, 4), (64, 4, 2), (64, 3, 1)],   # (out channels, kernel, stride)
                  fc=512)


def make_net(n_actions: int, **overrides) -> dict:
    net = dict(NATURE_CNN)
    net["conv"] = list(NATURE_CNN["conv"])
    net["n_actions"] = int(n_actions)
    net.update(overrides)
    return net


def param_segments(net: dict) -> list[tuple[str, tuple[int, ...], int]]:
    """Canonical parameter order: (name, shape, fan_in) for every tensor.

    conv weights are OIHW, dense weights are (out, in); the dense layer after
    the last convolution sees its input flattened in C, H, W order."""
    segs = []
    c, h, w = net["in_c"], net["in_h"], net["in_w"]
    for li, (o, k, s) in enumerate(net["conv"], start=1):
        segs.append((f"conv{li}.w", (o, c, k, k), c * k * k))
        segs.append((f"conv{li}.b", (o,), 0))
        h = (h - k) // s + 1
        w = (w - k) // s + 1
        c = o
    flat = c * h * w
    segs.append(("fc.w", (net["fc"], flat), flat))
    segs.append(("fc.b", (net["fc"],), 0))
    segs.append(("pi.w", (net["n_actions"], net["fc"]), net["fc"]))
    segs.append(("pi.b", (net["n_actions"],), 0))
    segs.append(("v.w", (1, net["fc"]), net["fc"]))
    segs.append(("v.b", (1,), 0))
    return segs


def param_count(net: dict) -> int:
    return sum(int(np.prod(shape)) for _, shape, _ in param_segments(net))


def segment_slices(net: dict) -> dict[str, slice]:
    out, off = {}, 0
    for name, shape, _ in param_segments(net):
        n = int(np.prod(shape))
        out[name] = slice(off, off + n)
        off += n
    return out


# --------------------------------------------------------------------------
# draws
# --------------------------------------------------------------------------

def init_params(net: dict, n_agents: int, seed: int = BASE_SEED, shared: bool = False,
                bias_scale: float = 0.0) -> np.ndarray:
    """[n_agents, d] float32 initial parameters, N(0, 1/fan_in) weights.

    shared=True gives every agent the same vector (the identical-initialisation
    assumption under which the consensus bound's first term vanishes).
    bias_scale > 0 draws biases N(0, bias_scale^2) instead of zeros; tests use it
    so that a dropped bias term cannot hide."""
    d = param_count(net)
    x = np.empty((n_agents, d), dtype=np.float32)
    for i in range(n_agents):
        src = 0 if shared else i
        off = 0
        for si, (name, shape, fan_in) in enumerate(param_segments(net)):
            n = int(np.prod(shape))
            if fan_in > 0:
                vals = _normal(seed, 1000 + 64 * src + si, n) / np.sqrt(float(fan_in))
            elif bias_scale > 0.0:
                vals = _normal(seed, 1000 + 64 * src + si, n) * bias_scale
            else:
                vals = np.zeros(n)
            x[i, off:off + n] = vals.astype(np.float32)
            off += n
    return x


def rollout(net: dict, n_agents: int, T: int, B: int, seed: int) -> dict[str, np.ndarray]:
    """One synthetic rollout batch for all agents.

    obs       uint8  [N, T, B, C, H, W]
    boot_obs  uint8  [N, B, C, H, W]      the state after the last action
    actions   int32  [N, T, B]
    rewards   float32[N, T, B]
    dones     uint8  [N, T, B]
    """
    C, H, W = net["in_c"], net["in_h"], net["in_w"]
    A = net["n_actions"]
    n_obs = n_agents * T * B * C * H * W
    n_boot = n_agents * B * C * H * W
    n_s = n_agents * T * B
    obs = _bytes(seed, 1, n_obs).reshape(n_agents, T, B, C, H, W)
    boot = _bytes(seed, 2, n_boot).reshape(n_agents, B, C, H, W)
    actions = (_stream(seed, 3, n_s) % np.uint64(A)).astype(np.int32).reshape(n_agents, T, B)
    u = _uniform01(seed, 4, n_s)
    rewards = np.where(u < 0.05, -1.0, np.where(u < 0.90, 0.0, 1.0)).astype(np.float32)
    rewards = rewards.reshape(n_agents, T, B)
    dones = (_uniform01(seed, 5, n_s) < 0.01).astype(np.uint8).reshape(n_agents, T, B)
    return dict(obs=obs, boot_obs=boot, actions=actions, rewards=rewards, dones=dones)


def round_seed(cfg: int, rnd: int) -> int:
    return BASE_SEED + 1000 * cfg + rnd


# The five workload shapes (number of agents, topology, actions, T, B, rounds, delay bound).
CONFIGS = {
    1: dict(n_agents=2, topology="ring", n_actions=6, T=5, B=4, rounds=1, max_delay=0),
    2: dict(n_agents=4, topology="exp", n_actions=18, T=5, B=16, rounds=100, max_delay=0),
    3: dict(n_agents=8, topology="exp", n_actions=18, T=5, B=16, rounds=200, max_delay=2),
    4: dict(n_agents=32, topology="exp", n_actions=18, T=5, B=16, rounds=1000, max_delay=0),
    5: dict(n_agents=64, topology="exp", n_actions=18, T=5, B=32, rounds=1, max_delay=0),
}

HPARAMS = dict(gamma=0.99, vf_coef=0.5, ent_coef=0.01, lr=7e-4, rms_alpha=0.99,
               rms_eps=1e-5, max_grad_norm=0.5)
