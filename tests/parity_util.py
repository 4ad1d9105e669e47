"""Helpers shared by the GPU parity tests: run one round on both sides, compare."""
from __future__ import annotations

import numpy as np

import gala_synth as gs

# Tolerance (fp32 path vs. fp64 oracle): per tensor, max |gpu - ref| / max |ref| <= 1e-4.
# Element-wise relative error is meaningless for gradients that are exactly or nearly
# zero behind a ReLU, hence the norm-wise form.  Derivation: every output is a sum of at
# most 32000 fp32 products accumulated in fp32 (unit round-off 6e-8), giving a relative
# error of the order sqrt(32000) * 6e-8 ~ 1e-5 against the largest entry.
RTOL = 1e-4


def rel_err(got, ref, scale=None) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max() if scale is None else scale
    return float(np.abs(got - ref).max() / (scale + 1e-30))


def grad_scale(ref_agent, sl, name) -> float:
    """Magnitude a gradient tensor's error is measured against: its own largest entry; for a
    bias (a plain sum of the layer's output gradients, which can cancel to almost nothing, e.g.
    the value head's bias = -2 c_v mean(G - V)) not less than the largest entry of the layer."""
    own = np.abs(ref_agent[sl[name]]).max()
    if name.endswith(".b"):
        own = max(own, np.abs(ref_agent[sl[name[:-2] + ".w"]]).max())
    return float(own)


def upload(ro: dict):
    import torch
    return {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in ro.items()}


# A ReLU unit whose pre-activation is within single-precision rounding of zero has its
# derivative decided by rounding; fp32 and fp64 may legitimately disagree there.  The
# decision is then taken in the kernel's precision: the test reads the GPU's activations,
# requires every disagreeing unit to have |z| <= KINK * max|z| of its layer *in the oracle's
# own forward pass*, and only for those units tells the oracle which way the GPU went.
KINK = 1e-5


def relu_gates(gpu, net, X, ro, agents=None):
    """Per agent ReLU-derivative marks [len(agents), M, act_size] (0 = oracle decides) and
    the number of marked units.  Also checks every activation tensor against the oracle."""
    from oracle import gala_oracle as orc
    agents = list(range(gpu.N)) if agents is None else list(agents)
    M = gpu.T * gpu.B
    offs = orc.act_offsets(net)
    layers = [("conv1", 1), ("conv2", 2), ("conv3", 3), ("fc", 4)]
    gpu_acts = {}
    for name, li in layers:
        a = gpu.get_activations(li)
        if a.ndim == 5:
            a = a.transpose(0, 1, 4, 2, 3)             # channels-last -> channel, row, column
        gpu_acts[name] = a.reshape(gpu.N, a.shape[1], -1)
    gates = None
    marked = 0
    for gi, i in enumerate(agents):
        obs = ro["obs"][i].reshape((M,) + ro["obs"].shape[3:])
        _, _, acts, pre = orc.forward_acts(net, np.asarray(X[i], dtype=np.float64), obs, with_pre=True)
        if gates is None:
            gates = np.zeros((len(agents), M, acts.shape[1]), dtype=np.uint8)
        for name, li in layers:
            off, shape = offs[name]
            n = int(np.prod(shape))
            z = pre[:, off:off + n]
            ga = gpu_acts[name][i, :M]
            scale = np.abs(z).max()
            e = np.abs(ga - np.maximum(z, 0.0)).max() / scale
            assert e <= RTOL, f"activation {name} agent {i}: rel err {e:.3e}"
            mism = (ga > 0) != (z > 0)
            if mism.any():
                assert np.abs(z[mism]).max() <= KINK * scale, \
                    f"{name} agent {i}: ReLU decision differs away from zero (|z| = {np.abs(z[mism]).max():.3e})"
                g = gates[gi, :, off:off + n]
                g[mism & (ga > 0)] = 1
                g[mism & ~(ga > 0)] = 2
                marked += int(mism.sum())
    return gates, marked


def step_both(gpu, orc_model, ro: dict, dev: dict | None = None):
    """One learner step on both sides from the oracle's current state (which the caller has
    made equal to the GPU's).  Returns the number of ReLU units decided in the GPU's precision."""
    dev = dev or upload(ro)
    gpu.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
    gates, marked = relu_gates(gpu, orc_model.net, orc_model.X, ro)
    orc_model.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"],
                           gates=gates if marked else None)
    return marked


def compare_learner_step(gpu, orc_model, net, tag="", rtol=RTOL):
    """Gradients per tensor and agent, loss terms, norms, clip factors, parameters, RMSprop state."""
    sl = gs.segment_slices(net)
    g = gpu.get_grads()
    worst = {}
    for i in range(gpu.N):
        for name, s in sl.items():
            e = rel_err(g[i, s], orc_model.grads[i, s], grad_scale(orc_model.grads[i], sl, name))
            worst[name] = max(worst.get(name, 0.0), e)
            assert e <= rtol, f"{tag} grad {name} agent {i}: rel err {e:.3e}"
    st = gpu.get_step_stats()
    for i in range(gpu.N):
        for k, name in enumerate(("pg", "td", "entropy", "grad_norm", "clip")):
            ref = orc_model.stats[i, k]
            scale = max(abs(ref), 1e-2 if k < 2 else 1e-30)   # pg / td terms can cancel to ~0
            assert abs(st[i, k] - ref) <= rtol * scale, f"{tag} stat {name} agent {i}: {st[i, k]} vs {ref}"
    x = gpu.get_params()
    v = gpu.get_opt_state()
    for i in range(gpu.N):
        for name, s in sl.items():
            e = rel_err(x[i, s], orc_model.X[i, s])
            assert e <= rtol, f"{tag} param {name} agent {i}: rel err {e:.3e}"
            # v holds squared gradients: twice the relative error, measured like the gradient
            ev = rel_err(v[i, s], orc_model.V[i, s], grad_scale(orc_model.V[i], sl, name))
            assert ev <= 2 * rtol, f"{tag} rmsprop {name} agent {i}: rel err {ev:.3e}"
    return worst


def compare_params(gpu, orc_model, net, tag="", rtol=RTOL):
    sl = gs.segment_slices(net)
    x = gpu.get_params()
    for i in range(gpu.N):
        for name, s in sl.items():
            e = rel_err(x[i, s], orc_model.X[i, s])
            assert e <= rtol, f"{tag} param {name} agent {i}: rel err {e:.3e}"
    return x
