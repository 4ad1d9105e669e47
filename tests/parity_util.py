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


def rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / (np.abs(ref).max() + 1e-30))


def upload(ro: dict):
    import torch
    return {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in ro.items()}


def step_both(gpu, orc_model, ro: dict, dev: dict | None = None):
    dev = dev or upload(ro)
    gpu.learner_step(dev["obs"], dev["actions"], dev["rewards"], dev["dones"], dev["boot_obs"])
    orc_model.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])


def compare_learner_step(gpu, orc_model, net, tag="", rtol=RTOL):
    """Gradients per tensor and agent, loss terms, norms, clip factors, parameters, RMSprop state."""
    sl = gs.segment_slices(net)
    g = gpu.get_grads()
    worst = {}
    for i in range(gpu.N):
        for name, s in sl.items():
            e = rel_err(g[i, s], orc_model.grads[i, s])
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
            ev = rel_err(v[i, s], orc_model.V[i, s])
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
