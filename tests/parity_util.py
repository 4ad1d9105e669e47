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
# The three loss terms are means of per-sample quantities of order one (log-probabilities times
# advantages, squared TD errors, entropies up to ln A) that single precision carries to ~1e-7
# absolute.  The policy term cancels between samples and the entropy of a nearly deterministic
# policy is itself ~1e-5, so their errors are measured against max(|term|, 1e-2) (and the policy
# term against the magnitude it is made of, pg_scale): an absolute floor of 1e-6.


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


# The hidden layer's fp32 activations agree with exact arithmetic to about 1e-6 of their largest
# value; measured against the tolerance of 1e-4 that is this fraction of a sum's term magnitude.
TERM_FRACTION = 1e-2


def loss_conditioning(net, hp, x, ro: dict, i: int):
    """(pg_scale, kappa, rho_v) of agent i from an oracle forward pass.

    pg_scale = mean |log pi(a_m | s_m) * A_m|: the magnitude the policy term is made of.  The term
    itself, mean(-log pi * A), is a sum of signed products that can cancel to a small fraction of
    this, so its absolute error is measured against it (never against less than the term).

    kappa = max(1, max |G| / max |A|): how much the advantage A = G - V cancels.  V and G carry
    the relative error of the fp32 network (a few 1e-6) times their own size, so A carries that
    error times kappa, and every gradient is linear in A (policy term) or in G - V (value term).
    At initialisation kappa is about 1; after many updates on random rewards the values grow
    into the hundreds while advantages stay of order one, and the gradients cannot agree with
    the oracle better than kappa times the usual error.  Gradient tolerances are scaled by it.

    rho_v = max_j sum_f |A_f| h_fj / max_j |sum_f A_f h_fj|: how much the value head's weight
    gradient, a sum over frames of advantages of both signs times the hidden activations, cancels.
    Once the value regression has converged on an agent's data this gradient sits near a
    stationary point and is hundreds to thousands of times smaller than its terms, while its
    absolute error stays that of the terms (about 1e-6 of them).  The value head's two tensors
    are therefore measured against max(own size, TERM_FRACTION * term magnitude)."""
    from oracle import gala_oracle as orc
    T, B = ro["actions"].shape[1:3]
    M = T * B
    frames = np.concatenate([ro["obs"][i].reshape((M,) + ro["obs"].shape[3:]), ro["boot_obs"][i]], axis=0)
    logits, values, acts = orc.forward_acts(net, np.asarray(x, dtype=np.float64), frames)
    off, shape = orc.act_offsets(net)["fc"]
    h = acts[:M, off:off + shape[0]]
    G, adv = orc.nstep_returns(ro["rewards"][i], ro["dones"][i], values[M:], values[:M].reshape(T, B), hp["gamma"])
    z = logits[:M]
    logp = z - z.max(1, keepdims=True)
    logp = logp - np.log(np.exp(logp).sum(1, keepdims=True))
    la = logp[np.arange(M), ro["actions"][i].reshape(M)]
    kappa = max(1.0, float(np.abs(G).max() / max(np.abs(adv).max(), 1e-30)))
    a = adv.reshape(M, 1)
    rho_v = float((np.abs(a) * h).sum(0).max() / max(np.abs((a * h).sum(0)).max(), 1e-300))
    return float(np.abs(la * adv.reshape(M)).mean()), kappa, rho_v


def pg_scale(net, hp, x, ro: dict, i: int) -> float:
    return loss_conditioning(net, hp, x, ro, i)[0]


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
    # decisions taken in the kernel's precision must stay the rare exception they are meant to be: a handful
    # (2 to 10 of 55 to 220 million in the full-size configurations) of the N * M * 21 632 units of a round (a kernel that rounded systematically differently would mark many)
    total = len(agents) * M * (gates.shape[2] if gates is not None else 1)
    assert marked <= max(64, 2e-5 * total), f"{marked} of {total} ReLU units decided in the kernel's precision"
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


def compare_learner_step(gpu, orc_model, net, tag="", rtol=RTOL, ro=None, X_before=None, max_cond=None, plain=False):
    """Gradients per tensor and agent, loss terms, norms, clip factors, parameters, RMSprop state.

    With the rollout and the pre-step parameters the policy term is measured against pg_scale and the
    conditioning factors kappa (all gradients) and max(1, TERM_FRACTION * rho_v) (value head) widen the
    gradient tolerances; without them every tensor is held to the plain rtol.  Returns the worst
    error per tensor (already divided by the factor applied) under the tensor's name, and the largest
    factors applied under "kappa" and "rho_v_factor"; both are printed.  max_cond, when given, is an
    upper bound both factors must respect: a round started from freshly initialised parameters passes
    it as 2, so that such a round demonstrably passes at (about) the plain rtol.  plain=True computes
    the factors (they are printed and returned) but applies none: every tensor is held to rtol itself
    and only the policy term keeps its pg_scale."""
    sl = gs.segment_slices(net)
    g = gpu.get_grads()
    worst = {}
    cond = [loss_conditioning(net, orc_model.hp, X_before[i], ro, i) if ro is not None else (0.0, 1.0, 1.0)
            for i in range(gpu.N)]
    kappa_max = max(c[1] for c in cond)
    rho_factor_max = max(max(1.0, TERM_FRACTION * c[2]) for c in cond)
    if plain:
        print(f"{tag}: plain tolerance (conditioning factors kappa {kappa_max:.3f}, value head {rho_factor_max:.3f} "
              f"computed, not applied)", flush=True)
        cond = [(c[0], 1.0, 1.0) for c in cond]
    else:
        print(f"{tag}: " + ("plain tolerance, no conditioning factors" if ro is None else
                            f"largest conditioning factors applied: kappa {kappa_max:.3f}, value head {rho_factor_max:.3f}"),
              flush=True)
    if max_cond is not None:
        assert kappa_max <= max_cond and rho_factor_max <= max_cond, \
            f"{tag}: conditioning factors kappa {kappa_max:.2f}, value head {rho_factor_max:.2f} exceed {max_cond}"
    for i in range(gpu.N):
        for name, s in sl.items():
            scale = grad_scale(orc_model.grads[i], sl, name)
            if name.startswith("v."):
                scale *= max(1.0, TERM_FRACTION * cond[i][2])
            e = rel_err(g[i, s], orc_model.grads[i, s], scale)
            worst[name] = max(worst.get(name, 0.0), e / cond[i][1])
            assert e <= rtol * cond[i][1], f"{tag} grad {name} agent {i}: rel err {e:.3e} (kappa {cond[i][1]:.1f})"
    st = gpu.get_step_stats()
    for i in range(gpu.N):
        for k, name in enumerate(("pg", "td", "entropy", "grad_norm", "clip")):
            ref = orc_model.stats[i, k]
            scale = max(abs(ref), 1e-2 if k < 3 else 1e-30)   # loss terms: absolute floor, see the module comment
            if k == 0:
                scale = max(scale, cond[i][0])
            if k >= 3:
                scale *= cond[i][1]                       # norm and clip factor of a gradient that carries kappa
            assert abs(st[i, k] - ref) <= rtol * scale, f"{tag} stat {name} agent {i}: {st[i, k]} vs {ref}"
    x = gpu.get_params()
    v = gpu.get_opt_state()
    for i in range(gpu.N):
        for name, s in sl.items():
            e = rel_err(x[i, s], orc_model.X[i, s])
            assert e <= rtol, f"{tag} param {name} agent {i}: rel err {e:.3e}"
            # v holds squared gradients: twice the relative error, measured like the gradient
            ev = rel_err(v[i, s], orc_model.V[i, s], grad_scale(orc_model.V[i], sl, name))
            assert ev <= 2 * rtol * cond[i][1], f"{tag} rmsprop {name} agent {i}: rel err {ev:.3e}"
    worst["kappa"] = kappa_max
    worst["rho_v_factor"] = rho_factor_max
    return worst


def compare_params(gpu, orc_model, net, tag="", rtol=RTOL):
    sl = gs.segment_slices(net)
    x = gpu.get_params()
    for i in range(gpu.N):
        for name, s in sl.items():
            e = rel_err(x[i, s], orc_model.X[i, s])
            assert e <= rtol, f"{tag} param {name} agent {i}: rel err {e:.3e}"
    return x
