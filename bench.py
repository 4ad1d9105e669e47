#!/usr/bin/env python3
"""Throughput of the GALA-A2C hot path on one MI355X.

A step is one round of Algorithm 1 for all agents: returns, A2C loss, forward/backward,
clip and RMSprop for every agent, then one mixing iteration over the 1-peer exponential
graph.  --mode fused (default) issues it as one gala_round call, whose optimizer and mixing
step share a kernel; --mode split as gala_learner_step followed by gala_gossip; both
compute the same values bit for bit.  Inputs are synthetic
Atari-shaped rollouts that are resident in HBM before the timed region starts; a
pool of four rollouts is cycled.  One JSON line is printed on stdout.

The 32-agent workload (--config 4, the default) runs 1000 timed rounds and then a second pass of
the same length in which the distance from consensus (Prop. 1) is taken after every round by
gala_consensus_distance_noalloc into a device-side log (no host round trip inside the loop); the
per-round values go to consensus_distance_cfg4.csv in the output directory (--out-dir) and their
first/last/largest values and the cost of logging to the JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MACs per frame of each layer (unpadded 8x8/4, 4x4/2, 3x3/1 convolutions on 4x84x84, 512 hidden)
MACS = dict(conv1=3_276_800, conv2=2_654_208, conv3=1_806_336, fc=1_605_632)
PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # dense matrix-instruction peaks of MI355X
PEAK_HBM_GBS = 8000.0

# event-timed phase -> kernel name in the rocprofv3 summaries under profiles/
# phases whose kernels reach fp32 accuracy with bf16 matrix instructions on exact bf16 pieces of the
# operands: pieces multiplied per algorithmic product
SPLIT_PRODUCTS = {"conv1_fwd": 3, "conv1_wgrad": 3, "conv2_fwd": 6, "conv3_fwd": 6, "fc_fwd": 6,
                  "fc_dgrad": 6, "fc_wgrad": 6, "conv3_dgrad": 6, "conv3_wgrad": 6, "conv2_wgrad": 6, "conv2_dgrad": 6}


def kernel_of_phase(dtype: str) -> dict:
    """Event-timed phase -> kernel name as the rocprofv3 summaries under profiles/ print it.  The last
    template argument is the MFMA mode: 0 = fp32, 1 = bf16 operands, 2 = byte operand exact in bf16 and
    the fp32 operand as three bf16 pieces (the first convolution in an fp32 run), 3 = both operands as
    three bf16 pieces, six piece products."""
    def mode(phase):
        if dtype != "f32":
            return "1"
        return {3: "2", 6: "3"}.get(SPLIT_PRODUCTS.get(phase, 0), "0")
    names = {
        "conv1_fwd": "Conv1Fwd", "conv2_fwd": "ConvFwd<32, 20, 20, 64, 9, 9, 4, 2>",
        "conv3_fwd": "ConvFwd<64, 9, 9, 64, 7, 7, 3, 1>", "fc_fwd": "FcFwdT<96>", "fc_wgrad": "FcWgrad",
        "fc_dgrad": "FcDgrad", "conv3_wgrad": "ConvWgrad<64, 9, 9, 64, 7, 7, 3, 1, 64>",
        "conv3_dgrad": "Conv3Dgrad", "conv2_wgrad": "ConvWgrad<32, 20, 20, 64, 9, 9, 4, 2, 128>",
        "conv2_dgrad": "Conv2Dgrad", "conv1_wgrad": "Conv1Wgrad",
    }
    out = {ph: f"igemm_kernel<{nm}, {mode(ph)}>" for ph, nm in names.items()}
    out.update({
        "conv1_wgrad_reduce": "reduce_grads_kernel", "step_stats": "step_stats_kernel", "clip_rmsprop": "rmsprop_kernel", "gossip_mix": "mix_kernel",
        # one in-peer per agent and no delays (the only workload with a committed traffic summary): the
        # cycle-walking pass; with delays or several in-peers the same phase runs rmsprop_mix_kernel<..>
        "gossip_publish": "copy_kernel", "clip_rmsprop_mix": "rmsprop_mix_cycle_kernel",
    })
    return out


TRAFFIC_SUMMARY = os.path.join("profiles", "hbm_traffic_n32_exp_5x16_fp32.txt")


def measured_traffic(phase: str, config: int, dtype: str):
    """HBM bytes per launch of the kernel behind `phase` from the committed FETCH_SIZE / WRITE_SIZE
    summary (counters are not read in this run), or None when there is none for this workload or the
    kernel sources changed since."""
    import glob
    import hashlib
    path = os.path.join(ROOT, TRAFFIC_SUMMARY)
    if config != 4 or dtype != "f32" or not os.path.exists(path):
        return None
    rec = None
    for line in open(path):
        if line.startswith("JSON "):
            rec = json.loads(line[5:])
    if rec is None:
        return None
    sha = hashlib.sha256()
    for fn in sorted(glob.glob(os.path.join(ROOT, "paper_1906_04585_amd", "csrc", "*.h*"))):
        sha.update(open(fn, "rb").read())
    if sha.hexdigest() != rec["source_sha256"]:
        return None
    k = rec["kernels"].get(kernel_of_phase(dtype).get(phase, ""))
    return k["bytes"] if k else None


def kernel_work(N: int, M: int, F: int, d: int, tau: int, dtype: str) -> dict:
    """Algorithmic work of one launch of each kernel: ('mfma', flop), ('split', flop, n) or ('hbm', bytes).
    'split': in an fp32 run these kernels cut their operands into exact bf16 pieces and execute n bf16
    piece products per algorithmic product (3 where one operand is a byte image, which bf16 holds
    exactly; 6 otherwise).  They are priced against the bf16 matrix peak with n x the algorithmic flops."""
    w = {}
    for layer, macs in MACS.items():
        for kind, frames in (("fwd", F), ("wgrad", M), ("dgrad", M)):
            if layer == "conv1" and kind == "dgrad":         # the input needs no gradient
                continue
            ph = f"{layer}_{kind}"
            flop = 2.0 * macs * frames * N
            w[ph] = ("split", flop, SPLIT_PRODUCTS[ph]) if (dtype == "f32" and ph in SPLIT_PRODUCTS) else ("mfma", flop)
    # the gradient norm is assembled from partial sums the weight-gradient kernels emit: no pass over g
    w["clip_rmsprop"] = ("hbm", 20.0 * d * N)    # read g, x, v; write x, v
    w["gossip_mix"] = ("hbm", 12.0 * d * N)      # read x_i, x_j; write x_i
    if tau > 0:
        w["gossip_publish"] = ("hbm", 8.0 * d * N)
    # fused: read g, x, v; write v, x (+ write the history slot and read stale messages with delays)
    w["clip_rmsprop_mix"] = ("hbm", (20.0 + (8.0 if tau > 0 else 0.0)) * d * N)
    return w


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed rounds (default: 1000 for the 32-agent workload, 300 otherwise)")
    ap.add_argument("--consensus-log", choices=["auto", "on", "off"], default="auto",
                    help="second pass of --steps rounds with the distance from consensus taken every round "
                         "(auto: on for --config 4 in the fused or split mode)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--out-dir", default="gpurun_out", help="where the per-round consensus log is written (relative to the repository)")
    ap.add_argument("--config", type=int, default=4, help="workload shape 1..5 (default: 32 agents)")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32",
                    help="matrix-instruction operand type of the conv/fc kernels (parameters stay fp32)")
    ap.add_argument("--mode", choices=["fused", "split", "a2c_allreduce"], default="fused",
                    help="one gala_round call per step, or gala_learner_step + gala_gossip; a2c_allreduce times "
                         "the synchronous comparator (gradients averaged over agents, no gossip) instead")
    ap.add_argument("--extras", choices=["on", "off"], default="on",
                    help="off: skip the acting and diagnostics measurements (profiling runs of the headline path)")
    ap.add_argument("--overlap-optimizer", action="store_true",
                    help="create the context with GALA_OVERLAP_OPTIMIZER set: the hidden layer's share of the fused "
                         "optimizer + mixing pass runs on the library's side stream beside the next round's convolutions")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-rounds", type=int, default=20)
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 1000 if args.config == 4 else 300
    if args.gpus != 1:
        print("bench.py measures one GPU: N agents share a single MI355X and nothing here "
              "uses a second device; run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import gala_synth as gs
    from paper_1906_04585_amd import Gala

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    cfg = gs.CONFIGS[args.config]
    N, A, T, B = cfg["n_agents"], cfg["n_actions"], cfg["T"], cfg["B"]
    M, F = T * B, T * B + B
    net = gs.make_net(A)
    hparams = dict(gs.HPARAMS, compute_dtype=1 if args.dtype == "bf16" else 0)
    peak_mfma = PEAK_MFMA_TFLOPS[args.dtype]
    if args.overlap_optimizer:
        os.environ["GALA_OVERLAP_OPTIMIZER"] = "1"
    gpu = Gala(N, A, T, B, hparams, cfg["topology"], max_delay=cfg["max_delay"], delay_seed=7)
    X0 = gs.init_params(net, N, shared=True)
    gpu.set_params(X0)
    pool = []
    for r in range(4):
        ro = gs.rollout(net, N, T, B, gs.round_seed(args.config, r))
        pool.append({k: torch.from_numpy(v).cuda() for k, v in ro.items()})
    torch.cuda.synchronize()

    def one_round(r, actions=None):
        d = pool[r % len(pool)]
        acts = d["actions"] if actions is None else actions
        if args.mode == "fused":
            gpu.round(d["obs"], acts, d["rewards"], d["dones"], d["boot_obs"], r)
        elif args.mode == "a2c_allreduce":
            gpu.a2c_allreduce_step(d["obs"], acts, d["rewards"], d["dones"], d["boot_obs"])
        else:
            gpu.learner_step(d["obs"], acts, d["rewards"], d["dones"], d["boot_obs"])
            gpu.gossip(r)

    rnd = 0
    for _ in range(args.warmup):
        one_round(rnd)
        rnd += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_round(rnd)
        rnd += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    agent_steps = N * args.steps / elapsed
    frames = agent_steps * M

    # Second pass of the same length with the distance from consensus logged after every round
    # (Prop. 1; max_i ||x_i - mean|| and the Frobenius norm), into a device buffer in stream order.
    consensus = None
    want_log = args.consensus_log == "on" or (args.consensus_log == "auto" and args.config == 4
                                             and args.mode != "a2c_allreduce")
    if want_log:
        log = torch.zeros((args.steps, 2), dtype=torch.float32, device="cuda")
        first_round = rnd
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            one_round(rnd)
            gpu.consensus_distance_noalloc(log[i])
            rnd += 1
        torch.cuda.synchronize()
        logged_ms = 1e3 * (time.perf_counter() - t0) / args.steps
        vals = log.cpu().numpy()
        out_dir = os.path.join(ROOT, args.out_dir)
        os.makedirs(out_dir, exist_ok=True)
        csv = os.path.join(out_dir, f"consensus_distance_cfg{args.config}.csv")
        with open(csv, "w") as fh:
            fh.write("round,max_row_distance,frobenius\n")
            for i in range(args.steps):
                fh.write(f"{first_round + i},{vals[i, 0]:.9g},{vals[i, 1]:.9g}\n")
        consensus = dict(call="gala_consensus_distance_noalloc after every round", rounds=args.steps,
                         first_round=first_round, file=os.path.relpath(csv, ROOT),
                         max_row_distance=dict(first=float(vals[0, 0]), last=float(vals[-1, 0]),
                                               largest=float(vals[:, 0].max()), smallest=float(vals[:, 0].min())),
                         frobenius=dict(first=float(vals[0, 1]), last=float(vals[-1, 1]),
                                        largest=float(vals[:, 1].max()), smallest=float(vals[:, 1].min())),
                         ms_per_step_with_logging=logged_ms,
                         logging_overhead_ms=logged_ms - ms_per_step,
                         logging_overhead_frac=(logged_ms - ms_per_step) / ms_per_step,
                         note="agents start from identical parameters (distance 0 before the first round) and see "
                              "different synthetic rollouts; rounds continue the timed pass's count")

    # per-kernel durations from HIP events recorded on the library's stream
    gpu.set_profiling(True)
    acc: dict[str, float] = {}
    for _ in range(args.profile_rounds):
        one_round(rnd)
        rnd += 1
        for k, v in gpu.get_phase_times().items():
            acc[k] = acc.get(k, 0.0) + v / args.profile_rounds
    gpu.set_profiling(False)
    work = kernel_work(N, M, F, gpu.d, cfg["max_delay"], args.dtype)
    if args.mode == "a2c_allreduce":
        work["grad_mean_norm"] = ("hbm", 4.0 * gpu.d * N)      # read every agent's gradient once
        work["clip_rmsprop"] = ("hbm", 16.0 * gpu.d * N)       # read x, v; write x, v (the mean stays in cache)
    kernels = {}
    for k, ms in acc.items():
        ent = {"ms": round(ms, 5)}
        if k in work:
            kind, amount = work[k][0], work[k][1]
            if kind == "mfma":
                ent.update(bound="mfma", achieved=round(amount / (ms * 1e-3) / 1e12, 2), unit="TFLOP/s",
                           frac=round(amount / (ms * 1e-3) / 1e12 / peak_mfma, 4))
            elif kind == "split":
                n = work[k][2]
                ent.update(bound="mfma", dtype=f"bf16 pieces, {n} products (fp32-exact)",
                           algorithmic_tflops=round(amount / (ms * 1e-3) / 1e12, 2),
                           achieved=round(n * amount / (ms * 1e-3) / 1e12, 2), unit="TFLOP/s",
                           frac=round(n * amount / (ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS["bf16"], 4))
            else:
                ent.update(bound="hbm", achieved=round(amount / (ms * 1e-3) / 1e9, 1), unit="GB/s",
                           frac=round(amount / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4))
        kernels[k] = ent
    dominant = max((k for k in acc if k in work), key=lambda k: acc[k])
    kind, amount = work[dominant][0], work[dominant][1]
    dur = acc[dominant] * 1e-3
    if kind in ("mfma", "split"):
        mult, pk = (float(work[dominant][2]), PEAK_MFMA_TFLOPS["bf16"]) if kind == "split" else (1.0, peak_mfma)
        roofline = dict(kernel=dominant, bound="mfma", achieved=mult * amount / dur / 1e12, peak=pk,
                        unit="TFLOP/s", frac=mult * amount / dur / 1e12 / pk,
                        traffic=measured_traffic(dominant, args.config, args.dtype), avg_launch_ms=acc[dominant])
    else:
        roofline = dict(kernel=dominant, bound="hbm", achieved=amount / dur / 1e9, peak=PEAK_HBM_GBS,
                        unit="GB/s", frac=amount / dur / 1e9 / PEAK_HBM_GBS,
                        traffic=measured_traffic(dominant, args.config, args.dtype), avg_launch_ms=acc[dominant])
    roofline["traffic_source"] = (f"{TRAFFIC_SUMMARY} (rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                  f"workload on these kernel sources; not measured in this run)"
                                  if roofline["traffic"] is not None else None)
    mfma_ms = sum(acc[k] for k in acc if k in work and work[k][0] == "mfma")
    mfma_flop = sum(work[k][1] for k in acc if k in work and work[k][0] == "mfma")
    m3_ms = sum(acc[k] for k in acc if k in work and work[k][0] == "split")
    m3_flop = sum(work[k][1] for k in acc if k in work and work[k][0] == "split")
    m3_exec = sum(work[k][1] * work[k][2] for k in acc if k in work and work[k][0] == "split")
    hbm_ms = sum(acc[k] for k in acc if k in work and work[k][0] == "hbm")
    hbm_bytes = sum(work[k][1] for k in acc if k in work and work[k][0] == "hbm")
    phase_summary = dict(
        optimizer_gossip=dict(ms=round(hbm_ms, 4), gbs=round(hbm_bytes / (hbm_ms * 1e-3) / 1e9, 1),
                              frac_hbm=round(hbm_bytes / (hbm_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)),
        other_ms=round(sum(acc.values()) - mfma_ms - m3_ms - hbm_ms, 4))
    if mfma_ms > 0:
        # the conv/fc kernels that run plain matrix instructions of the run's dtype (in an fp32 run: the few
        # kernels left on fp32 MFMAs; in a bf16 run: all of them)
        phase_summary["fp32_mfma_kernels" if args.dtype == "f32" else "bf16_mfma_kernels"] = dict(
            ms=round(mfma_ms, 4), tflops=round(mfma_flop / (mfma_ms * 1e-3) / 1e12, 2),
            frac_mfma=round(mfma_flop / (mfma_ms * 1e-3) / 1e12 / peak_mfma, 4))
    conv_fc_ms, conv_fc_flop = mfma_ms + m3_ms, mfma_flop + m3_flop
    conv_fc_exec = mfma_flop + m3_exec
    if m3_ms > 0:
        # kernels on bf16 pieces: algorithmic (fp32-equivalent) rate and the rate of the bf16 matrix work they
        # execute; then all conv/fc kernels together
        phase_summary["conv_fc_bf16_pieces"] = dict(
            ms=round(m3_ms, 4), algorithmic_tflops=round(m3_flop / (m3_ms * 1e-3) / 1e12, 2),
            executed_bf16_tflops=round(m3_exec / (m3_ms * 1e-3) / 1e12, 2),
            frac_of_bf16_mfma_peak=round(m3_exec / (m3_ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS["bf16"], 4))
    # the whole conv/fc phase (every contraction kernel of the round, forward and backward)
    all_tf = conv_fc_flop / (conv_fc_ms * 1e-3) / 1e12
    phase_summary["conv_fc"] = dict(ms=round(conv_fc_ms, 4), algorithmic_tflops=round(all_tf, 2))
    if args.dtype == "f32":
        phase_summary["conv_fc"].update(
            frac_of_fp32_mfma_peak=round(all_tf / PEAK_MFMA_TFLOPS["f32"], 4),
            note="algorithmic flops against the fp32 matrix peak; most kernels execute them as 3 or 6 exact bf16 piece "
                 "products on the bf16 matrix pipe, see conv_fc_bf16_pieces for the executed rate against that pipe's peak")
    else:
        phase_summary["conv_fc"]["frac_of_bf16_mfma_peak"] = round(all_tf / PEAK_MFMA_TFLOPS["bf16"], 4)
    # beside the top-level `roofline` (the single longest kernel of the round): the phase that takes most of it
    roofline_conv_fc = dict(
        phase="conv_fc (all contraction kernels of the round)", bound="mfma", ms=conv_fc_ms,
        share_of_round=conv_fc_ms / sum(acc.values()), algorithmic_tflops=all_tf,
        frac_of_fp32_mfma_peak=all_tf / PEAK_MFMA_TFLOPS["f32"] if args.dtype == "f32" else None,
        executed_tflops=conv_fc_exec / (conv_fc_ms * 1e-3) / 1e12,
        frac_of_bf16_mfma_peak=(m3_exec / (m3_ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS["bf16"]) if m3_ms > 0 else
                               (all_tf / PEAK_MFMA_TFLOPS["bf16"] if args.dtype == "bf16" else None),
        unit="TFLOP/s")

    acting = diagnostics = None
    if args.extras == "on":
        # acting step of Algorithm 1 (policy forward + categorical draw for every agent's B simulators);
        # reported beside the learner-side metric, not part of `value`
        act_out = torch.empty((N, B), dtype=torch.int32, device="cuda")
        val_out = torch.empty((N, B), dtype=torch.float32, device="cuda")
        for s_ in range(10):
            gpu.act(pool[0]["boot_obs"], 1, s_, act_out, val_out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_act = 200
        for s_ in range(n_act):
            gpu.act(pool[s_ % len(pool)]["boot_obs"], 1, 10 + s_, act_out, val_out)
        torch.cuda.synchronize()
        act_s = (time.perf_counter() - t0) / n_act
        # One iteration of Algorithm 1 as a loop: T acting steps whose drawn actions become the
        # rollout's actions, then the learner step and the gossip round.  States, rewards and
        # episode ends stay synthetic (there is no simulator), so this times the GPU side of an
        # actor-learner iteration, not a training run.
        acts_buf = pool[0]["actions"].clone()

        def actor_learner_iteration(r, step0):
            d = pool[r % len(pool)]
            for t in range(T):
                gpu.act(d["boot_obs"], 1, step0 + t, act_out, val_out)
                acts_buf[:, t].copy_(act_out)
            one_round(r, acts_buf)

        step_ctr = 1000
        for _ in range(5):
            actor_learner_iteration(rnd, step_ctr)
            rnd += 1
            step_ctr += T
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_it = 100
        for _ in range(n_it):
            actor_learner_iteration(rnd, step_ctr)
            rnd += 1
            step_ctr += T
        torch.cuda.synchronize()
        it_s = (time.perf_counter() - t0) / n_it
        acting = dict(call="gala_act", us_per_call=round(act_s * 1e6, 1), frames_per_call=N * B,
                      frames_per_s=round(N * B / act_s, 1),
                      actor_learner_iteration_ms=round(it_s * 1e3, 4),
                      actor_learner_frames_per_s=round(N * T * B / it_s, 1),
                      note=f"an actor-learner iteration = {T} acting steps (policy forward + draw; the drawn actions "
                           f"are the rollout's actions) + 1 learner/gossip step, measured as one loop; states, "
                           f"rewards and episode ends synthetic")

        # diagnostics of Sec. 5 (gradient cosine matrix, update norm, consensus distance): event-timed per call
        gpu.set_profiling(True)
        dacc: dict[str, float] = {}
        n_diag = 10
        for _ in range(n_diag):
            one_round(rnd)
            rnd += 1
            gpu.grad_cosine()
            gpu.update_norm()
            gpu.consensus_distance()
            for k, v in gpu.get_phase_times().items():
                if k in ("grad_cosine", "update_norm", "consensus_distance"):
                    dacc[k] = dacc.get(k, 0.0) + v / n_diag
        gpu.set_profiling(False)
        # algorithmic bytes: every gradient (parameter) read once; update norm reads g and v
        diag_bytes = {"grad_cosine": 4.0 * gpu.d * N, "update_norm": 8.0 * gpu.d * N, "consensus_distance": 4.0 * gpu.d * N}
        diagnostics = {k: dict(ms=round(ms, 5), bound="hbm", achieved=round(diag_bytes[k] / (ms * 1e-3) / 1e9, 1),
                               unit="GB/s", frac=round(diag_bytes[k] / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4))
                       for k, ms in dacc.items()}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import gala_oracle as orc
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        n_s, n_r = min(N, 32), 2               # a bounded sample: two rounds of (up to) 32 agents
        om = orc.OracleGala(net, n_s, T, B, gs.HPARAMS, cfg["topology"])
        om.set_params(X0[:n_s])
        ros = [gs.rollout(net, n_s, T, B, gs.round_seed(args.config, r)) for r in range(n_r)]
        t0 = time.perf_counter()
        for r, ro in enumerate(ros):
            om.learner_step(ro["obs"], ro["actions"], ro["rewards"], ro["dones"], ro["boot_obs"])
            om.gossip(r)
        cpu_t = time.perf_counter() - t0
        cpu_baseline = dict(value=n_s * n_r / cpu_t, unit="agent-steps/s", cores=threads, kind="oracle",
                            sample=f"{n_r} rounds (learner step + gossip) of {n_s} of the {N} agents, "
                                   f"{n_s * n_r * M} frames, fp64, {cpu_t:.2f} s wall on {threads} threads")
        # the same oracle on one thread (one round of two agents), through the OpenMP runtime's own switch
        try:
            import ctypes
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            n1 = min(N, 2)
            om1 = orc.OracleGala(net, n1, T, B, gs.HPARAMS, "ring")
            om1.set_params(X0[:n1])
            ro1 = {k: v[:n1] for k, v in ros[0].items()}
            t0 = time.perf_counter()
            om1.learner_step(ro1["obs"], ro1["actions"], ro1["rewards"], ro1["dones"], ro1["boot_obs"])
            om1.gossip(0)
            t1 = time.perf_counter() - t0
            gomp.omp_set_num_threads(threads)
            cpu_baseline["single_thread"] = dict(value=n1 / t1, unit="agent-steps/s",
                                                 sample=f"1 round of {n1} agents, {t1:.2f} s wall on 1 thread")
        except OSError:
            pass

    out = {
        "metric": "agent learner-steps/sec (one learner step + one gossip round per agent)"
                  if args.mode != "a2c_allreduce" else "agent learner-steps/sec (synchronous A2C, gradients averaged)",
        "value": agent_steps,
        "unit": "agent-steps/s",
        "env_frames_per_s": frames,
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "arithmetic": ("fp32 parameters, activations and accumulators; products on fp32 matrix instructions or, "
                       "equally accurate, on bf16 matrix instructions over exact bf16 pieces of the fp32 operands "
                       "(see kernels[*].dtype)") if args.dtype == "f32" else
                      "fp32 parameters, activations and accumulators; operands rounded to bf16 for the matrix instructions",
        "data": "synthetic",
        "config": {"workload": f"N={N} agents, 1-peer {cfg['topology']} graph, Nature-CNN, {A} actions, "
                               f"rollout {T}x{B} per agent ({N * M} frames/round), "
                               f"{'fp32' if args.dtype == 'f32' else 'bf16 operands / fp32 accumulation'}",
                   "n_agents": N, "T": T, "B": B, "n_actions": A, "topology": cfg["topology"],
                   "max_delay": cfg["max_delay"],
                   "overlap_optimizer": bool(args.overlap_optimizer),
                   "calls": {"fused": "gala_round", "split": "gala_learner_step + gala_gossip",
                             "a2c_allreduce": "gala_a2c_allreduce_step (comparator, not GALA)"}[args.mode]},
        "roofline": roofline,
        "roofline_conv_fc": roofline_conv_fc,
        "consensus_distance": consensus,
        "phases": phase_summary,
        "kernels": kernels,
        "acting": acting,
        "diagnostics": diagnostics,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
