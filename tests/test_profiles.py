"""Consistency of the committed rocprofv3 summaries with bench.py: every kernel bench.py attributes a
phase to is present in the kernel-trace summary, and the traffic summary carries the hash of the
kernel sources it was measured on (bench.py reports measured traffic only while that hash matches)."""
import glob
import hashlib
import json
import os

import pytest

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_phase_kernel_appears_in_the_kernel_trace_summary():
    text = open(os.path.join(ROOT, "profiles", "all_kernels_n32_exp_5x16_fp32.txt")).read()
    for phase, kernel in bench.kernel_of_phase("f32").items():
        if phase in ("clip_rmsprop", "gossip_mix", "gossip_publish"):      # two-call path: not in the fused round
            continue
        assert kernel in text, f"{phase}: {kernel} missing from the kernel-trace summary"


def test_traffic_summary_matches_the_algorithmic_bytes_of_the_fused_pass():
    path = os.path.join(ROOT, "profiles", "hbm_traffic_n32_exp_5x16_fp32.txt")
    rec = [json.loads(l[5:]) for l in open(path) if l.startswith("JSON ")][-1]
    sha = hashlib.sha256()
    for fn in sorted(glob.glob(os.path.join(ROOT, "paper_1906_04585_amd", "csrc", "*.h*"))):
        sha.update(open(fn, "rb").read())
    if rec["source_sha256"] != sha.hexdigest():
        pytest.skip("kernel sources changed after the traffic counters were taken: bench.py reports traffic as null")
    fused = rec["kernels"][bench.kernel_of_phase("f32")["clip_rmsprop_mix"]]
    # read g, x, v and write x, v of 32 agents: 20 bytes per parameter, within 2 %
    d_pad = 1694208
    assert abs(fused["bytes"] / (20.0 * d_pad * 32) - 1.0) < 0.02
