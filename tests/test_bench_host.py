"""Host-side pieces of bench.py that need no GPU: the algorithmic work table its per-kernel fractions divide by, and the
lookup of the measured HBM traffic in the rocprofv3 summaries under profiles/."""
import importlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    sys.path.insert(0, ROOT)
    return importlib.import_module("bench")


def test_algorithmic_work_of_a_bert_base_forward():
    """C2 shapes: the GEMM operation counts are 2 T N K per layer, and the FFN1 kernel's bytes per 2048-token launch are
    the 10.22 MB the roofline object quotes (input + weights + output, once each)."""
    b = load_bench()
    import samp_workloads as W
    w = W.config("C2")
    lens = np.full(w.batch, w.seq, np.int64)
    work = b.algorithmic_work(w, w.modes, lens)
    T, H, F, L = w.batch * w.seq, w.hidden, w.ffn, w.layers
    assert work["qkv"][0] == 2.0 * T * 3 * H * H * L
    assert work["ffn1"][0] == work["ffn2"][0] == 2.0 * T * H * F * L
    assert work["attention"][0] == 4.0 * w.batch * w.seq * w.seq * H * L
    per_launch = (2048 * (H + F) + H * F)                     # int8: one byte per element
    assert abs(per_launch - 10.22e6) < 0.01e6
    assert work["ffn1"][1] == (T * (H + F) + H * F) * L        # weights once per layer, activations once
    # with the QKV GEMM and the attention in one kernel, their operations add up and the q, k, v codes are no traffic
    one = b.algorithmic_work(w, w.modes, lens, fused=True)
    assert one["qkv"] == [0.0, 0.0] and one["attention"] == [0.0, 0.0]
    assert one["qkv_attention"][0] == work["qkv"][0] + work["attention"][0]
    assert one["qkv_attention"][1] == (2 * T * H + 3 * H * H) * L
    assert one["ffn1"] == work["ffn1"] and work["qkv_attention"] == [0.0, 0.0]
    half = b.algorithmic_work(w, (0,) * L, lens, fused=True)
    assert half["qkv_attention"] == [one["qkv_attention"][0], 2 * one["qkv_attention"][1]] and half["qkv"] == [0.0, 0.0]
    # an FP16 stack moves two bytes per element in every kernel
    fp16 = b.algorithmic_work(w, (0,) * L, lens)
    assert fp16["ffn1"][1] == 2 * work["ffn1"][1] and fp16["ln1"][1] == 2 * work["ln1"][1]


def test_measured_traffic_comes_from_the_tracked_profiles():
    b = load_bench()
    got = b.measured_traffic("C2", "FULL_INT8", "ffn1", 2048)
    assert got is not None and 10.22e6 < got < 60e6            # at least the algorithmic bytes, the same order of magnitude
    assert b.measured_traffic("C2", "FULL_INT8", "ffn1", 4096) is None      # another launch size: no figure, no guess
    assert b.measured_traffic("C9", "FULL_INT8", "ffn1", 2048) is None


def test_more_than_one_gpu_is_refused_with_a_message():
    """Everything here runs on one GPU: bench.py --gpus 2 exits with a message that says so, before touching any GPU."""
    import subprocess
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr and r.stdout.strip() == ""
