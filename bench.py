#!/usr/bin/env python3
"""Benchmark of the mixed-precision encoder on one MI355X.

Workload: BERT-base 12-layer encoder, batch 32 x 128 tokens, all sequences full length (synthetic
N(0,0.02) weights, N(0,1) inputs, min-max calibration on a seeded 8x128 batch run on the GPU).
A step is one forward of the whole encoder, inputs resident in HBM.  The headline `value` is
sequences/s of the full-INT8 stack; the other precision modes are timed the same way and reported
under "modes".  Every figure is the median of --repeats timed runs of --steps forwards each.

Extra objects on the JSON line:
  roofline       - the FFN1 INT8 GEMM (+bias+GELU+quantise) kernel: algorithmic ops per launch
                   (2 * tokens * ffn * hidden) over its mean launch duration, measured with HIP events
                   attached to the dispatches over a repeat of the timed steps, against the int8 MFMA
                   dense peak; `traffic` is the measured HBM bytes per launch, read from the rocprofv3
                   summary under profiles/ that covers this workload, mode and launch size (null if none).
  kernels        - every kernel class of the headline mode timed the same way (one class per pass,
                   launches isolated): mean launch duration, and its algorithmic ops or bytes over
                   that duration against the MFMA or HBM peak.  kernels_fp16: the same for the FP16 mode
                   against the fp16 MFMA peak.
  modes          - per precision mode: median ms per forward with graph replay (the default) and with
                   plain launches, sequences/s.
  peaks_measured - what this GPU delivers in the library's probes: int8 and fp16 matrix-instruction
                   issue rate with constant and with pseudo-random operands, device copy rate.
  cpu_baseline   - the CPU oracle (as it stands, OpenMP over sequences) on the same batch.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0        # MI355X dense int8 MFMA, published: 5.0 POP/s
FP16_PEAK_TFLOPS = 2500.0      # dense fp16
HBM_PEAK_GBS = 8000.0


def measured_traffic(workload: str, mode: str, kernel: str, tokens_per_launch: int):
    """HBM bytes per launch from the rocprofv3 counter summaries under profiles/ (lines of the form
    `traffic_bytes_per_launch <workload> <mode> <kernel> <tokens per launch> <bytes>`), or None."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    for name in sorted(os.listdir(pdir)):
        if not name.endswith((".txt", ".md")):
            continue
        for line in open(os.path.join(pdir, name), errors="replace"):
            m = re.match(r"\s*#?\s*traffic_bytes_per_launch\s+(\S+)\s+(\S+)\s+(\S+)\s+(\d+)\s+([0-9.eE+]+)", line)
            if m and (m.group(1), m.group(2), m.group(3), int(m.group(4))) == (workload, mode, kernel, tokens_per_launch):
                return float(m.group(5))
    return None


def algorithmic_work(w, modes, lens, fused=False):
    """Per kernel class, summed over one forward: (ops, bytes) that the method itself needs - operands read once,
    results written once, weights once per layer.  fused: attention blocks (INT8 ones with symmetric softmax codes, and FP16
    ones) run the QKV GEMM and the attention as one kernel (class qkv_attention: q, k, v are not traffic any more)."""
    T = int(lens.sum())
    H, F = w.hidden, w.ffn
    att = float((lens.astype("float64") ** 2).sum()) * 4 * H
    work = {k: [0.0, 0.0] for k in ("qkv", "attention", "qkv_attention", "attn_out", "ln1", "ffn1", "ffn2", "ln2")}
    for i, m in enumerate(modes):
        em = 1 if m & 1 else 2
        ef = 1 if m & 2 else 2
        en = 2 if i + 1 == len(modes) else (1 if modes[i + 1] & 1 else 2)
        one_kernel = fused and not ((m & 1) and (m & ~3))        # not for the unsigned / binary16 softmax variants
        front = ((("qkv_attention", 2.0 * T * 3 * H * H + att, (T * 2 * H + 3 * H * H) * em),) if one_kernel else
                 (("qkv", 2.0 * T * 3 * H * H, (T * 4 * H + 3 * H * H) * em), ("attention", att, T * 4 * H * em)))
        for k, ops, byts in front + (("attn_out", 2.0 * T * H * H, (T * 2 * H + H * H) * em),
                                     ("ln1", 10.0 * T * H, T * H * (2 * em + ef)),
                                     ("ffn1", 2.0 * T * H * F, (T * (H + F) + H * F) * ef),
                                     ("ffn2", 2.0 * T * H * F, (T * (H + F) + H * F) * ef),
                                     ("ln2", 10.0 * T * H, T * H * (2 * ef + en))):
            work[k][0] += ops
            work[k][1] += byts
    work["entry"] = [0.0, T * H * (2 + (1 if modes[0] & 1 else 2))]
    return work


def timed(enc, hid, mask, out, steps, repeats, torch):
    """Median over `repeats` runs of the wall-clock time of `steps` forwards, in ms per forward."""
    runs = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            enc.forward(hid, mask, out)
        torch.cuda.synchronize()
        runs.append((time.perf_counter() - t0) / steps * 1e3)
    return statistics.median(runs), runs


def kernel_table(P, enc, hid, mask, out, w0, modes, lens, steps, torch):
    """Every kernel class, one pass each, HIP events on the dispatches (groups run one after another meanwhile)."""
    all_i8 = all((m & 3) == P.FULL_INT8 for m in modes)
    all_f16 = all(m == P.FP16 for m in modes)
    measured = {}
    n_pass = min(steps, 20)
    for kname, which in (("entry", P.PROF_ENTRY), ("qkv", P.PROF_QKV), ("attention", P.PROF_ATTN), ("qkv_attention", P.PROF_QKV_ATTN),
                         ("attn_out", P.PROF_ATTN_OUT), ("ln1", P.PROF_LN1), ("ffn1", P.PROF_FFN1),
                         ("ffn2", P.PROF_FFN2), ("ln2", P.PROF_LN2)):
        enc.profile(which)
        for _ in range(n_pass):
            enc.forward(hid, mask, out)
        torch.cuda.synchronize()
        measured[kname] = enc.profile_read()
        enc.profile(P.PROF_OFF)
    work = algorithmic_work(w0, modes, lens, fused=measured["qkv_attention"][1] > 0)
    kernels = {}
    for kname, (kms, launches) in measured.items():
        if launches == 0:
            continue
        tot_s = kms * 1e-3 * launches / n_pass          # summed duration of the class in one forward
        ops_f, bytes_f = work[kname]
        ent = {"mean_launch_us": round(kms * 1e3, 2), "launches_per_step": launches / n_pass,
               "GB/s": round(bytes_f / tot_s / 1e9, 1), "frac_hbm": round(bytes_f / tot_s / 1e9 / HBM_PEAK_GBS, 4)}
        if kname in ("qkv", "qkv_attention", "attn_out", "ffn1", "ffn2") and (all_i8 or all_f16):
            peak = INT8_PEAK_TOPS if all_i8 else FP16_PEAK_TFLOPS
            ent["TOP/s" if all_i8 else "TFLOP/s"] = round(ops_f / tot_s / 1e12, 1)
            ent["frac_mfma"] = round(ops_f / tot_s / 1e12 / peak, 4)
        kernels[kname] = ent
    return kernels


def measure_peaks(P):
    pk = {}
    for name, f16 in (("int8", False), ("fp16", True)):
        unit = 1e12
        pk[f"mfma_{name}_constant_operands_T{'FL' if f16 else ''}OP/s"] = round(P.probe_mfma_rate(f16, False) / unit, 1)
        pk[f"mfma_{name}_random_operands_T{'FL' if f16 else ''}OP/s"] = round(P.probe_mfma_rate(f16, True) / unit, 1)
    pk["device_copy_GB/s"] = round(P.probe_copy_rate(1 << 30, 10) / 1e9, 1)
    # operand feed of the GEMM main loops without arithmetic: the QKV shape at 65536 tokens (all CUs busy for many tiles)
    # and the FFN1 shape at 2048 tokens (one launch of the headline workload: 384 tiles)
    big = P.probe_feed_rate(65536, 2304, 768)
    small = P.probe_feed_rate(2048, 3072, 768)
    pk["l2_to_lds_feed_TB/s"] = round(big / 1e12, 2)
    pk["l2_to_lds_feed_bytes_per_ns_per_CU"] = round(big / 1e9 / 256, 1)
    pk["l2_to_lds_feed_2048_tokens_TB/s"] = round(small / 1e12, 2)
    pk["note"] = ("issue rate of v_mfma_i32_32x32x32_i8 / v_mfma_f32_32x32x16_f16 from registers on all SIMDs; copy = bytes read + "
                  "written of a 1 GiB device copy; feed = bytes per second that blocks streaming 128 x 128 tile operands "
                  "(128-byte stages, direct loads into a 3-deep LDS ring, no matrix instruction) pull into LDS")
    return pk


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=5, help="timed runs of --steps forwards each; the median is reported")
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--groups", type=int, default=0, help="batch groups run concurrently (0 = library default)")
    ap.add_argument("--no-graph", action="store_true", help="headline from plain launches instead of HIP graph replay")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 256 MiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--only-mode", default=None, help="time a single precision mode (FULL_INT8, FP16, ...)")
    ap.add_argument("--peaks", action="store_true", help="only run the library's peak probes and print them")
    ap.add_argument("--no-peaks", action="store_true", help="skip the peak probes")
    ap.add_argument("--kernel-passes-only", action="store_true",
                    help="skip the throughput loops: only the per-kernel passes with isolated launches run (for profilers, "
                         "whose per-kernel averages then cover exactly the launches the kernel tables are made from)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent, so more GPUs would each take a "
              "share of the batch; nothing here does that). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2209_09130_amd as P
    import samp_workloads as W

    if not os.path.exists(P.lib_path()):
        from paper_2209_09130_amd import build as hip_build
        hip_build.build(force=True)
    P.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    print(f"bench.py: host cores {os.cpu_count()}", file=sys.stderr, flush=True)

    if a.peaks:
        print(json.dumps({"peaks_measured": measure_peaks(P)}), flush=True)
        return 0

    w0 = W.config(a.workload)
    cfg = (w0.layers, w0.hidden, w0.heads, w0.ffn, w0.ln_eps)
    wts = W.make_weights(w0)
    hid_np, lens, mask_np = W.make_hidden(w0)
    hid = torch.from_numpy(hid_np).cuda()
    mask = torch.from_numpy(mask_np).cuda() if w0.varlen else None
    T = int(lens.sum())

    # calibration on the GPU: all-FP16 encoder, absmax taps (product path, no oracle involved)
    cal = torch.from_numpy(W.make_calibration_batch(w0)).cuda()
    enc16 = P.Encoder(*cfg, (P.FP16,) * w0.layers, wts, None, max_batch=max(w0.batch, cal.shape[0]),
                      max_seq=max(w0.seq, cal.shape[1]))
    scales = enc16.calibrate(cal)

    if a.copy_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    uniform = [("FULL_INT8", P.FULL_INT8), ("FFN_INT8", P.FFN_INT8), ("MHA_INT8", P.MHA_INT8), ("FP16", P.FP16)]
    # C2 is timed in every uniform mode; the other workloads in the per-layer mask their configuration names
    mode_list = uniform if a.workload == "C2" else [("CONFIG", None)]
    if a.only_mode:
        # the softmax-output variants of the INT8 attention block are timed on request only
        named = uniform + [("CONFIG", None), ("FULL_INT8+PU", P.FULL_INT8 | P.P_UNSIGNED), ("FULL_INT8+P16", P.FULL_INT8 | P.P_FP16)]
        mode_list = [m for m in named if m[0] == a.only_mode]
        if not mode_list:
            raise SystemExit(f"unknown mode {a.only_mode}")
        if mode_list[0][1] is not None and mode_list[0][1] & P.P_UNSIGNED:
            scales = scales.copy()
            scales[:, 4] *= np.float32(127.0 / 255.0)          # the same range on 255 levels

    results = {}
    roof = None
    kernels = None
    kernels_fp16 = None
    for name, mode in mode_list:
        modes = w0.modes if mode is None else (mode,) * w0.layers
        enc = enc16 if (mode == P.FP16) else P.Encoder(*cfg, modes, wts, scales, max_batch=w0.batch, max_seq=w0.seq)
        out = torch.empty_like(hid)
        enc.set_groups(a.groups)
        per = {}
        for label, graph in (("graph", True), ("eager", False)):
            if a.kernel_passes_only:
                per[label], per[label + "_runs"] = float("nan"), []
                continue
            enc.set_graph(graph)
            for _ in range(a.warmup):
                enc.forward(hid, mask, out)
            med, runs = timed(enc, hid, mask, out, a.steps, a.repeats, torch)
            per[label] = med
            per[label + "_runs"] = [round(r, 4) for r in runs]
        enc.set_graph(not a.no_graph)
        ms = per["eager"] if a.no_graph else per["graph"]
        results[name] = {"ms_per_step": ms, "seq_per_s": w0.batch / (ms * 1e-3), "ms_per_step_graph": per["graph"],
                         "ms_per_step_eager": per["eager"], "runs_graph_ms": per["graph_runs"], "runs_eager_ms": per["eager_runs"]}
        headline = name == mode_list[0][0]                # FULL_INT8 (or the workload's own mask), unless --only-mode
        if headline:
            # The dominant kernel's launch duration: the same K steps once more with HIP events attached
            # to that kernel's dispatches (an event-carrying dispatch costs a few microseconds of queue
            # time, so this pass is kept out of the throughput figure above).
            enc.profile(P.PROF_FFN1)
            prof_steps = min(a.steps, 100)
            for _ in range(prof_steps):
                enc.forward(hid, mask, out)
            torch.cuda.synchronize()
            kms, launches = enc.profile_read()
            enc.profile(P.PROF_OFF)
            ffn_int8 = bool(modes[0] & 2)
            # the batch may be cut into groups that run concurrently: one launch covers tokens / groups
            per_forward = launches / prof_steps
            ops = 2.0 * T * w0.ffn * w0.hidden * w0.layers / per_forward
            achieved = ops / (kms * 1e-3) / 1e12 if kms > 0 else 0.0
            peak = INT8_PEAK_TOPS if ffn_int8 else FP16_PEAK_TFLOPS
            tokens_per_launch = int(round(T / (per_forward / w0.layers)))
            roof = {"kernel": "FFN1 INT8 GEMM + bias + GELU (threshold table) + quantise" if ffn_int8 else "FFN1 FP16 GEMM + bias + GELU",
                    "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TOP/s" if ffn_int8 else "TFLOP/s",
                    "frac": achieved / peak,
                    "traffic": measured_traffic(a.workload, name, "ffn1", tokens_per_launch),
                    "algorithmic_bytes": (T * w0.hidden + T * w0.ffn) / (per_forward / w0.layers) + w0.ffn * w0.hidden,
                    "launches_timed": launches, "launches_per_step": per_forward, "tokens_per_launch": tokens_per_launch,
                    "mean_launch_us": kms * 1e3, "ops_per_launch": ops,
                    "choice": "the largest dense contraction of a step (2 T F H operations per layer); where the QKV GEMM and the "
                              "attention run as one kernel, that mixed kernel (GEMM + softmax) can take longer per launch: its "
                              "figures are kernels.qkv_attention"}
            kernels = kernel_table(P, enc, hid, mask, out, w0, modes, lens, a.steps, torch)
        elif mode == P.FP16:
            kernels_fp16 = kernel_table(P, enc, hid, mask, out, w0, modes, lens, a.steps, torch)
        if enc is not enc16:
            enc.close()
    enc16.close()

    head = "FULL_INT8" if "FULL_INT8" in results else next(iter(results))
    line = {
        "metric": "sequences/sec BERT-base encoder b32xs128 per precision mode; % int8/fp16 MFMA peak",
        "value": results[head]["seq_per_s"], "unit": "sequences/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "repeats": a.repeats, "ms_per_step": results[head]["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8" if head != "FP16" else "f16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {w0.layers}-layer H{w0.hidden} F{w0.ffn} encoder, batch {w0.batch} x "
                               f"seq {w0.seq}, mode {head}", "tokens": T, "headline_mode": head,
                   "launch": "plain launches" if a.no_graph else "HIP graph replay"},
        "modes": results,
    }
    if roof:
        line["roofline"] = roof
        line["kernels"] = kernels
    if kernels_fp16:
        line["kernels_fp16"] = kernels_fp16
    if not a.no_peaks:
        line["peaks_measured"] = measure_peaks(P)

    if not a.no_cpu_baseline:
        import oracle
        n_seq = min(w0.batch, 32)
        modes = w0.modes if head == "CONFIG" else (P.FULL_INT8,) * w0.layers
        oenc = oracle.Encoder(*cfg, modes, wts, scales)
        t0 = time.perf_counter()
        oenc.forward(hid_np[:n_seq], lens[:n_seq])
        dt = time.perf_counter() - t0
        oenc.close()
        line["cpu_baseline"] = {"value": n_seq / dt, "unit": "sequences/s", "cores": oracle.max_threads(), "kind": "oracle",
                                "sample": f"{n_seq} of {w0.batch} sequences of the same batch, mode {head}, one pass, "
                                          f"{dt:.1f} s wall"}
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
