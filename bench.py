#!/usr/bin/env python3
"""Benchmark of the mixed-precision encoder on one MI355X.

Workload: BERT-base 12-layer encoder, batch 32 x 128 tokens, all sequences full length (synthetic
N(0,0.02) weights, N(0,1) inputs, min-max calibration on a seeded 8x128 batch run on the GPU).
A step is one forward of the whole encoder.  The headline `value` is sequences/s of the full-INT8
stack; the other precision modes are timed the same way and reported under "modes".

Extra objects on the JSON line:
  roofline     - the FFN1 INT8 GEMM (+bias+GELU+quantise) kernel: algorithmic ops per launch
                 (2 * tokens * ffn * hidden) over its mean launch duration, measured with HIP events
                 attached to the dispatches over a repeat of the timed steps, against the int8 MFMA dense peak.
  cpu_baseline - the CPU oracle (as it stands, OpenMP over sequences) on the same batch.
  kernels      - every kernel class of the headline mode timed the same way (one class per pass, launches
                 isolated): mean launch duration, and its algorithmic ops or bytes over that duration against
                 the MFMA or HBM peak.
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

# HBM bytes per launch of the dominant kernel, from profiles/c2_full_int8_hbm_traffic.txt (rocprofv3 FETCH_SIZE x 2.0 +
# WRITE_SIZE x 1.0, factors from a 256 MiB copy): workload C2, full-INT8, FFN1 kernel, 2048 tokens per launch.
MEASURED_TRAFFIC_BYTES = {("C2", "FULL_INT8", 2048): 27.15e6}

INT8_PEAK_TOPS = 5000.0        # MI355X dense int8 MFMA, published: 5.0 POP/s
FP16_PEAK_TFLOPS = 2500.0      # dense fp16
HBM_PEAK_GBS = 8000.0


def algorithmic_work(w, modes, lens):
    """Per kernel class, summed over one forward: (ops, bytes, bound, dtype-is-int8) that the method itself
    needs - operands read once, results written once, weights once per layer."""
    T = int(lens.sum())
    H, F = w.hidden, w.ffn
    att = float((lens.astype("float64") ** 2).sum()) * 4 * H
    work = {k: [0.0, 0.0] for k in ("qkv", "attention", "attn_out", "ln1", "ffn1", "ffn2", "ln2")}
    for i, m in enumerate(modes):
        em = 1 if m & 1 else 2
        ef = 1 if m & 2 else 2
        en = 2 if i + 1 == len(modes) else (1 if modes[i + 1] & 1 else 2)
        for k, ops, byts in (("qkv", 2.0 * T * 3 * H * H, (T * 4 * H + 3 * H * H) * em),
                             ("attention", att, T * 4 * H * em),
                             ("attn_out", 2.0 * T * H * H, (T * 2 * H + H * H) * em),
                             ("ln1", 10.0 * T * H, T * H * (2 * em + ef)),
                             ("ffn1", 2.0 * T * H * F, (T * (H + F) + H * F) * ef),
                             ("ffn2", 2.0 * T * H * F, (T * (H + F) + H * F) * ef),
                             ("ln2", 10.0 * T * H, T * H * (2 * ef + en))):
            work[k][0] += ops
            work[k][1] += byts
    work["entry"] = [0.0, T * H * (2 + (1 if modes[0] & 1 else 2))]
    return work


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--groups", type=int, default=0, help="batch groups run concurrently (0 = library default)")
    ap.add_argument("--no-graph", action="store_true", help="plain launches instead of HIP graph replay")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 256 MiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--only-mode", default=None, help="time a single precision mode (FULL_INT8, FP16, ...)")
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

    mode_list = [("FULL_INT8", P.FULL_INT8), ("FFN_INT8", P.FFN_INT8), ("MHA_INT8", P.MHA_INT8), ("FP16", P.FP16)]
    if a.workload != "C2":
        mode_list = [("CONFIG", None)]
    if a.only_mode:
        # the softmax-output variants of the INT8 attention block are timed on request only
        mode_list += [("FULL_INT8+PU", P.FULL_INT8 | P.P_UNSIGNED), ("FULL_INT8+P16", P.FULL_INT8 | P.P_FP16)]
        mode_list = [m for m in mode_list if m[0] == a.only_mode]
        if not mode_list:
            raise SystemExit(f"unknown mode {a.only_mode}")
        if mode_list[0][1] is not None and mode_list[0][1] & P.P_UNSIGNED:
            scales = scales.copy()
            scales[:, 4] *= np.float32(127.0 / 255.0)          # the same range on 255 levels

    results = {}
    roof = None
    for name, mode in mode_list:
        modes = w0.modes if mode is None else (mode,) * w0.layers
        enc = enc16 if (mode == P.FP16) else P.Encoder(*cfg, modes, wts, scales, max_batch=w0.batch, max_seq=w0.seq)
        out = torch.empty_like(hid)
        enc.set_groups(a.groups)
        if a.no_graph:
            enc.set_graph(False)
        for _ in range(a.warmup):
            enc.forward(hid, mask, out)
        headline = name == mode_list[0][0]                # FULL_INT8 (or the workload's own mask), unless --only-mode
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            enc.forward(hid, mask, out)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ms = dt / a.steps * 1e3
        results[name] = {"ms_per_step": ms, "seq_per_s": w0.batch / (ms * 1e-3)}
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
            roof = {"kernel": "gemm_nt_kernel<I8,EpiGeluQuant> (FFN1 GEMM + bias + GELU + quantise)" if ffn_int8
                    else "gemm_nt_kernel<F16,EpiF16> (FFN1)",
                    "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TOP/s" if ffn_int8 else "TFLOP/s",
                    "frac": achieved / peak,
                    "traffic": MEASURED_TRAFFIC_BYTES.get((a.workload, name, int(round(T / (per_forward / w0.layers))))),
                    "algorithmic_bytes": (T * w0.hidden + T * w0.ffn) / (per_forward / w0.layers) + w0.ffn * w0.hidden, "launches_timed": launches, "launches_per_step": per_forward,
                    "mean_launch_us": kms * 1e3, "ops_per_launch": ops}
            # every kernel class, one pass each
            work = algorithmic_work(w0, modes, lens)
            all_i8 = all((m & 3) == P.FULL_INT8 for m in modes)
            kernels = {}
            for kname, which in (("entry", P.PROF_ENTRY), ("qkv", P.PROF_QKV), ("attention", P.PROF_ATTN),
                                 ("attn_out", P.PROF_ATTN_OUT), ("ln1", P.PROF_LN1), ("ffn1", P.PROF_FFN1),
                                 ("ffn2", P.PROF_FFN2), ("ln2", P.PROF_LN2)):
                enc.profile(which)
                n_pass = min(a.steps, 20)
                for _ in range(n_pass):
                    enc.forward(hid, mask, out)
                torch.cuda.synchronize()
                kms, launches = enc.profile_read()
                enc.profile(P.PROF_OFF)
                if launches == 0:
                    continue
                tot_s = kms * 1e-3 * launches / n_pass          # summed duration of the class in one forward
                ops_f, bytes_f = work[kname]
                ent = {"mean_launch_us": round(kms * 1e3, 2), "launches_per_step": launches / n_pass,
                       "GB/s": round(bytes_f / tot_s / 1e9, 1), "frac_hbm": round(bytes_f / tot_s / 1e9 / HBM_PEAK_GBS, 4)}
                if kname in ("qkv", "attn_out", "ffn1", "ffn2") and (all_i8 or all(m == P.FP16 for m in modes)):
                    peak = INT8_PEAK_TOPS if all_i8 else FP16_PEAK_TFLOPS
                    ent["TOP/s" if all_i8 else "TFLOP/s"] = round(ops_f / tot_s / 1e12, 1)
                    ent["frac_mfma"] = round(ops_f / tot_s / 1e12 / peak, 4)
                kernels[kname] = ent
        if enc is not enc16:
            enc.close()
    enc16.close()

    head = "FULL_INT8" if "FULL_INT8" in results else next(iter(results))
    line = {
        "metric": "sequences/sec BERT-base encoder b32xs128 per precision mode; % int8/fp16 MFMA peak",
        "value": results[head]["seq_per_s"], "unit": "sequences/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": results[head]["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8" if head != "FP16" else "f16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {w0.layers}-layer H{w0.hidden} F{w0.ffn} encoder, batch {w0.batch} x "
                               f"seq {w0.seq}, mode {head}", "tokens": T, "headline_mode": head},
        "modes": results,
    }
    if roof:
        line["roofline"] = roof
        line["kernels"] = kernels

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
