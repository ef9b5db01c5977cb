"""Latency side of the accuracy / latency trade-off (Section 3.2; Table 2's "Quantized Layer" columns): times the
encoder with the first k layers in a quantised mode and the rest in FP16, for a list of k.  The accuracies that
Algorithm 1 also needs come from the caller's own evaluation of each setting."""
from __future__ import annotations

import time
from typing import Iterable, List

import torch

from . import binding as B


def measure_latencies(workload, mode: int, counts: Iterable[int], steps: int = 50, warmup: int = 10) -> List[float]:
    """Seconds per forward for each k in counts (layers 0..k-1 in `mode`, layers k.. in FP16), on synthetic inputs of
    the workload's shape; scales come from the library's own calibration pass."""
    import samp_workloads as W
    wts = W.make_weights(workload)
    hid_np, lens, mask_np = W.make_hidden(workload)
    hid = torch.from_numpy(hid_np).cuda()
    mask = torch.from_numpy(mask_np).cuda() if workload.varlen else None
    cal = torch.from_numpy(W.make_calibration_batch(workload)).cuda()
    cfg = (workload.layers, workload.hidden, workload.heads, workload.ffn, workload.ln_eps)
    enc16 = B.Encoder(*cfg, (B.FP16,) * workload.layers, wts, None, max_batch=max(workload.batch, cal.shape[0]),
                      max_seq=max(workload.seq, cal.shape[1]))
    scales = enc16.calibrate(cal)
    enc16.close()
    out = torch.empty_like(hid)
    result = []
    for k in counts:
        modes = (mode,) * k + (B.FP16,) * (workload.layers - k)
        enc = B.Encoder(*cfg, modes, wts, scales, max_batch=workload.batch, max_seq=workload.seq)
        for _ in range(warmup):
            enc.forward(hid, mask, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            enc.forward(hid, mask, out)
        torch.cuda.synchronize()
        result.append((time.perf_counter() - t0) / steps)
        enc.close()
    return result
