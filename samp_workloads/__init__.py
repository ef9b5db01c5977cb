"""Seeded synthetic inputs for the mixed-precision encoder.

This module only draws random tensors with the shapes, value distributions and
length mixes of the benchmark configurations.  It holds none of the method's
arithmetic (no quantisation, no scales, no encoder maths): both the CPU oracle
and the HIP library receive exactly these arrays and do their own work on them.

The paper evaluates on fine-tuned BERT-base checkpoints and CLUE text data
(Section 4.1), neither of which is available; the tensors drawn here stand in
for them with the same model shapes (BERT-base 12 x 768, BERT-large 24 x 1024).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

# per-layer precision mode: bit0 = attention block INT8, bit1 = feed-forward block INT8
FP16, MHA_INT8, FFN_INT8, FULL_INT8 = 0, 1, 2, 3
P_UNSIGNED = 4          # flag on top of MHA_INT8 / FULL_INT8: softmax codes 0..255 instead of the symmetric range
P_FP16 = 8              # flag on top of MHA_INT8 / FULL_INT8 (not with P_UNSIGNED): the softmax output stays binary16
MODE_NAMES = {FP16: "FP16", MHA_INT8: "MHA_INT8", FFN_INT8: "FFN_INT8", FULL_INT8: "FULL_INT8",
              MHA_INT8 | P_UNSIGNED: "MHA_INT8+PU", FULL_INT8 | P_UNSIGNED: "FULL_INT8+PU",
              MHA_INT8 | P_FP16: "MHA_INT8+P16", FULL_INT8 | P_FP16: "FULL_INT8+P16"}


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    hidden: int
    heads: int
    ffn: int
    batch: int
    seq: int
    modes: tuple                 # one mode per layer
    head_dim: int = 64
    ln_eps: float = 1e-12
    varlen: bool = False         # lengths uniform in [min_len, seq], right padded
    min_len: int = 16
    outlier_frac: float = 0.0    # fraction of hidden channels scaled by outlier_gain
    outlier_gain: float = 20.0
    plain_params: bool = True    # zero biases, gamma=1, beta=0 (benchmark recipe)
    weight_seed: int = 1000
    hidden_seed: int = 42
    calib_seed: int = 7
    len_seed: int = 99
    outlier_seed: int = 5
    calib_batch: int = 8
    calib_seq: int = 128

    def with_modes(self, modes) -> "Workload":
        if isinstance(modes, int):
            modes = (modes,) * self.layers
        return replace(self, modes=tuple(modes))


def bert_base(name, layers, batch, seq, modes, **kw) -> Workload:
    if isinstance(modes, int):
        modes = (modes,) * layers
    return Workload(name, layers, 768, 12, 3072, batch, seq, tuple(modes), **kw)


def bert_large(name, layers, batch, seq, modes, **kw) -> Workload:
    if isinstance(modes, int):
        modes = (modes,) * layers
    return Workload(name, layers, 1024, 16, 4096, batch, seq, tuple(modes), **kw)


def config(name: str) -> Workload:
    """The five benchmark configurations (C1..C5)."""
    if name == "C1":
        return bert_base("C1", 1, 1, 128, FFN_INT8)
    if name == "C2":
        return bert_base("C2", 12, 32, 128, FULL_INT8)
    if name == "C3":
        return bert_base("C3", 12, 64, 128, (FULL_INT8,) * 6 + (FP16,) * 6, varlen=True)
    if name == "C4":
        return bert_large("C4", 24, 32, 256, FULL_INT8, outlier_frac=0.01)
    if name == "C5":
        return bert_base("C5", 12, 128, 512, FULL_INT8)
    raise KeyError(name)


def make_weights(w: Workload) -> List[Dict[str, np.ndarray]]:
    """Per layer: fp16 matrices in [out, in] row-major, fp32 vectors.

    Benchmark recipe: N(0, 0.02) drawn in fp32 and cast to fp16, zero biases,
    LayerNorm gamma = 1 and beta = 0.  With plain_params=False the vectors are
    random too, so that tests exercise the bias / gamma / beta terms.
    """
    out = []
    H, F = w.hidden, w.ffn
    for layer in range(w.layers):
        rng = np.random.default_rng(w.weight_seed + layer)

        def mat(n, k):
            return (rng.standard_normal((n, k), dtype=np.float32) * np.float32(0.02)).astype(np.float16)

        d = {
            "w_qkv": mat(3 * H, H),
            "w_o": mat(H, H),
            "w_ffn1": mat(F, H),
            "w_ffn2": mat(H, F),
        }
        if w.plain_params:
            d.update(
                b_qkv=np.zeros(3 * H, np.float32), b_o=np.zeros(H, np.float32),
                b_ffn1=np.zeros(F, np.float32), b_ffn2=np.zeros(H, np.float32),
                ln1_g=np.ones(H, np.float32), ln1_b=np.zeros(H, np.float32),
                ln2_g=np.ones(H, np.float32), ln2_b=np.zeros(H, np.float32),
            )
        else:
            def vec(n, scale, shift=0.0):
                return (rng.standard_normal(n, dtype=np.float32) * np.float32(scale) + np.float32(shift))
            d.update(
                b_qkv=vec(3 * H, 0.05), b_o=vec(H, 0.05), b_ffn1=vec(F, 0.05), b_ffn2=vec(H, 0.05),
                ln1_g=vec(H, 0.1, 1.0), ln1_b=vec(H, 0.1), ln2_g=vec(H, 0.1, 1.0), ln2_b=vec(H, 0.1),
            )
        out.append(d)
    return out


def _outlier_channels(w: Workload) -> np.ndarray:
    n = int(round(w.outlier_frac * w.hidden))
    if n == 0:
        return np.zeros(0, np.int64)
    rng = np.random.default_rng(w.outlier_seed)
    return np.sort(rng.choice(w.hidden, size=n, replace=False))


def _draw_hidden(w: Workload, seed: int, batch: int, seq: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, seq, w.hidden), dtype=np.float32)
    ch = _outlier_channels(w)
    if ch.size:
        x[:, :, ch] *= np.float32(w.outlier_gain)
    return x.astype(np.float16)


def make_lengths(w: Workload, batch: Optional[int] = None) -> np.ndarray:
    batch = w.batch if batch is None else batch
    if not w.varlen:
        return np.full(batch, w.seq, np.int32)
    rng = np.random.default_rng(w.len_seed)
    return rng.integers(w.min_len, w.seq + 1, size=batch, dtype=np.int32)


def make_hidden(w: Workload, batch: Optional[int] = None):
    """(hidden fp16 [B,S,H], lengths int32 [B], mask int32 [B,S]).

    Padded rows hold N(0,1) garbage on purpose: they must not influence the
    valid rows and must come back as zeros.
    """
    batch = w.batch if batch is None else batch
    hidden = _draw_hidden(w, w.hidden_seed, batch, w.seq)
    lens = make_lengths(w, batch)
    mask = (np.arange(w.seq, dtype=np.int32)[None, :] < lens[:, None]).astype(np.int32)
    return hidden, lens, mask


def make_calibration_batch(w: Workload) -> np.ndarray:
    """Full-length calibration batch (8 x 128 by default), same channel recipe."""
    return _draw_hidden(w, w.calib_seed, w.calib_batch, w.calib_seq)


def make_embedding(w: Workload, vocab: int = 21128, segments: int = 2, seed: int = 300, plain: bool = False):
    """Embedding tables of a BERT-style model (token, segment, position; fp16) and the LayerNorm vectors that end the
    embedding.  N(0, 0.02) like the other weights; vocab defaults to the size of the Chinese BERT-base vocabulary."""
    rng = np.random.default_rng(seed)
    H = w.hidden
    emb = {
        "tok": (rng.standard_normal((vocab, H)) * 0.02).astype(np.float16),
        "seg": (rng.standard_normal((segments, H)) * 0.02).astype(np.float16),
        "pos": (rng.standard_normal((max(w.seq, 8), H)) * 0.02).astype(np.float16),
        "gamma": np.ones(H, np.float32) if plain else (1.0 + 0.1 * rng.standard_normal(H)).astype(np.float32),
        "beta": np.zeros(H, np.float32) if plain else (0.1 * rng.standard_normal(H)).astype(np.float32),
        "eps": w.ln_eps,
    }
    return emb


def make_ids(w: Workload, vocab: int = 21128, segments: int = 2, seed: int = 301):
    """Token and segment ids [B,S] int32 for the workload's batch: uniform tokens, segment 0 then 1 split at a random
    point of each sequence; ids in padded positions are random too (they must not matter)."""
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, vocab, (w.batch, w.seq)).astype(np.int32)
    split = rng.integers(0, w.seq + 1, w.batch)
    seg = (np.arange(w.seq)[None, :] >= split[:, None]).astype(np.int32) % segments
    return ids, seg
