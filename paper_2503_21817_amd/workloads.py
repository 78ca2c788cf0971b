"""Seeded synthetic inputs with the token-count shapes of the paper's workloads.

This module only draws random numbers and lays them out; it holds none of the
Skip-FFN arithmetic and imports neither the GPU binding nor the CPU oracle, so
both sides can be fed from it.

Shapes follow the paper: LLaVA-1.5 sequences are 576 visual + 40 text tokens
(Introduction); LLaVA-HD uses up to four local tiles plus one global view of
576 tokens each (Sections 4.1 and 5.4); the backbone layer is LLaMA-3-8B,
C = 4096 and M = I = 14336 (Table 1: 10.5 = 3 * I / C).  The retained / skipped
partition itself is a caller input to the block (Section 4.1 produces it from
vision features, which are not available here), so it is drawn: per sequence,
exactly `keep` visual tokens retained at seeded-uniform positions without
replacement; text tokens are always retained.

All tensors are returned as numpy arrays; bf16 tensors are uint16 bit patterns
(the conversion from float32 is torch's own round-to-nearest-even converter).
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    cfg: int
    C: int
    I: int
    visual: List[int]          # visual tokens per sequence
    text: List[int]            # text tokens per sequence
    keep: List[int]            # retained visual tokens per sequence
    layers: int = 1
    passes: str = "fwd"        # "fwd" or "fwd+bwd"
    eps: float = 1e-5
    seed: int = 0
    structured: bool = False   # retained visual tokens = leading contiguous run
    extra: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return int(sum(self.visual) + sum(self.text))

    @property
    def R(self) -> int:
        return int(sum(self.keep) + sum(self.text))

    def flops(self) -> int:
        """Model FLOPs, two per multiply-add: the 3*N2*C*M term of the paper's
        cost model (Section 5.2) with N2 = R, times 2; backward costs twice the
        forward."""
        per_layer = 6 * self.R * self.C * self.I
        if self.passes == "fwd+bwd":
            per_layer *= 3
        return per_layer * self.layers


def _bf16_bits(a32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(a32, dtype=np.float32))
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def config(n: int, structured: bool = False) -> Workload:
    """The five configurations the build is measured and tested on."""
    if n == 1:
        return Workload("cfg1-tiny-llava", 1, 256, 688, [64], [16], [16],
                        passes="fwd", seed=1001)
    if n == 2:
        return Workload("cfg2-llava-b8", 2, 4096, 14336, [576] * 8, [40] * 8,
                        [144] * 8, passes="fwd", seed=1002)
    if n == 3:
        return Workload("cfg3-llava-hd-b4" + ("-structured" if structured else ""),
                        3, 4096, 14336, [2880] * 4, [64] * 4, [576] * 4,
                        passes="fwd+bwd", seed=1003, structured=structured)
    if n == 4:
        rng = np.random.default_rng(1004)
        vis = rng.integers(576, 2881, size=16)
        txt = rng.integers(20, 201, size=16)
        ratio = rng.uniform(0.1, 0.5, size=16)
        keep = np.rint(ratio * vis).astype(np.int64)
        return Workload("cfg4-ragged-b16", 4, 4096, 14336, vis.tolist(),
                        txt.tolist(), keep.tolist(), passes="fwd+bwd", seed=1004)
    if n == 5:
        return Workload("cfg5-llava-b16-32layers", 5, 4096, 14336, [576] * 16,
                        [40] * 16, [144] * 16, layers=32, passes="fwd+bwd",
                        seed=1005)
    raise ValueError(f"unknown config {n}")


def small(C=256, I=512, visual=(96, 57), text=(9, 14), keep=(24, 11),
          passes="fwd+bwd", seed=7, name="small") -> Workload:
    """A free-form workload for tests."""
    return Workload(name, 0, C, I, list(visual), list(text), list(keep),
                    passes=passes, seed=seed)


def make_mask(w: Workload) -> np.ndarray:
    """uint8 [T]; non-zero = the token skips the FFN.  Layout per sequence:
    [visual tokens][text tokens], sequences packed back to back."""
    rng = np.random.default_rng(w.seed)
    parts = []
    for v, t, k in zip(w.visual, w.text, w.keep):
        m = np.ones(v + t, dtype=np.uint8)
        if w.structured:
            m[:k] = 0
        else:
            m[rng.choice(v, size=k, replace=False)] = 0
        m[v:] = 0
        parts.append(m)
    if not parts:
        return np.zeros(0, dtype=np.uint8)
    return np.concatenate(parts)


def make_hidden(w: Workload) -> np.ndarray:
    """bf16 bits [T, C], values ~ N(0, 1)."""
    rng = np.random.default_rng(w.seed + 10_000)
    return _bf16_bits(rng.standard_normal((w.T, w.C), dtype=np.float32))


def make_grad(w: Workload) -> np.ndarray:
    """Upstream gradient on all T rows, bf16 bits [T, C], ~ N(0, 1)."""
    rng = np.random.default_rng(w.seed + 20_000)
    return _bf16_bits(rng.standard_normal((w.T, w.C), dtype=np.float32))


def make_weights(w: Workload, layer: int = 0):
    """(w_gate [I, C], w_up [I, C], w_down [C, I]) as bf16 bits, ~ N(0, 0.02)."""
    rng = np.random.default_rng(2000 + w.cfg * 100 + layer + (w.seed if w.cfg == 0 else 0))
    out = []
    for shape in ((w.I, w.C), (w.I, w.C), (w.C, w.I)):
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(0.02)
        out.append(_bf16_bits(a))
    return tuple(out)


def make_gain(w: Workload, unit: bool = True) -> np.ndarray:
    """RMSNorm gain, bf16 bits [C]: ones (the configurations' setting) or
    1 + 0.1 * N(0, 1) for tests that exercise the gain."""
    if unit:
        return _bf16_bits(np.ones(w.C, dtype=np.float32))
    rng = np.random.default_rng(w.seed + 30_000)
    return _bf16_bits(1.0 + 0.1 * rng.standard_normal(w.C, dtype=np.float32))


def make_summary_sets(w: Workload):
    """Token sets for the adaptive summary layer (Section 4.2): per sequence two disjoint
    sets, the retained and then the skipped visual tokens (the paper puts one summary token
    at each end of the skipped run).  Returns (tok int32 [n_tok], seg int32 [2 B + 1])."""
    mask = make_mask(w)
    tok, seg = [], [0]
    base = 0
    for v, t in zip(w.visual, w.text):
        vis = np.arange(base, base + v)
        m = mask[base:base + v]
        for part in (vis[m == 0], vis[m != 0]):
            tok.append(part)
            seg.append(seg[-1] + len(part))
        base += v + t
    tok = np.concatenate(tok) if tok else np.zeros(0, np.int64)
    return tok.astype(np.int32), np.asarray(seg, dtype=np.int32)


def make_summary_weight(w: Workload) -> np.ndarray:
    """Weight row of the summary layer, bf16 bits [C], ~ N(0, 0.02): scores X w have a
    standard deviation of about 0.02 * sqrt(C), i.e. a softmax that is neither flat nor
    one-hot at C = 4096."""
    rng = np.random.default_rng(w.seed + 40_000)
    return _bf16_bits(np.float32(0.02) * rng.standard_normal(w.C, dtype=np.float32))

