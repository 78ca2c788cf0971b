"""Shared helpers for the GPU parity tests: host bit arrays <-> device tensors,
error metrics, and running the HIP path on a workload."""
from __future__ import annotations

import numpy as np
import torch

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import workloads as W

REL_L2_TOL = 1e-2   # relative L2 bound on retained outputs and gradients (bf16 in, fp32 accumulate)


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f64_of(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return O.bf16_bits_to_f64(bits_of(t))
    return t.detach().cpu().numpy().astype(np.float64)


def rel_l2(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want)
    num = np.linalg.norm(got - want)
    return float(num / den) if den > 0 else float(num)


def max_slice_rel_l2(got: np.ndarray, want: np.ndarray, axis: int) -> float:
    """Largest relative L2 error over the slices along `axis` (axis=1: per row, axis=0: per
    column): one wrong tile edge, chunk or row cannot hide in the norm of a whole tensor."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    num = np.sqrt(np.einsum("ij,ij->i" if axis == 1 else "ij,ij->j", got - want, got - want))
    den = np.sqrt(np.einsum("ij,ij->i" if axis == 1 else "ij,ij->j", want, want))
    return float((num / np.maximum(den, 1e-300)).max())


class Problem:
    """Host inputs of one workload plus their device copies."""

    def __init__(self, w, unit_gain=True, with_gain_tensor=False, layer=0):
        self.w = w
        self.mask = W.make_mask(w)
        self.hidden = W.make_hidden(w)
        self.grad = W.make_grad(w)
        self.wg, self.wu, self.wd = W.make_weights(w, layer)
        self.gain = None
        if with_gain_tensor:
            self.gain = W.make_gain(w, unit=unit_gain)
        self.d_mask = torch.from_numpy(self.mask).cuda()
        self.d_hidden = to_dev_bf16(self.hidden)
        self.d_grad = to_dev_bf16(self.grad)
        self.d_wg, self.d_wu, self.d_wd = (to_dev_bf16(a) for a in (self.wg, self.wu, self.wd))
        self.d_gain = None if self.gain is None else to_dev_bf16(self.gain)
