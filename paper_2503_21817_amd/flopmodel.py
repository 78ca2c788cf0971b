"""The paper's per-layer cost model (Section 5.2, efficiency evaluation).

One count per multiply-add:  4*N*C^2 + 2*N^2*C + 3*N*C*M  for a LLaMA layer on
N tokens, and with Skip-Vision  4*N1*C^2 + 2*N1^2*C + 3*N2*C*M  where N1 tokens
go through attention and N2 through the FFN.  The benchmark prices the
Skip-FFN block with the third term only (N2 = retained rows), at two FLOPs per
multiply-add.
"""

from __future__ import annotations


def layer_macs(n_attn: int, n_ffn: int, C: int, M: int) -> int:
    """Multiply-adds of one decoder layer: attention on n_attn tokens, FFN on
    n_ffn tokens."""
    return 4 * n_attn * C * C + 2 * n_attn * n_attn * C + 3 * n_ffn * C * M


def flops_ratio(n_attn: int, n_ffn: int, n_base: int, C: int = 4096, M: int = 14336) -> float:
    """Cost of a Skip-Vision layer relative to the same layer on n_base tokens
    that all take the FFN (the FLOPs column of Table 3)."""
    return layer_macs(n_attn, n_ffn, C, M) / layer_macs(n_base, n_base, C, M)


def ffn_macs(n_ffn: int, C: int, M: int) -> int:
    """The 3*N2*C*M term alone: what the Skip-FFN block computes, forward."""
    return 3 * n_ffn * C * M


def ffn_params(C: int, M: int, layers: int) -> int:
    """FFN parameters of the whole model: three C x M matrices per layer
    (Table 1)."""
    return 3 * C * M * layers


def skipffn_flops(R: int, C: int, I: int, backward: bool, layers: int = 1) -> int:
    """Model FLOPs (two per multiply-add) of the block on R retained rows:
    6*R*C*I forward; backward adds twice that (dX and dW GEMMs)."""
    f = 2 * ffn_macs(R, C, I)
    if backward:
        f *= 3
    return f * layers
