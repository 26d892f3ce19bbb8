"""Bit-budget bookkeeping of appendix D of the paper.  Test infrastructure only.

These closed forms relate the average target bit-width t, the dense bit-width
w, the hidden size d and the number k of weak columns; the bench uses them to
print the paper-style "effective bits" next to the bytes the kernel moves.
"""
from __future__ import annotations


def fp16_ratio_per_block(t: float, w: int) -> float:
    """r of appendix D.2: a decoder block of 12 d^2 weights keeps r d^2 of them in fp16."""
    return (t - w) / (16 - w) * 12


def weak_columns(t: float, w: int, d: int, n_layers: int = 6) -> int:
    """k of appendix D.2 for a self-attention projection (d x d) of an OPT block."""
    return int(round(fp16_ratio_per_block(t, w) / n_layers * d))


def overhead_owq(d: int, t: float, w: int) -> float:
    """Appendix D.1: fp16 elements per OPT decoder block kept by OWQ."""
    return 12 * d * d * (t - w) / (16 - w) + 9 * d


def overhead_group(d: int, g: int) -> float:
    """Appendix D.1: fp16 quantisation parameters per OPT block at group size g."""
    return 12 * d * d / g


def effective_bits(d_out: int, d_in: int, w: int, k: int, zero_filled: bool) -> float:
    """Average bits per weight of one layer (quantisation parameters not counted).

    Storage-favoured (appendix B.2): the low-bit matrix has d_in - k columns.
    Latency-favoured: it keeps all d_in columns, weak positions zero-filled.
    """
    dense_cols = d_in if zero_filled else d_in - k
    return (w * dense_cols + 16 * k) / d_in


def wct_vs_qlora_params(d: int, D: int, k: int, r: int):
    """Appendix D.3: learnable parameters per LLaMA decoder block, (WCT, QLoRA)."""
    return (5 * d + 2 * D) * k, (11 * d + 3 * D) * r
