"""Size and work bookkeeping for the factorised layer (host-side, no GPU).

Sec. 3.2: a dense d_in x d_out weight has d_in*d_out parameters and costs that
many multiplications per token; the factor pair A (d_in x r), B (r x d_out) has
r*(d_in + d_out) of each (n^2 -> 2nr for a square layer).
"""
from __future__ import annotations


def dense_params(d_in: int, d_out: int) -> int:
    return d_in * d_out


def lowrank_params(d_in: int, r: int, d_out: int) -> int:
    return r * (d_in + d_out)


def lowrank_mults_per_token(d_in: int, r: int, d_out: int) -> int:
    """Multiplications of y = (x A) B for one token."""
    return r * (d_in + d_out)


def lowrank_flops(M: int, d_in: int, r: int, d_out: int, fwd: bool = True, bwd: bool = True) -> int:
    """Algorithmic flop of the factorised layer: fwd = 2 GEMMs, bwd = 4 GEMMs,
    each 2*M*r*d (recomputing H in backward is not counted)."""
    per_gemm_pair = 2 * M * r * (d_in + d_out)
    return (per_gemm_pair if fwd else 0) + (2 * per_gemm_pair if bwd else 0)


def qlinear_lowrank_flops(M: int, d_in: int, r: int, d_out: int, fwd: bool = True, bwd: bool = True) -> int:
    """Frozen dense base (X*W fwd, dY*W^T bwd; no dW) plus the low-rank branch."""
    base = 2 * M * d_in * d_out
    return lowrank_flops(M, d_in, r, d_out, fwd, bwd) + (base if fwd else 0) + (base if bwd else 0)


def compression_ratio(d_in: int, r: int, d_out: int) -> float:
    """Sec. 4.1: a square n x n layer shrinks by n / (2 r)."""
    return dense_params(d_in, d_out) / lowrank_params(d_in, r, d_out)
