"""SiLU-gated FFN built from three factorised linears (Sec. 3.1 eq. FFN with every
weight replaced by a factor pair, Sec. 3.2).  Pure sequencing of library calls."""
from __future__ import annotations

from . import (fhpc_add, lowrank_ffn_down_bwd, lowrank_ffn_gate_up_fwd, lowrank_linear_bwd,
               lowrank_linear_bwd_shared_x, lowrank_linear_fwd, swiglu_fwd)


def ffn_fwd(X, Ag, Bg, Au, Bu, Ad, Bd):
    """Returns (Y, saved) with saved = tensors the backward pass reuses."""
    G, Hg = lowrank_linear_fwd(X, Ag, Bg, save_H=True)
    U, Hu = lowrank_linear_fwd(X, Au, Bu, save_H=True)
    Z = swiglu_fwd(G, U)
    Y, Hd = lowrank_linear_fwd(Z, Ad, Bd, save_H=True)
    return Y, (G, U, Z, Hg, Hu, Hd)


def ffn_bwd(X, Ag, Bg, Au, Bu, Ad, Bd, dY, saved):
    """Returns dX and the six weight gradients (fp32)."""
    G, U, Z, Hg, Hu, Hd = saved
    dG, dU, dAd, dBd = lowrank_ffn_down_bwd(Z, Ad, Bd, dY, G, U, H_saved=Hd)
    dXg, dAg, dBg = lowrank_linear_bwd(X, Ag, Bg, dG, H_saved=Hg)
    dXu, dAu, dBu = lowrank_linear_bwd(X, Au, Bu, dU, H_saved=Hu)
    dX = fhpc_add(dXg, dXu, out=dXg)
    return dX, (dAg, dBg, dAu, dBu, dAd, dBd)


def ffn_fwd_shared_x(X, A_gu, Bg, Bu, Ad, Bd):
    """The same FFN with the gate and up factors side by side in A_gu = [Ag | Au] (d x 2r): X is read
    once for both projections, and the gate is applied where U is produced (lowrank_ffn_gate_up_fwd).
    Returns (Y, saved)."""
    G, U, Z, H_gu = lowrank_ffn_gate_up_fwd(X, A_gu, Bg, Bu, save_H=True)
    Y, Hd = lowrank_linear_fwd(Z, Ad, Bd, save_H=True)
    return Y, (G, U, Z, H_gu, Hd)


def ffn_bwd_shared_x(X, A_gu, Bg, Bu, Ad, Bd, dY, saved):
    """Returns dX and (dA_gu, dBg, dBu, dAd, dBd), fp32.  The down projection's input gradient goes through the
    gate's backward where it is produced (lowrank_ffn_down_bwd); dX is one product over [dHg | dHu], so the two
    projections' input gradients are summed in the accumulators and rounded once."""
    G, U, Z, H_gu, Hd = saved
    dG, dU, dAd, dBd = lowrank_ffn_down_bwd(Z, Ad, Bd, dY, G, U, H_saved=Hd)
    dX, dA_gu, (dBg, dBu) = lowrank_linear_bwd_shared_x(X, A_gu, [Bg, Bu], [dG, dU], H_all_saved=H_gu)
    return dX, (dA_gu, dBg, dBu, dAd, dBd)
