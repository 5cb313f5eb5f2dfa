"""GPU parity of the SiLU gate and of the SiLU-gated FFN built from three factorised
linears (config 3), per call and end to end."""
import numpy as np
import pytest

import oracle
from harness import TOL_BF16, TOL_F32, Bf16, from_device, sample_rows
from paper_2402_13533_amd import synth

pytestmark = pytest.mark.gpu


def _fhpc():
    import paper_2402_13533_amd as fhpc
    return fhpc


def test_swiglu_elementwise():
    import torch
    fhpc = _fhpc()
    n = 1000 * 1031 + 7                                # ragged length
    G = Bf16.normal(901, (n,), 2.0)
    U = Bf16.normal(902, (n,), 1.0)
    dZ = Bf16.normal(903, (n,), 1.0)
    G.bits[:4] = synth.f32_to_bf16_bits(np.array([0.0, 30.0, -30.0, -100.0], dtype=np.float32))
    Z = fhpc.swiglu_fwd(G.cuda(), U.cuda())
    dG, dU = fhpc.swiglu_bwd(G.cuda(), U.cuda(), dZ.cuda())
    Zr = oracle.swiglu_fwd(G.f64, U.f64)
    dGr, dUr = oracle.swiglu_bwd(G.f64, U.f64, dZ.f64)
    # one bf16 rounding of an fp32 result: 2^-9 relative per element
    for got, ref in ((Z, Zr), (dG, dGr), (dU, dUr)):
        g = from_device(got)
        assert np.all(np.isfinite(g))
        assert np.all(np.abs(g - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-30)
    # fp32 storage
    Gf, Uf = synth.normal(904, (4099,), 2.0), synth.normal(905, (4099,), 1.0)
    Zf = fhpc.swiglu_fwd(torch.from_numpy(Gf).cuda(), torch.from_numpy(Uf).cuda())
    assert oracle.rel_fro(from_device(Zf), oracle.swiglu_fwd(Gf, Uf)) <= TOL_F32


def _ffn_inputs(M, d, r, f, base=0):
    s = lambda i: synth.tensor_seed(3, base + i)
    X = Bf16.normal(s(0), (M, d), 1.0)
    dY = Bf16.normal(s(1), (M, d), 1.0)
    Ag = Bf16.normal(s(2), (d, r), d ** -0.5); Bg = Bf16.normal(s(3), (r, f), r ** -0.5)
    Au = Bf16.normal(s(4), (d, r), d ** -0.5); Bu = Bf16.normal(s(5), (r, f), r ** -0.5)
    Ad = Bf16.normal(s(6), (f, r), f ** -0.5); Bd = Bf16.normal(s(7), (r, d), r ** -0.5)
    return X, dY, (Ag, Bg, Au, Bu, Ad, Bd)


def _oracle_ffn(X, dY, W, want_weight_grads=True):
    Ag, Bg, Au, Bu, Ad, Bd = [w.f64 for w in W]
    G, _ = oracle.lowrank_fwd(X, Ag, Bg)
    U, _ = oracle.lowrank_fwd(X, Au, Bu)
    Z = oracle.swiglu_fwd(G, U)
    Y, _ = oracle.lowrank_fwd(Z, Ad, Bd)
    dZ, dAd, dBd = oracle.lowrank_bwd(Z, Ad, Bd, dY)
    dG, dU = oracle.swiglu_bwd(G, U, dZ)
    dXg, dAg, dBg = oracle.lowrank_bwd(X, Ag, Bg, dG)
    dXu, dAu, dBu = oracle.lowrank_bwd(X, Au, Bu, dU)
    return Y, dXg + dXu, (dAg, dBg, dAu, dBu, dAd, dBd)


def test_config3_chain_reduced_tokens():
    """Config 3 with its real widths (4096 -> r 1024 -> 11008 -> r 1024 -> 4096) on 320
    tokens: every output of the chain, end to end, against the full oracle."""
    from paper_2402_13533_amd import ffn
    M, d, r, f = 320, 4096, 1024, 11008
    X, dY, W = _ffn_inputs(M, d, r, f)
    Yr, dXr, gr = _oracle_ffn(X.f64, dY.f64, W)
    Wd = [w.cuda() for w in W]
    Y, saved = ffn.ffn_fwd(X.cuda(), *Wd)
    dX, grads = ffn.ffn_bwd(X.cuda(), *Wd, dY.cuda(), saved)
    errs = {"Y": oracle.rel_fro(from_device(Y), Yr), "dX": oracle.rel_fro(from_device(dX), dXr)}
    for name, g, r_ in zip(("dAg", "dBg", "dAu", "dBu", "dAd", "dBd"), grads, gr):
        errs[name] = oracle.rel_fro(from_device(g), r_)
    print("c3 chain M=%d:" % M, {k: "%.3e" % v for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= TOL_BF16, (k, v)


def test_config3_chain_shared_x():
    """The same chain with the gate and up factors side by side (one X A product, one input-gradient
    product): every output against the full oracle; dA of gate and up arrive as the two column blocks."""
    import numpy as np
    from paper_2402_13533_amd import ffn
    M, d, r, f = 320, 4096, 1024, 11008
    X, dY, W = _ffn_inputs(M, d, r, f)
    Yr, dXr, gr = _oracle_ffn(X.f64, dY.f64, W)
    Ag, Bg, Au, Bu, Ad, Bd = W
    A_gu = Bf16(np.concatenate([Ag.bits, Au.bits], axis=1)).cuda()
    Wd = [A_gu, Bg.cuda(), Bu.cuda(), Ad.cuda(), Bd.cuda()]
    Y, saved = ffn.ffn_fwd_shared_x(X.cuda(), *Wd)
    dX, (dA_gu, dBg, dBu, dAd, dBd) = ffn.ffn_bwd_shared_x(X.cuda(), *Wd, dY.cuda(), saved)
    dA_gu = from_device(dA_gu)
    got = {"Y": from_device(Y), "dX": from_device(dX), "dAg": dA_gu[:, :r], "dBg": from_device(dBg),
           "dAu": dA_gu[:, r:], "dBu": from_device(dBu), "dAd": from_device(dAd), "dBd": from_device(dBd)}
    ref = dict(zip(("dAg", "dBg", "dAu", "dBu", "dAd", "dBd"), gr), Y=Yr, dX=dXr)
    errs = {k: oracle.rel_fro(got[k], ref[k]) for k in got}
    print("c3 chain shared-x M=%d:" % M, {k: "%.3e" % v for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= TOL_BF16, (k, v)


def test_config3_full_size_sampled():
    """Config 3 at 16384 tokens: Y and dX of the whole chain on sampled rows (every step
    of the chain is row-wise independent), and each weight gradient's additivity over
    token blocks (a sum over tokens must equal the sum of its two halves).  The halves may
    run on another tile shape than the whole, which sums k in another order, so a few per
    cent of the bf16 intermediates (H, dH) differ by one ulp between the two runs: the bound
    is a fraction of the bf16 tolerance, far below what a dropped or doubled token block
    would cause (64 of 16384 tokens missing: about 6e-2)."""
    from paper_2402_13533_amd import ffn
    fhpc = _fhpc()
    M, d, r, f = 16384, 4096, 1024, 11008
    X, dY, W = _ffn_inputs(M, d, r, f, base=20)
    Wd = [w.cuda() for w in W]
    Xd, dYd = X.cuda(), dY.cuda()
    Y, saved = ffn.ffn_fwd(Xd, *Wd)
    dX, grads = ffn.ffn_bwd(Xd, *Wd, dYd, saved)
    rows = sample_rows(M, 33, 128)
    Yr, dXr, _ = _oracle_ffn(X.rows(rows).f64, dY.rows(rows).f64, W)
    eY = oracle.rel_fro(from_device(Y)[rows], Yr)
    eX = oracle.rel_fro(from_device(dX)[rows], dXr)
    print("c3 full: Y %.3e dX %.3e" % (eY, eX), flush=True)
    assert eY <= TOL_BF16 and eX <= TOL_BF16
    grads = [from_device(g) for g in grads]
    del Y, dX, saved
    h = M // 2
    parts = []
    for lo in (0, h):
        Yh, sv = ffn.ffn_fwd(Xd[lo:lo + h].contiguous(), *Wd)
        _, gh = ffn.ffn_bwd(Xd[lo:lo + h].contiguous(), *Wd, dYd[lo:lo + h].contiguous(), sv)
        parts.append([from_device(g) for g in gh])
        del Yh, sv, gh
    for name, g, a, b in zip(("dAg", "dBg", "dAu", "dBu", "dAd", "dBd"), grads, parts[0], parts[1]):
        e = oracle.rel_fro(g, a + b)
        print("c3 full additivity %s %.3e" % (name, e), flush=True)
        assert e <= 2e-3, (name, e)
