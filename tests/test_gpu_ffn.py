"""GPU parity of the SiLU gate and of the SiLU-gated FFN built from three factorised
linears (config 3), per call and end to end."""
import numpy as np
import pytest

import oracle
from harness import TOL_BF16, TOL_F32, Bf16, from_device, sample_rows, parity_err
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
    assert parity_err(from_device(Zf), oracle.swiglu_fwd(Gf, Uf)) <= TOL_F32


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
    errs = {"Y": parity_err(from_device(Y), Yr), "dX": parity_err(from_device(dX), dXr)}
    for name, g, r_ in zip(("dAg", "dBg", "dAu", "dBu", "dAd", "dBd"), grads, gr):
        errs[name] = parity_err(from_device(g), r_)
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
    errs = {k: parity_err(got[k], ref[k]) for k in got}
    print("c3 chain shared-x M=%d:" % M, {k: "%.3e" % v for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= TOL_BF16, (k, v)


def test_config3_chain_error_spread_over_seeds():
    """The chain's error is a sum over millions of independent roundings (every stored intermediate is bf16:
    H_gate/up, G, U, Z, H_down, Y on the way forward; dH_down, dZ, dG, dU, dH_gate/up, dX on the way back), so its
    relative Frobenius norm depends on how many roundings the chain has, hardly on the data: over six seeds
    the values agree to a few per cent, and the worst keeps the distance to the tolerance that the first has."""
    import numpy as np
    from paper_2402_13533_amd import ffn
    M, d, r, f = 320, 4096, 1024, 11008
    seen = {"Y": [], "dX": []}
    for seed in range(6):
        X, dY, W = _ffn_inputs(M, d, r, f, base=100 * (seed + 1))
        Yr, dXr, _ = _oracle_ffn(X.f64, dY.f64, W, want_weight_grads=False)
        Ag, Bg, Au, Bu, Ad, Bd = W
        A_gu = Bf16(np.concatenate([Ag.bits, Au.bits], axis=1)).cuda()
        Wd = [A_gu, Bg.cuda(), Bu.cuda(), Ad.cuda(), Bd.cuda()]
        Y, saved = ffn.ffn_fwd_shared_x(X.cuda(), *Wd)
        dX, _ = ffn.ffn_bwd_shared_x(X.cuda(), *Wd, dY.cuda(), saved)
        seen["Y"].append(parity_err(from_device(Y), Yr))
        seen["dX"].append(parity_err(from_device(dX), dXr))
        print("c3 chain seed %d: Y %.3e dX %.3e" % (seed, seen["Y"][-1], seen["dX"][-1]), flush=True)
    for k, v in seen.items():
        assert max(v) <= TOL_BF16, (k, v)
        assert (max(v) - min(v)) <= 0.05 * min(v), (k, v)


@pytest.mark.parametrize("M,d,r,f", [(3900, 256, 64, 4040), (300, 256, 32, 520), (4096, 512, 128, 4096), (37, 128, 8, 264),
                                     (4096, 256, 24, 4096), (4000, 128, 8, 4352)])
def test_gate_in_the_epilogue_gives_the_bits_of_the_separate_calls(M, d, r, f):
    """lowrank_ffn_gate_up_fwd and lowrank_ffn_down_bwd against the calls they stand for (shared-X forward with
    g = 2 + swiglu_fwd; lowrank_linear_bwd + swiglu_bwd): every output bit for bit, on shapes whose tiles pass the
    gate in the GEMM epilogue (256 x 256 tiles; the first with ragged edges both ways, the last two with ranks that are
    padded to the matrix instruction's depth) and on shapes that take the streaming gate kernel inside the call; outputs between guard regions.  And against the
    oracle directly."""
    import torch
    from harness import Guarded
    fhpc = _fhpc()
    X, dY, W = _ffn_inputs(M, d, r, f, base=40)
    Ag, Bg, Au, Bu, Ad, Bd = [w.cuda() for w in W]
    A_gu = torch.cat([Ag, Au], dim=1).contiguous()
    Xc, dYc = X.cuda(), dY.cuda()
    bf = torch.bfloat16
    # forward
    (G0, U0), H0 = fhpc.lowrank_linear_fwd_shared_x(Xc, A_gu, [Bg, Bu], save_H=True)
    Z0 = fhpc.swiglu_fwd(G0, U0)
    gd = Guarded()
    G1, U1, Z1, H1 = gd.alloc((M, f), bf), gd.alloc((M, f), bf), gd.alloc((M, f), bf), gd.alloc((M, 2 * r), bf)
    fhpc.lowrank_ffn_gate_up_fwd(Xc, A_gu, Bg, Bu, G=G1, U=U1, Z=Z1, H_all_out=H1)
    gd.check("gate/up forward")
    for name, a, b in (("G", G0, G1), ("U", U0, U1), ("Z", Z0, Z1), ("H", H0, H1)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), name
    # backward of the down projection
    Hd = fhpc.lowrank_linear_fwd(Z0, Ad, Bd, save_H=True)[1]
    dZ0, dAd0, dBd0 = fhpc.lowrank_linear_bwd(Z0, Ad, Bd, dYc, H_saved=Hd)
    dG0, dU0 = fhpc.swiglu_bwd(G0, U0, dZ0)
    gd = Guarded()
    dG1, dU1 = gd.alloc((M, f), bf), gd.alloc((M, f), bf)
    dAd1, dBd1 = gd.alloc((f, r), torch.float32), gd.alloc((r, d), torch.float32)
    fhpc.lowrank_ffn_down_bwd(Z0, Ad, Bd, dYc, G0, U0, H_saved=Hd, dG=dG1, dU=dU1, dA=dAd1, dB=dBd1)
    gd.check("down backward")
    assert torch.equal(dG0.view(torch.int16), dG1.view(torch.int16)), "dG"
    assert torch.equal(dU0.view(torch.int16), dU1.view(torch.int16)), "dU"
    assert torch.equal(dAd0, dAd1) and torch.equal(dBd0, dBd1)
    # without the saved H (recomputed inside the call), and with the weight gradients left out
    dG2, dU2, dAd2, dBd2 = fhpc.lowrank_ffn_down_bwd(Z0, Ad, Bd, dYc, G0, U0)
    assert torch.equal(dG0.view(torch.int16), dG2.view(torch.int16)) and torch.equal(dBd0, dBd2)
    dG3, dU3, dAd3, dBd3 = fhpc.lowrank_ffn_down_bwd(Z0, Ad, Bd, dYc, G0, U0, need_dA=False, need_dB=False)
    assert dAd3 is None and dBd3 is None
    assert torch.equal(dG0.view(torch.int16), dG3.view(torch.int16)) and torch.equal(dU0.view(torch.int16), dU3.view(torch.int16))
    # the oracle: the gate on the very tensors it was applied to (G, U and the bf16 dZ of the separate call, decoded
    # exactly), so that one bf16 rounding of an fp32 result is all that separates the two: 2^-9 relative per element;
    # the products around it against the fp64 chain
    Wf = [w.f64 for w in W]
    Gd, Ud, Zd, dZd = from_device(G0), from_device(U0), from_device(Z0), from_device(dZ0)
    dGr, dUr = oracle.swiglu_bwd(Gd, Ud, dZd)
    for name, got, ref in (("Z", Z1, oracle.swiglu_fwd(Gd, Ud)), ("dG", dG1, dGr), ("dU", dU1, dUr)):
        g = from_device(got)
        assert np.all(np.isfinite(g)), name
        assert np.all(np.abs(g - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-30), name
    Gr, _ = oracle.lowrank_fwd(X.f64, Wf[0], Wf[1])
    Ur, _ = oracle.lowrank_fwd(X.f64, Wf[2], Wf[3])
    assert parity_err(from_device(G1), Gr) <= TOL_BF16 and parity_err(from_device(U1), Ur) <= TOL_BF16
    _, dAdr, dBdr = oracle.lowrank_bwd(Zd, Wf[4], Wf[5], dY.f64)
    for name, got, ref in (("dAd", dAd1, dAdr), ("dBd", dBd1, dBdr)):
        assert parity_err(from_device(got), ref) <= TOL_BF16, name


def _oracle_ffn_full_size(X, dY, W, rows, J):
    """The oracle's chain on every token (G, U, Z, dZ, dG, dU in fp64), then: Y and dX on the token rows `rows`, and
    each weight gradient restricted to the rank indices J (column j of dA and row j of dB depend on the pair only
    through column j of A and row j of B, so the oracle runs the layer restricted to those indices).
    dZ = (dY Bd^T) Ad^T is the factorised layer's forward with the transposed pair."""
    Ag, Bg, Au, Bu, Ad, Bd = [w.f64 for w in W]
    Xf, dYf = X.f64, dY.f64
    G, _ = oracle.lowrank_fwd(Xf, Ag, Bg)
    U, _ = oracle.lowrank_fwd(Xf, Au, Bu)
    Z = oracle.swiglu_fwd(G, U)
    dZ, _ = oracle.lowrank_fwd(dYf, np.ascontiguousarray(Bd.T), np.ascontiguousarray(Ad.T))
    dG, dU = oracle.swiglu_bwd(G, U, dZ)
    del dZ
    Y, _ = oracle.lowrank_fwd(Z[rows], Ad, Bd)
    dXg, _, _ = oracle.lowrank_bwd(Xf[rows], Ag, Bg, dG[rows])
    dXu, _, _ = oracle.lowrank_bwd(Xf[rows], Au, Bu, dU[rows])
    sub = lambda A, B: (np.ascontiguousarray(A[:, J]), np.ascontiguousarray(B[J, :]))
    _, dAg, dBg = oracle.lowrank_bwd(Xf, *sub(Ag, Bg), dG)
    _, dAu, dBu = oracle.lowrank_bwd(Xf, *sub(Au, Bu), dU)
    _, dAd, dBd = oracle.lowrank_bwd(Z, *sub(Ad, Bd), dYf)
    return Y, dXg + dXu, {"dAg": dAg, "dBg": dBg, "dAu": dAu, "dBu": dBu, "dAd": dAd, "dBd": dBd}


_full_size_cache = {}


def _config3_full_size_case():
    """Inputs and oracle results of the full-size test, computed once for both routes (the fp64 chain over
    16384 tokens is about a minute of host time)."""
    if not _full_size_cache:
        M, d, r, f = 16384, 4096, 1024, 11008
        X, dY, W = _ffn_inputs(M, d, r, f, base=20)
        rows = sample_rows(M, 33, 128)
        J = np.unique(np.random.default_rng(34).integers(0, r, size=6))
        print("c3 full size: oracle chain on %d tokens ..." % M, flush=True)
        _full_size_cache["case"] = (X, dY, W, rows, J, _oracle_ffn_full_size(X, dY, W, rows, J))
        print("c3 full size: oracle done", flush=True)
    return _full_size_cache["case"]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("shared_x", [False, True])
def test_config3_full_size_sampled(shared_x):
    """Config 3 at 16384 tokens, as separate gate / up calls and through the shared-X chain the benchmark times:
    Y and dX of the whole chain on sampled rows (every step of the chain is row-wise independent) and all six
    weight gradients on sampled rank indices, against the oracle run on every token."""
    from paper_2402_13533_amd import ffn
    r = 1024
    X, dY, W, rows, J, (Yr, dXr, gr) = _config3_full_size_case()
    Ag, Bg, Au, Bu, Ad, Bd = W
    Xd, dYd = X.cuda(), dY.cuda()
    if shared_x:
        A_gu = Bf16(np.concatenate([Ag.bits, Au.bits], axis=1)).cuda()
        Wd = [A_gu, Bg.cuda(), Bu.cuda(), Ad.cuda(), Bd.cuda()]
        Y, saved = ffn.ffn_fwd_shared_x(Xd, *Wd)
        dX, (dA_gu, dBg, dBu, dAd, dBd) = ffn.ffn_bwd_shared_x(Xd, *Wd, dYd, saved)
        dA_gu = from_device(dA_gu)
        grads = {"dAg": dA_gu[:, :r], "dBg": from_device(dBg), "dAu": dA_gu[:, r:], "dBu": from_device(dBu),
                 "dAd": from_device(dAd), "dBd": from_device(dBd)}
    else:
        Wd = [w.cuda() for w in W]
        Y, saved = ffn.ffn_fwd(Xd, *Wd)
        dX, g6 = ffn.ffn_bwd(Xd, *Wd, dYd, saved)
        grads = dict(zip(("dAg", "dBg", "dAu", "dBu", "dAd", "dBd"), [from_device(g) for g in g6]))
    Y, dX = from_device(Y)[rows], from_device(dX)[rows]
    del saved
    errs = {"Y": parity_err(Y, Yr, what="Y"), "dX": parity_err(dX, dXr, what="dX")}
    for name, ref in gr.items():
        got = grads[name][:, J] if name.startswith("dA") else grads[name][J, :]
        errs[name] = parity_err(got, ref, what=name)
    print("c3 full shared_x=%s: %s" % (shared_x, {k: "%.3e" % v for k, v in errs.items()}), flush=True)
    for k, v in errs.items():
        assert v <= TOL_BF16, (k, v)
