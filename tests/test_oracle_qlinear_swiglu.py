"""Pins for the oracle's finetuning layer (Sec. 5.1 eq. new_linear_layer with a
frozen quantised W) and the SiLU gate (Sec. 3.1 eq. FFN)."""
import numpy as np

import oracle

rng = np.random.default_rng(99)


def _setup(M=6, K=64, r=3, N=5, scheme=8):
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    if scheme == 8:
        Wq, sc = oracle.quantize_int8_perchannel(W)
    else:
        Wq, sc = oracle.quantize_int4_block(W, 64)
    Wd = oracle.dequant(Wq, sc, scheme, 64)
    return (rng.standard_normal((M, K)), Wd, rng.standard_normal((K, r)) / 8,
            rng.standard_normal((r, N)), rng.standard_normal((M, N)))


def test_fwd_special_cases_and_linearity():
    for scheme in (8, 4):
        X, Wd, A, B, _ = _setup(scheme=scheme)
        Y0, _ = oracle.qlinear_lowrank_fwd(X, Wd, A, B, 0.0)
        assert oracle.rel_fro(Y0, X @ Wd) < 1e-13                      # s = 0: plain base layer
        Yl, H = oracle.qlinear_lowrank_fwd(X, np.zeros_like(Wd), A, B, 1.5)
        assert oracle.rel_fro(Yl, 1.5 * oracle.lowrank_fwd(X, A, B)[0]) < 1e-13  # W = 0: low-rank branch
        assert oracle.rel_fro(H, X @ A) < 1e-13
        Y1, _ = oracle.qlinear_lowrank_fwd(X, Wd, A, B, 1.0)
        Y3, _ = oracle.qlinear_lowrank_fwd(X, Wd, A, B, 3.0)
        assert oracle.rel_fro(Y3 - Y1, 2.0 * (Y1 - Y0)) < 1e-11          # affine in s
        assert oracle.rel_fro(Y3, X @ (Wd + 3.0 * A @ B)) < 1e-12        # merged weight W' = W + s A B


def test_bwd_identities_and_no_dw():
    X, Wd, A, B, dY = _setup(M=9, K=128, r=4, N=7, scheme=4)
    s = 2.0
    dX, dA, dB = oracle.qlinear_lowrank_bwd(X, Wd, A, B, s, dY)
    assert oracle.rel_fro(dX, dY @ (Wd + s * A @ B).T) < 1e-12
    lX, lA, lB = oracle.lowrank_bwd(X, A, B, dY)
    assert oracle.rel_fro(dA, s * lA) < 1e-13 and oracle.rel_fro(dB, s * lB) < 1e-13
    dX0, dA0, dB0 = oracle.qlinear_lowrank_bwd(X, Wd, A, B, 0.0, dY)
    assert oracle.rel_fro(dX0, dY @ Wd.T) < 1e-13 and not dA0.any() and not dB0.any()


def test_bwd_finite_differences():
    X, Wd, A, B, dY = _setup(M=3, K=64, r=2, N=4, scheme=8)
    s = 2.0
    dX, dA, dB = oracle.qlinear_lowrank_bwd(X, Wd, A, B, s, dY)
    loss = lambda x, a, b: float(np.sum(oracle.qlinear_lowrank_fwd(x, Wd, a, b, s)[0] * dY))
    h = 1e-6
    for which, T, g in ((0, X, dX), (1, A, dA), (2, B, dB)):
        for idx in list(np.ndindex(*T.shape))[::3]:
            args = [X.copy(), A.copy(), B.copy()]
            args[which][idx] += h
            fp = loss(*args)
            args[which][idx] -= 2 * h
            fm = loss(*args)
            assert abs((fp - fm) / (2 * h) - g[idx]) <= 2e-7 * max(1.0, abs(g[idx]))


def test_swiglu_values_limits_and_fd():
    G = np.array([0.0, 1.0, -1.0, 40.0, -40.0, 800.0, -800.0])
    U = np.array([3.0, 2.0, 2.0, 0.5, 0.5, 1.0, 1.0])
    Z = oracle.swiglu_fwd(G, U)
    assert Z[0] == 0.0
    assert np.isclose(Z[1], 2.0 / (1 + np.exp(-1.0)), rtol=1e-15)
    assert np.isclose(Z[2], -2.0 / (1 + np.exp(1.0)), rtol=1e-15)
    assert np.isclose(Z[3], 20.0, rtol=1e-15) and abs(Z[4]) < 1e-15       # sigma -> 1 / 0
    assert Z[5] == 800.0 and Z[6] == 0.0 and np.all(np.isfinite(Z))       # no overflow
    dZ = np.ones_like(G)
    dG, dU = oracle.swiglu_bwd(G, U, dZ)
    assert dG[0] == 1.5 and dU[0] == 0.0                                   # G = 0: dG = dZ U / 2
    assert np.all(np.isfinite(dG)) and np.all(np.isfinite(dU))
    g = rng.standard_normal(50) * 3
    u = rng.standard_normal(50)
    dz = rng.standard_normal(50)
    dG, dU = oracle.swiglu_bwd(g, u, dz)
    h = 1e-6
    fdG = (oracle.swiglu_fwd(g + h, u) - oracle.swiglu_fwd(g - h, u)) / (2 * h) * dz
    fdU = (oracle.swiglu_fwd(g, u + h) - oracle.swiglu_fwd(g, u - h)) / (2 * h) * dz
    assert np.allclose(dG, fdG, rtol=1e-7, atol=1e-8) and np.allclose(dU, fdU, rtol=1e-7, atol=1e-8)
