"""Pins for the oracle's blend layer (Sec. 4.1 item 3: y = alpha W x + (1 - alpha) B A x with
the pretrained W frozen)."""
import numpy as np

import oracle

rng = np.random.default_rng(314)


def _setup(M=7, K=20, r=3, N=6):
    return (rng.standard_normal((M, K)), rng.standard_normal((K, N)) / 4, rng.standard_normal((K, r)) / 4,
            rng.standard_normal((r, N)), rng.standard_normal((M, N)))


def test_end_points_and_convexity():
    X, W, A, B, _ = _setup()
    Y1, H = oracle.blend_fwd(X, W, A, B, 1.0)
    assert oracle.rel_fro(Y1, X @ W) < 1e-13                            # alpha = 1: the pretrained layer
    assert oracle.rel_fro(H, X @ A) < 1e-13
    Y0, _ = oracle.blend_fwd(X, W, A, B, 0.0)
    assert oracle.rel_fro(Y0, oracle.lowrank_fwd(X, A, B)[0]) < 1e-13   # alpha = 0: the factorised layer
    for alpha in (0.25, 0.9):
        Ya, _ = oracle.blend_fwd(X, W, A, B, alpha)
        assert oracle.rel_fro(Ya, alpha * Y1 + (1 - alpha) * Y0) < 1e-13
        assert oracle.rel_fro(Ya, X @ (alpha * W + (1 - alpha) * A @ B)) < 1e-12   # one merged weight
        # the same layer written as the finetuning layer: base alpha W, branch scaling 1 - alpha
        Yq, _ = oracle.qlinear_lowrank_fwd(X, alpha * W, A, B, 1 - alpha)
        assert oracle.rel_fro(Ya, Yq) < 1e-13


def test_bwd_identities_and_no_dw():
    X, W, A, B, dY = _setup(M=9, K=16, r=4, N=7)
    alpha = 0.3
    dX, dA, dB = oracle.blend_bwd(X, W, A, B, alpha, dY)
    assert oracle.rel_fro(dX, dY @ (alpha * W + (1 - alpha) * A @ B).T) < 1e-12
    lX, lA, lB = oracle.lowrank_bwd(X, A, B, dY)
    assert oracle.rel_fro(dA, (1 - alpha) * lA) < 1e-13 and oracle.rel_fro(dB, (1 - alpha) * lB) < 1e-13
    dX1, dA1, dB1 = oracle.blend_bwd(X, W, A, B, 1.0, dY)
    assert oracle.rel_fro(dX1, dY @ W.T) < 1e-13 and not dA1.any() and not dB1.any()
    dX0, dA0, dB0 = oracle.blend_bwd(X, W, A, B, 0.0, dY)
    assert oracle.rel_fro(dX0, lX) < 1e-13 and oracle.rel_fro(dA0, lA) < 1e-13 and oracle.rel_fro(dB0, lB) < 1e-13


def test_bwd_finite_differences():
    X, W, A, B, dY = _setup(M=3, K=5, r=2, N=4)
    alpha = 0.6
    dX, dA, dB = oracle.blend_bwd(X, W, A, B, alpha, dY)
    loss = lambda x, a, b: float(np.sum(oracle.blend_fwd(x, W, a, b, alpha)[0] * dY))
    h = 1e-6
    for which, T, g in ((0, X, dX), (1, A, dA), (2, B, dB)):
        for idx in np.ndindex(*T.shape):
            args = [X.copy(), A.copy(), B.copy()]
            args[which][idx] += h
            fp = loss(*args)
            args[which][idx] -= 2 * h
            fm = loss(*args)
            assert abs((fp - fm) / (2 * h) - g[idx]) <= 2e-7 * max(1.0, abs(g[idx]))
