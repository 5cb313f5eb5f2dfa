"""Pins for the oracle's factorised linear layer (Sec. 3.2 eq. low_rank_layer and
its matrix-calculus backward).  Nothing here calls the HIP library."""
import numpy as np
import pytest

import oracle

rng = np.random.default_rng(1234)


def _rand(*shape):
    return rng.standard_normal(shape)


@pytest.mark.parametrize("M,K,r,N", [(7, 13, 3, 11), (33, 64, 8, 40), (5, 6, 6, 9)])
def test_fwd_other_association_and_numpy(M, K, r, N):
    X, A, B = _rand(M, K), _rand(K, r), _rand(r, N)
    Y, H = oracle.lowrank_fwd(X, A, B)
    W = A @ B                      # dense weight the pair stands for
    assert oracle.rel_fro(Y, X @ W) < 1e-12
    assert oracle.rel_fro(H, X @ A) < 1e-13
    assert oracle.rel_fro(Y, (X @ A) @ B) < 1e-13


def test_fwd_identity_special_cases():
    M, K, N = 9, 12, 10
    X = _rand(M, K)
    B = _rand(K, N)
    Y, H = oracle.lowrank_fwd(X, np.eye(K), B)      # A = I  => Y = X B, H = X
    assert np.array_equal(H, X)
    assert oracle.rel_fro(Y, X @ B) < 1e-13
    A = _rand(K, 4)
    Y, H = oracle.lowrank_fwd(X, A, np.eye(4))      # B = I  => Y = X A
    assert np.array_equal(Y, H)
    assert oracle.rel_fro(Y, X @ A) < 1e-13


def test_fwd_rank_bound_and_non_commuting_shapes():
    M, K, r, N = 40, 30, 5, 35
    Y, _ = oracle.lowrank_fwd(_rand(M, K), _rand(K, r), _rand(r, N))
    sv = np.linalg.svd(Y, compute_uv=False)
    assert sv[r - 1] > 1e-6 and sv[r] < 1e-10 * sv[0]


def test_fwd_single_entry_indexing():
    # one-hot operands catch a transposed operand or a swapped index
    M, K, r, N = 4, 5, 3, 6
    X = np.zeros((M, K)); X[2, 4] = 2.0
    A = np.zeros((K, r)); A[4, 1] = 3.0
    B = np.zeros((r, N)); B[1, 5] = 5.0
    Y, H = oracle.lowrank_fwd(X, A, B)
    expY = np.zeros((M, N)); expY[2, 5] = 30.0
    expH = np.zeros((M, r)); expH[2, 1] = 6.0
    assert np.array_equal(Y, expY) and np.array_equal(H, expH)


@pytest.mark.parametrize("M,K,r,N", [(6, 9, 2, 7), (31, 48, 8, 24)])
def test_bwd_dense_identities(M, K, r, N):
    X, A, B, dY = _rand(M, K), _rand(K, r), _rand(r, N), _rand(M, N)
    dX, dA, dB = oracle.lowrank_bwd(X, A, B, dY)
    W = A @ B
    dW = X.T @ dY                               # gradient of the dense layer Y = X W
    assert oracle.rel_fro(dX, dY @ W.T) < 1e-12
    assert oracle.rel_fro(dA, dW @ B.T) < 1e-12  # chain rule through W = A B
    assert oracle.rel_fro(dB, A.T @ dW) < 1e-12


def test_bwd_finite_differences():
    M, K, r, N = 3, 5, 2, 4
    X, A, B, dY = _rand(M, K), _rand(K, r), _rand(r, N), _rand(M, N)
    dX, dA, dB = oracle.lowrank_bwd(X, A, B, dY)

    def loss(X_, A_, B_):
        return float(np.sum(oracle.lowrank_fwd(X_, A_, B_)[0] * dY))

    h = 1e-6
    for name, T, g in (("X", X, dX), ("A", A, dA), ("B", B, dB)):
        for idx in np.ndindex(*T.shape):
            Tp, Tm = T.copy(), T.copy()
            Tp[idx] += h
            Tm[idx] -= h
            args_p = {"X": X, "A": A, "B": B}; args_p[name] = Tp
            args_m = {"X": X, "A": A, "B": B}; args_m[name] = Tm
            fd = (loss(args_p["X"], args_p["A"], args_p["B"]) -
                  loss(args_m["X"], args_m["A"], args_m["B"])) / (2 * h)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


def test_bwd_adjoint():
    # <dY, J v> == <J^T dY, v> for the Jacobian w.r.t. each argument (the map is
    # linear in each argument separately)
    M, K, r, N = 20, 24, 4, 18
    X, A, B, dY = _rand(M, K), _rand(K, r), _rand(r, N), _rand(M, N)
    dX, dA, dB = oracle.lowrank_bwd(X, A, B, dY)
    vX, vA, vB = _rand(M, K), _rand(K, r), _rand(r, N)
    f = lambda x, a, b: oracle.lowrank_fwd(x, a, b)[0]
    assert np.isclose(np.sum(dY * f(vX, A, B)), np.sum(dX * vX), rtol=1e-11)
    assert np.isclose(np.sum(dY * f(X, vA, B)), np.sum(dA * vA), rtol=1e-11)
    assert np.isclose(np.sum(dY * f(X, A, vB)), np.sum(dB * vB), rtol=1e-11)
