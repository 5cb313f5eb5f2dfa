"""Pins for the oracle's rank-r factorisation of a pretrained weight (Sec. 4.1 item 2: W is
decomposed into A[K,r], B[r,N]; reading: the best rank-r approximation, factors balanced)."""
import numpy as np

import oracle

rng = np.random.default_rng(1618)


def test_diagonal_closed_form():
    # singular values are the absolute diagonal entries; the rank-2 cut keeps the two largest
    W = np.diag([3.0, -5.0, 1.0, 0.5])[:, :3]                  # 4 x 3: columns e1*3, e2*(-5), e3*1
    A, B, s = oracle.lowrank_factorize(W, 2)
    assert np.allclose(s, [5.0, 3.0, 1.0], atol=1e-14)
    expect = W.copy()
    expect[2, 2] = 0.0
    assert np.allclose(A @ B, expect, atol=1e-14)
    assert A.shape == (4, 2) and B.shape == (2, 3)


def test_exact_rank_is_recovered_and_rank_one_by_hand():
    K, r, N = 23, 4, 17
    W = rng.standard_normal((K, r)) @ rng.standard_normal((r, N))
    A, B, s = oracle.lowrank_factorize(W, r)
    assert oracle.rel_fro(A @ B, W) < 1e-13 and np.all(s[r:] < 1e-12 * s[0])
    # rank one: W = u v^T has the single singular value |u| |v|
    u, v = rng.standard_normal(9), rng.standard_normal(6)
    A1, B1, s1 = oracle.lowrank_factorize(np.outer(u, v), 1)
    assert abs(s1[0] - np.linalg.norm(u) * np.linalg.norm(v)) < 1e-13
    assert oracle.rel_fro(A1 @ B1, np.outer(u, v)) < 1e-13


def test_error_is_the_tail_of_the_spectrum_and_no_pair_beats_it():
    K, N, r = 30, 22, 5
    W = rng.standard_normal((K, N))
    A, B, s = oracle.lowrank_factorize(W, r)
    # singular values from a different routine: eigenvalues of W^T W
    ev = np.sort(np.linalg.eigvalsh(W.T @ W))[::-1]
    assert np.allclose(s ** 2, ev[: len(s)], rtol=1e-10, atol=1e-12)
    err2 = np.sum((W - A @ B) ** 2)
    assert abs(err2 - np.sum(ev[r:])) < 1e-10 * np.sum(ev)
    # Eckart-Young: least-squares fits on random r-dimensional column spaces are never better
    for _ in range(20):
        Q, _ = np.linalg.qr(rng.standard_normal((K, r)))
        assert np.sum((W - Q @ (Q.T @ W)) ** 2) >= err2 * (1 - 1e-12)
    # nor are small perturbations of the optimum
    for _ in range(20):
        A2 = A + 1e-3 * rng.standard_normal(A.shape)
        B2 = np.linalg.lstsq(A2, W, rcond=None)[0]
        assert np.sum((W - A2 @ B2) ** 2) >= err2 * (1 - 1e-12)


def test_factors_are_balanced_and_orientation():
    K, N, r = 12, 40, 3
    W = rng.standard_normal((K, N))
    A, B, s = oracle.lowrank_factorize(W, r)
    assert A.shape == (K, r) and B.shape == (r, N)
    assert np.allclose(A.T @ A, np.diag(s[:r]), atol=1e-12)
    assert np.allclose(B @ B.T, np.diag(s[:r]), atol=1e-12)
    # the transposed weight swaps the roles of the factors
    At, Bt, st = oracle.lowrank_factorize(W.T, r)
    assert np.allclose(st, s, atol=1e-12) and oracle.rel_fro(At @ Bt, (A @ B).T) < 1e-12
    # the layer built from the pair is the layer of the cut weight
    X = rng.standard_normal((7, K))
    Y, _ = oracle.lowrank_fwd(X, A, B)
    assert oracle.rel_fro(Y, X @ (A @ B)) < 1e-13
