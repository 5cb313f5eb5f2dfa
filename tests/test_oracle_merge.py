"""Pins for the oracle's merged weight (Sec. 5.1, eq. new_linear_layer: the adapted layer's weight
W' = W + Delta W with Delta W the product of the factor pair, built once for inference)."""
import numpy as np

import oracle

rng = np.random.default_rng(2718)


def test_hand_worked_case():
    # K = 2, r = 1, N = 3:  A B = [[2], [-1]] [[1, 0, 3]] = [[2, 0, 6], [-1, 0, -3]]
    W = np.array([[10.0, 20.0, 30.0], [40.0, 50.0, 60.0]])
    A = np.array([[2.0], [-1.0]])
    B = np.array([[1.0, 0.0, 3.0]])
    assert np.array_equal(oracle.merge(W, A, B, 1.0), [[12.0, 20.0, 36.0], [39.0, 50.0, 57.0]])
    assert np.array_equal(oracle.merge(W, A, B, -2.0), [[6.0, 20.0, 18.0], [42.0, 50.0, 66.0]])
    assert np.array_equal(oracle.merge(None, A, B, 1.0), [[2.0, 0.0, 6.0], [-1.0, 0.0, -3.0]])
    # r = 2 with a second, axis-aligned term: only element (1, 1) moves, by 5 * 7
    A2 = np.array([[2.0, 0.0], [-1.0, 5.0]])
    B2 = np.array([[1.0, 0.0, 3.0], [0.0, 7.0, 0.0]])
    assert np.array_equal(oracle.merge(W, A2, B2, 1.0), [[12.0, 20.0, 36.0], [39.0, 85.0, 57.0]])


def test_rank_one_closed_form_nonsquare():
    K, N = 9, 14
    W = rng.standard_normal((K, N))
    a = rng.standard_normal(K)
    b = rng.standard_normal(N)
    Wp = oracle.merge(W, a[:, None], b[None, :], 0.75)
    for k in range(K):
        for n in range(N):
            assert abs(Wp[k, n] - (W[k, n] + 0.75 * a[k] * b[n])) < 1e-14


def test_merged_weight_gives_the_adapted_layer():
    # the defining identity: (W + Delta W) x = W x + B A x, for every x
    M, K, r, N = 11, 24, 5, 16
    X = rng.standard_normal((M, K))
    W = rng.standard_normal((K, N)) / 4
    A = rng.standard_normal((K, r)) / 4
    B = rng.standard_normal((r, N))
    for s in (1.0, 0.125, -3.0):
        Y, _ = oracle.qlinear_lowrank_fwd(X, W, A, B, s)
        assert oracle.rel_fro(X @ oracle.merge(W, A, B, s), Y) < 1e-13
    Y0, _ = oracle.lowrank_fwd(X, A, B)
    assert oracle.rel_fro(X @ oracle.merge(None, A, B, 1.0), Y0) < 1e-13
    assert np.array_equal(oracle.merge(W, A, B, 0.0), W)


def test_update_has_rank_r_and_is_linear_in_each_factor():
    K, r, N = 30, 4, 26
    W = rng.standard_normal((K, N))
    A = rng.standard_normal((K, r))
    B = rng.standard_normal((r, N))
    sv = np.linalg.svd(oracle.merge(W, A, B, 1.0) - W, compute_uv=False)
    assert sv[r - 1] > 1e-3 and sv[r] < 1e-12 * sv[0]
    A2 = rng.standard_normal((K, r))
    lhs = oracle.merge(None, A + 2 * A2, B, 1.0)
    assert oracle.rel_fro(lhs, oracle.merge(None, A, B, 1.0) + 2 * oracle.merge(None, A2, B, 1.0)) < 1e-13
    # transposing the whole product swaps the roles of the factors
    assert oracle.rel_fro(oracle.merge(None, B.T, A.T, 1.0), oracle.merge(None, A, B, 1.0).T) < 1e-14
