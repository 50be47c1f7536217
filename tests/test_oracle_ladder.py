"""Pins for the oracle's ladder builder (Sec. III-C: the rank ladder comes from one SVD of the adapter
update; a rung slices its first r directions): closed-form cases, the defining identities of an SVD, and
the optimality of every truncation."""
import numpy as np
import pytest


def test_two_by_two_closed_form(oracle):
    # dW = [[3, 0], [4, 5]]: dW^T dW has eigenvalues 45 and 5
    A = np.array([[3.0, 0.0], [4.0, 5.0]], np.float32)
    A2, B2, sigma = oracle.build_ladder(A, np.eye(2, dtype=np.float32))
    np.testing.assert_allclose(sigma, [np.sqrt(45.0), np.sqrt(5.0)], rtol=1e-14)
    np.testing.assert_allclose(A2 @ B2, A, atol=1e-14)
    # leading direction of this matrix: u1 = (1, 3)/sqrt(10), v1 = (1, 1)/sqrt(2)
    P1 = np.sqrt(45.0) * np.outer([1, 3], [1, 1]) / np.sqrt(20.0)
    np.testing.assert_allclose(A2[:, :1] @ B2[:1, :], P1, atol=1e-13)


def test_diagonal_factors_are_sorted_and_split_evenly(oracle):
    # A = first r columns of a permutation scaled by a, B = rows scaled by b: sigma = a*b sorted
    a = np.array([2.0, 0.5, 3.0, 1.0], np.float32)
    b = np.array([1.0, 8.0, 0.5, 0.25], np.float32)
    A = np.zeros((6, 4), np.float32)
    B = np.zeros((4, 5), np.float32)
    for i in range(4):
        A[i + 1, i] = a[i]
        B[i, 4 - i] = b[i]
    A2, B2, sigma = oracle.build_ladder(A, B)
    want = np.sort(a.astype(np.float64) * b)[::-1]
    np.testing.assert_allclose(sigma, want, rtol=1e-14)
    order = np.argsort(-(a.astype(np.float64) * b), kind="stable")
    for k, i in enumerate(order):
        # direction k is e_{i+1} on the input side and e_{4-i} on the output side, each carrying sqrt(sigma)
        assert abs(abs(A2[i + 1, k]) - np.sqrt(want[k])) < 1e-13 and abs(abs(B2[k, 4 - i]) - np.sqrt(want[k])) < 1e-13
        assert np.count_nonzero(np.abs(A2[:, k]) > 1e-13) == 1 and np.count_nonzero(np.abs(B2[k, :]) > 1e-13) == 1


@pytest.mark.parametrize("d_in,d_out,r,seed", [(40, 30, 8, 0), (17, 64, 5, 1), (64, 9, 12, 2), (50, 50, 16, 3)])
def test_svd_identities_and_optimal_truncations(oracle, d_in, d_out, r, seed):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((d_in, r)).astype(np.float32)
    B = rng.standard_normal((r, d_out)).astype(np.float32)
    A2, B2, sigma = oracle.build_ladder(A, B)
    W = A.astype(np.float64) @ B.astype(np.float64)
    n = min(r, d_in, d_out)
    assert np.all(np.diff(sigma) <= 0) and np.all(sigma >= 0)
    np.testing.assert_allclose(A2 @ B2, W, atol=1e-12 * sigma[0])
    # orthogonal directions carrying sqrt(sigma) on each side
    np.testing.assert_allclose(A2.T @ A2, np.diag(sigma), atol=1e-12 * sigma[0])
    np.testing.assert_allclose(B2 @ B2.T, np.diag(sigma), atol=1e-12 * sigma[0])
    # sigma^2 are the eigenvalues of the r x r matrix (A^T A)(B B^T), by a different library routine
    ev = np.sort(np.linalg.eigvals((A.T.astype(np.float64) @ A) @ (B.astype(np.float64) @ B.T)).real)[::-1]
    np.testing.assert_allclose(sigma[:n] ** 2, ev[:n], rtol=1e-9)
    for k in range(1, r + 1):
        Pk = A2[:, :k] @ B2[:k, :]
        # Eckart-Young: the error of the best rank-k approximation is the tail of the spectrum
        assert abs(np.linalg.norm(W - Pk) ** 2 - np.sum(sigma[k:] ** 2)) <= 1e-10 * sigma[0] ** 2
        # and no random rank-k matrix of the same column space does better
        Q = np.linalg.qr(rng.standard_normal((d_in, k)))[0]
        assert np.linalg.norm(W - Q @ (Q.T @ W)) >= np.linalg.norm(W - Pk) - 1e-9


def test_rank_deficient_update(oracle):
    rng = np.random.default_rng(5)
    A = rng.standard_normal((20, 6)).astype(np.float32)
    B = rng.standard_normal((6, 15)).astype(np.float32)
    B[3:] = 0                                  # rows a fresh adapter still has at zero
    A2, B2, sigma = oracle.build_ladder(A, B)
    assert np.all(sigma[:3] > 0) and np.all(sigma[3:] == 0)
    assert np.all(A2[:, 3:] == 0) and np.all(B2[3:] == 0)
    np.testing.assert_allclose(A2 @ B2, A.astype(np.float64) @ B, atol=1e-12)
    A2, B2, sigma = oracle.build_ladder(A, np.zeros_like(B))
    assert np.all(sigma == 0) and np.all(A2 == 0) and np.all(B2 == 0)
