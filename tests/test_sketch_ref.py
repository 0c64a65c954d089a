"""Pins of oracle/sketch_ref.py (Eq. 13) against what linear algebra fixes: exact recovery of a rank-1 matrix,
convergence to the library SVD's leading triples under a spectral gap, the deflation invariants, the it = 0 closed
form, the Eckart-Young bound, and planted mistakes."""
import numpy as np
import pytest

from oracle.sketch_ref import sketch_lowrank


def _spectrum_matrix(rng, rows, cols, sv):
    A, _ = np.linalg.qr(rng.standard_normal((rows, len(sv))))
    B, _ = np.linalg.qr(rng.standard_normal((cols, len(sv))))
    return (A * np.asarray(sv)) @ B.T, A, B


def test_rank_one_matrix_is_recovered_exactly():
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal(12), rng.standard_normal(20)
    W = np.outer(a, b)
    S = rng.standard_normal((2, 20))
    U, sig, V, R = sketch_lowrank(W, 2, 1, S)
    sgn = np.sign(U[0] @ a)
    assert np.allclose(U[0], sgn * a / np.linalg.norm(a), atol=1e-12)
    assert np.allclose(V[0], sgn * b / np.linalg.norm(b), atol=1e-12)
    assert abs(sig[0] - np.linalg.norm(a) * np.linalg.norm(b)) < 1e-10
    assert np.max(np.abs(R)) < 1e-10 * np.max(np.abs(W))


def test_converges_to_the_leading_singular_triples_under_a_gap():
    rng = np.random.default_rng(2)
    sv = [100.0, 30.0, 9.0, 2.0, 0.5, 0.1]
    W, A, B = _spectrum_matrix(rng, 40, 60, sv)
    S = rng.standard_normal((3, 60))
    U, sig, V, R = sketch_lowrank(W, 3, 12, S)
    Ul, sl, Vl = np.linalg.svd(W, full_matrices=False)
    for i in range(3):
        assert abs(sig[i] - sl[i]) < 1e-6 * sl[0]
        assert abs(abs(U[i] @ Ul[:, i]) - 1.0) < 1e-8
        assert abs(abs(V[i] @ Vl[i]) - 1.0) < 1e-8
        assert np.sign(U[i] @ Ul[:, i]) == np.sign(V[i] @ Vl[i])        # U Sigma V reproduces the triple, sign included
    assert abs(np.linalg.norm(R) - np.sqrt(sum(s * s for s in sv[3:]))) < 1e-6 * sv[0]


def test_deflation_invariants_and_reconstruction():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((17, 24))
    S = rng.standard_normal((5, 24))
    U, sig, V, R = sketch_lowrank(W, 5, 2, S)
    assert np.allclose(np.linalg.norm(U, axis=1), 1.0) and np.allclose(np.linalg.norm(V, axis=1), 1.0)
    # W = sum U Sigma V + residual, exactly
    assert np.allclose((U.T * sig) @ V + R, W, atol=1e-12)
    # each deflation removes the whole component along its U: the left vectors are mutually orthogonal and the
    # residual has nothing left along any of them
    assert np.max(np.abs(U @ U.T - np.eye(5))) < 1e-10
    assert np.max(np.abs(U @ R)) < 1e-10
    # Sigma V = U^T (matrix before that deflation): the first one against the input
    assert np.allclose(sig[0] * V[0], U[0] @ W, atol=1e-12)
    # Eckart-Young: no rank-5 approximation beats the SVD's
    opt = np.sqrt(np.sum(np.linalg.svd(W, compute_uv=False)[5:] ** 2))
    assert np.linalg.norm(R) >= opt - 1e-12
    assert np.linalg.norm(R) <= 1.5 * opt


def test_no_iterations_is_the_plain_sketch():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((9, 16))
    s = rng.standard_normal((1, 16))
    U, sig, V, _ = sketch_lowrank(W, 1, 0, s)
    q = W @ s[0]
    assert np.allclose(U[0], q / np.linalg.norm(q))
    assert np.allclose(sig[0] * V[0], (q / np.linalg.norm(q)) @ W)


def test_more_iterations_never_hurt_a_decaying_spectrum():
    rng = np.random.default_rng(5)
    W, _, _ = _spectrum_matrix(rng, 30, 30, [2.0 ** -i for i in range(12)])
    W = W + 1e-3 * rng.standard_normal(W.shape)
    S = rng.standard_normal((4, 30))
    errs = [np.linalg.norm(sketch_lowrank(W, 4, it, S)[3]) for it in (0, 1, 3, 8)]
    assert errs[0] >= errs[1] >= errs[2] >= errs[3] - 1e-12
    opt = np.sqrt(np.sum(np.linalg.svd(W, compute_uv=False)[4:] ** 2))
    assert errs[3] <= 1.01 * opt


def test_rank_deficient_matrix_yields_zero_vectors():
    rng = np.random.default_rng(6)
    W = np.outer(rng.standard_normal(6), rng.standard_normal(8))
    U, sig, V, R = sketch_lowrank(W, 3, 0, rng.standard_normal((3, 8)))
    # after the first deflation only rounding noise is left: its Sigma is 1e-15 of the first
    assert sig[1] < 1e-12 * sig[0] and sig[2] < 1e-12 * sig[0]


@pytest.mark.parametrize("mistake", ["transpose", "no_deflation", "sigma_without_normalisation"])
def test_planted_mistakes_fail_the_pins(mistake):
    rng = np.random.default_rng(7)
    W = rng.standard_normal((10, 14))
    S = rng.standard_normal((2, 14))
    U, sig, V, R = sketch_lowrank(W, 2, 1, S)
    if mistake == "transpose":           # Q^T W confused with W Q
        bad_p = W @ (W.T @ U[0])
        assert not np.allclose(bad_p[:10], sig[0] * V[0][:10])
    elif mistake == "no_deflation":      # second rank computed on the undeflated matrix is not orthogonal to the first
        q = W @ (W.T @ (W @ S[1]))
        u2 = q / np.linalg.norm(q)
        assert abs(u2 @ U[0]) > 1e-3 and abs(U[1] @ U[0]) < 1e-10
    else:                                # Sigma = |Q^T W| without the division by |Q|
        q = W @ (W.T @ (W @ S[0]))
        assert abs(np.linalg.norm(q @ W) - sig[0]) > 1e-3 * sig[0]
