"""Pins for the oracle's RSVD compressor (randomized range finder + projection)."""
from fractions import Fraction

import numpy as np

from oracle import acc_oracle as orc


def _gram_schmidt_exact(Y):
    """Classical Gram-Schmidt on integer columns in exact rational arithmetic; returns the orthogonal
    (not yet normalised) columns as Fractions and their squared norms."""
    n, k = len(Y), len(Y[0])
    cols = [[Fraction(Y[i][j]) for i in range(n)] for j in range(k)]
    out, norms = [], []
    for j in range(k):
        v = cols[j][:]
        for q, nq in zip(out, norms):
            c = sum(a * b for a, b in zip(cols[j], q)) / nq
            v = [a - c * b for a, b in zip(v, q)]
        out.append(v)
        norms.append(sum(a * a for a in v))
    return out, norms


def test_orthonormal_basis_matches_exact_gram_schmidt():
    """The thin QR with diag(R) > 0 is the normalised Gram-Schmidt basis: column j is the part of
    Y[:, j] orthogonal to the earlier columns, scaled to unit length, sign kept."""
    rng = np.random.default_rng(0)
    Y = rng.integers(-4, 5, size=(7, 3))
    U, R = orc.orthonormal_basis(Y.astype(np.float64))
    cols, norms = _gram_schmidt_exact(Y.tolist())
    for j in range(3):
        want = np.array([float(v) for v in cols[j]]) / np.sqrt(float(norms[j]))
        assert np.allclose(U[:, j], want, rtol=0, atol=1e-13)
        assert R[j, j] > 0
    assert np.allclose(U @ R, Y, atol=1e-12)
    assert np.allclose(np.tril(R, -1), 0)


def test_factors_are_a_projection_of_the_input():
    rng = np.random.default_rng(1)
    n, d, k = 60, 24, 6
    X = rng.standard_normal((n, d))
    U, V = orc.rsvd_factors(X, seed=3, k=k)
    assert U.shape == (n, k) and V.shape == (d, k)
    assert np.allclose(U.T @ U, np.eye(k), atol=1e-13)
    Xh = U @ V.T
    # orthogonal projection onto span(U): residual orthogonal to U, idempotent, never longer than X
    assert np.allclose(U.T @ (X - Xh), 0, atol=1e-12)
    U2, V2 = orc.rsvd_factors(Xh, seed=3, k=k)
    assert np.allclose(U2 @ V2.T, Xh, atol=1e-11)
    assert np.linalg.norm(Xh) <= np.linalg.norm(X) + 1e-12
    # span(U) = span(X Omega) with the documented Omega
    Yr = X @ orc.range_finder_matrix(3, d, k)
    assert np.allclose(U @ (U.T @ Yr), Yr, atol=1e-11)
    # a different seed gives a different subspace
    U3, _ = orc.rsvd_factors(X, seed=4, k=k)
    assert np.linalg.norm(U3 @ U3.T - U @ U.T) > 0.1


def test_exact_for_inputs_of_rank_at_most_k():
    """rank(X) <= k: the range of X Omega is the range of X (almost surely), so X^ = X and the
    factored weight gradient equals X^T dY (Sec. 4: the gradient inherits the activation's rank)."""
    rng = np.random.default_rng(2)
    n, d, d_out, k = 50, 20, 12, 5
    X = rng.standard_normal((n, 4)) @ rng.standard_normal((4, d))
    W = rng.standard_normal((d, d_out))
    dY = rng.standard_normal((n, d_out))
    Y, U, V = orc.linear_fwd_rsvd(X, W, seed=0, k=k)
    dX, Gr, dW = orc.linear_bwd_rsvd(dY, W, U, V)
    assert np.allclose(Y, X @ W) and np.allclose(dX, dY @ W.T)
    assert np.allclose(U @ V.T, X, atol=1e-10)
    assert np.allclose(dW, X.T @ dY, atol=1e-10)
    assert Gr.shape == (k, d_out) and np.linalg.matrix_rank(dW) <= k


def test_error_is_bounded_below_by_the_best_rank_k_approximation():
    """Eckart-Young: no rank-k matrix is closer to X than the truncated SVD; the randomized
    projection stays within a modest factor of it on a matrix with decaying spectrum."""
    rng = np.random.default_rng(3)
    n, d, k = 200, 64, 8
    Uo, _ = np.linalg.qr(rng.standard_normal((n, d)))
    Vo, _ = np.linalg.qr(rng.standard_normal((d, d)))
    sig = 10.0 * 0.7 ** np.arange(d)
    X = (Uo * sig) @ Vo.T
    best = np.sqrt(np.sum(sig[k:] ** 2))
    errs = []
    for seed in range(20):
        U, V = orc.rsvd_factors(X, seed=seed, k=k)
        errs.append(np.linalg.norm(X - U @ V.T))
    assert min(errs) >= best * (1 - 1e-12)
    assert np.mean(errs) < 4.0 * best
    # full rank k = d: nothing is lost
    U, V = orc.rsvd_factors(X, seed=0, k=d)
    assert np.allclose(U @ V.T, X, atol=1e-9)


def test_rsvd_error_is_far_below_random_projection_error():
    """The paper's appendix table: at equal rank the RSVD reconstruction error is 18-40x below the
    random-projection error on real activations.  On an activation-like synthetic matrix (rank-64
    signal + noise, outlier channels) the same ordering holds by a similar margin (18x and 26x here),
    and the RP error halves from rank 8 to 32 (1/sqrt(r) law) while the RSVD error depends on the spectrum."""
    rng = np.random.default_rng(4)
    n, d = 1024, 256
    X = rng.standard_normal((n, 64)) @ rng.standard_normal((64, d)) / 8.0 + 0.1 * rng.standard_normal((n, d))
    X[:, ::32] *= 20.0
    err = {}
    for k in (8, 32):
        U, V = orc.rsvd_factors(X, seed=1, k=k)
        err["rsvd", k] = np.linalg.norm(X - U @ V.T)
        S = orc.sketch_matrix(1, n, k)
        err["rp", k] = np.linalg.norm(X - S @ (S.T @ X))
    assert err["rp", 8] / err["rsvd", 8] > 5 and err["rp", 32] / err["rsvd", 32] > 5
    assert 1.7 < err["rp", 8] / err["rp", 32] < 2.3
    assert err["rsvd", 32] < err["rsvd", 8] < np.linalg.norm(X)   # more rank, less error; never worse than dropping X


def test_paper_orientation_of_rsvd_gradient_factors():
    rng = np.random.default_rng(5)
    n, d, d_out, k = 30, 10, 7, 4
    X, W, dY = rng.standard_normal((n, d)), rng.standard_normal((d, d_out)), rng.standard_normal((n, d_out))
    Y, U, V = orc.linear_fwd_rsvd(X, W, seed=2, k=k)
    dX, Gr, dW = orc.linear_bwd_rsvd(dY, W, U, V)
    Y2, U2, V2 = orc.linear_fwd_rsvd(X, W.T.copy(), seed=2, k=k, w_out_in=True)
    dX2, Gr2, dW2 = orc.linear_bwd_rsvd(dY, W.T.copy(), U2, V2, w_out_in=True)
    assert np.allclose(Y, Y2) and np.allclose(dX, dX2) and np.array_equal(U, U2) and np.array_equal(V, V2)
    assert np.allclose(Gr2, Gr.T) and np.allclose(dW2, dW.T)
    # Sec. 4 written out: G^_W = ((grad_Z L)^T U) V^T
    assert np.allclose(dW2, (dY.T @ U) @ V.T)


def test_backward_factors_against_integer_loops():
    """Gr = U^T dY and dW = V Gr with explicit integer factors, element by element (Sec. 4)."""
    rng = np.random.default_rng(6)
    n, d, d_out, k = 6, 5, 4, 3
    U = rng.integers(-3, 4, size=(n, k)); V = rng.integers(-3, 4, size=(d, k))
    dY = rng.integers(-3, 4, size=(n, d_out)); W = rng.integers(-3, 4, size=(d, d_out))
    dX, Gr, dW = orc.linear_bwd_rsvd(dY, W, U, V)
    for j in range(k):
        for o in range(d_out):
            assert Gr[j, o] == sum(int(U[i, j]) * int(dY[i, o]) for i in range(n))
    for c in range(d):
        for o in range(d_out):
            assert dW[c, o] == sum(int(V[c, j]) * sum(int(U[i, j]) * int(dY[i, o]) for i in range(n)) for j in range(k))
            # = row c of X^ = U V^T against dY
            assert dW[c, o] == sum(sum(int(U[i, j]) * int(V[c, j]) for j in range(k)) * int(dY[i, o]) for i in range(n))
    for i in range(n):
        for c in range(d):
            assert dX[i, c] == sum(int(dY[i, o]) * int(W[c, o]) for o in range(d_out))


def test_subspace_iteration_approaches_the_best_rank_k_approximation():
    """With q rounds of subspace iteration the projection error falls towards the Eckart-Young optimum
    (it can never go below it), fast when the spectrum decays; q = 0 is the plain range finder; every
    iterate is still an orthogonal projection of X; a matrix of rank <= k is reproduced for every q."""
    rng = np.random.default_rng(8)
    n, d, k = 300, 80, 10
    Uo, _ = np.linalg.qr(rng.standard_normal((n, d)))
    Vo, _ = np.linalg.qr(rng.standard_normal((d, d)))
    sig = 5.0 * 0.85 ** np.arange(d)
    X = (Uo * sig) @ Vo.T
    best = np.sqrt(np.sum(sig[k:] ** 2))
    errs = []
    for q in range(4):
        U, V = orc.rsvd_factors(X, seed=2, k=k, power_iters=q)
        assert np.allclose(U.T @ U, np.eye(k), atol=1e-12)
        assert np.allclose(U.T @ (X - U @ V.T), 0, atol=1e-10)
        errs.append(np.linalg.norm(X - U @ V.T))
    U0, V0 = orc.rsvd_factors(X, seed=2, k=k)
    assert errs[0] == np.linalg.norm(X - U0 @ V0.T)
    assert all(e >= best * (1 - 1e-12) for e in errs)
    assert errs[3] < errs[2] < errs[1] < errs[0]
    assert errs[0] > 1.5 * best and errs[1] < 1.3 * best and errs[3] < 1.1 * best   # 2.11, 1.21, 1.09, 1.06 x optimum
    # the dominant left singular subspace is what the iteration converges to
    Uk = Uo[:, :k]
    U5, _ = orc.rsvd_factors(X, seed=2, k=k, power_iters=12)
    assert np.linalg.norm(Uk @ Uk.T - U5 @ U5.T) < 0.1 * np.linalg.norm(Uk @ Uk.T - U0 @ U0.T)
    Xl = rng.standard_normal((n, 6)) @ rng.standard_normal((6, d))
    for q in (0, 1, 3):
        U, V = orc.rsvd_factors(Xl, seed=1, k=k, power_iters=q)
        assert np.allclose(U @ V.T, Xl, atol=1e-9)
