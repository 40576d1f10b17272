"""Pins for the oracle against what the paper's theorems fix (Monte Carlo over seeds)."""
import numpy as np
import pytest

from oracle import acc_oracle as orc
from paper_2605_01255_amd import inputs
from conftest import golden_path


@pytest.fixture(scope="module")
def c1():
    lin = inputs.config("c1")[0]
    d = inputs.make(lin)
    return lin, inputs.as_f64(d["X"]), inputs.as_f64(d["W"]), inputs.as_f64(d["dY"])


@pytest.fixture(scope="module")
def monte_carlo(c1):
    """1000 seeds of the factored weight gradient at the tiny configuration."""
    lin, X, W, dY = c1
    dense = X.T @ dY
    running = np.zeros_like(dense)
    sq_err = []
    mean_err = {}
    for seed in range(1000):
        S = orc.sketch_matrix(seed, lin.n, lin.r)
        _, Xs = orc.linear_fwd(X, W, S=S)
        _, _, dW = orc.linear_bwd(dY, W, Xs, S=S)
        sq_err.append(np.sum((dW - dense) ** 2))
        running += dW
        if seed + 1 in (10, 100, 1000):
            mean_err[seed + 1] = np.linalg.norm(running / (seed + 1) - dense)
    return dense, np.array(sq_err), mean_err


def test_unbiased_weight_gradient(c1, monte_carlo):
    """Thm 3.2.1(a): the seed average converges to X^T dY at the 1/sqrt(N) rate."""
    lin, X, W, dY = c1
    dense, sq_err, mean_err = monte_carlo
    cf = orc.closed_form_variance(X, dY, lin.r)
    for N, err in mean_err.items():
        predicted = np.sqrt(cf / N)
        assert 0.9 < err / predicted < 1.1, (N, err, predicted)
    # a single seed is far off (the estimator is noisy, not wrong)
    assert np.sqrt(sq_err[0]) / np.linalg.norm(dense) > 1.0


def test_variance_matches_gaussian_closed_form(c1, monte_carlo):
    """Thm 3.3.1 per-layer term E||G_Z^T dX||_F^2 equals (||X||^2 ||dY||^2 + ||X^T dY||^2) / r."""
    lin, X, W, dY = c1
    _, sq_err, _ = monte_carlo
    cf = orc.closed_form_variance(X, dY, lin.r)
    assert abs(sq_err.mean() / cf - 1.0) < 0.015, sq_err.mean() / cf


def test_activation_error_law_and_paper_rank_ratio(c1):
    """E||(S S^T - I) X||_F^2 = (n + 1) ||X||_F^2 / r; so the error scales as 1/sqrt(r).

    The paper's RP error table prints rank-8 / rank-32 ratios near sqrt(32 / 8) = 2.
    """
    lin, X, W, dY = c1
    n = lin.n
    x2 = np.sum(X * X)
    rms = {}
    for r in (8, 32):
        errs = []
        for seed in range(200):
            S = orc.sketch_matrix(seed, n, r)
            errs.append(np.sum((S @ (S.T @ X) - X) ** 2))
        assert abs(np.mean(errs) / ((n + 1) * x2 / r) - 1.0) < 0.02
        rms[r] = np.sqrt(np.mean(errs))
    ours = rms[8] / rms[32]
    assert abs(ours - 2.0) < 0.03
    paper = []
    for line in open(golden_path("rp_error_table.txt")):
        line = line.split("#")[0].split()
        if line:
            paper.append(float(line[1]) / float(line[2]))
    assert len(paper) == 4
    assert min(paper) - 0.05 < ours < max(paper) + 0.05       # paper: 1.89 .. 2.06


def test_dense_products_match_definition(c1):
    """Y and dX at the tiny configuration against an independent einsum formulation."""
    lin, X, W, dY = c1
    Y, Xs = orc.linear_fwd(X, W, 0, lin.r)
    dX, Gr, dW = orc.linear_bwd(dY, W, Xs, 0, lin.r)
    assert np.allclose(Y, np.einsum("nk,ko->no", X, W), rtol=1e-12, atol=1e-14)
    assert np.allclose(dX, np.einsum("no,ko->nk", dY, W), rtol=1e-12, atol=1e-16)
    S = orc.sketch_matrix(0, lin.n, lin.r)
    assert np.allclose(Xs, np.einsum("nk,nr->kr", X, S), rtol=1e-12, atol=1e-14)
    assert np.allclose(Gr, np.einsum("nr,no->ro", S, dY), rtol=1e-12, atol=1e-16)
    assert np.allclose(dW, np.einsum("kr,ro->ko", Xs, Gr), rtol=1e-12, atol=1e-16)
