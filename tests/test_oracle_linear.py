"""Pins for the oracle's layer algebra against definitions, brute force and special cases."""
import numpy as np

from oracle import acc_oracle as orc


def _loops_matmul(A, B):
    """Definition of a matrix product with Python integers (exact)."""
    m, k = len(A), len(A[0])
    n = len(B[0])
    return [[sum(int(A[i][t]) * int(B[t][j]) for t in range(k)) for j in range(n)] for i in range(m)]


def _ints(rng, shape, lo=-5, hi=6):
    return rng.integers(lo, hi, size=shape).astype(np.int64)


def test_forward_backward_against_integer_loops():
    """Small integer matrices of four different sizes: every operand order/transposition is exercised."""
    rng = np.random.default_rng(0)
    n, d_in, d_out, r = 7, 5, 6, 3
    X, W, dY, S = _ints(rng, (n, d_in)), _ints(rng, (d_in, d_out)), _ints(rng, (n, d_out)), _ints(rng, (n, r))
    Y, Xs = orc.linear_fwd(X, W, S=S.astype(np.float64))
    dX, Gr, dW = orc.linear_bwd(dY, W, Xs, S=S.astype(np.float64))
    assert Y.shape == (n, d_out) and Xs.shape == (d_in, r)
    assert dX.shape == (n, d_in) and Gr.shape == (r, d_out) and dW.shape == (d_in, d_out)
    assert np.array_equal(Y, np.array(_loops_matmul(X.tolist(), W.tolist()), dtype=np.float64))
    assert np.array_equal(Xs, np.array(_loops_matmul(X.T.tolist(), S.tolist()), dtype=np.float64))
    assert np.array_equal(dX, np.array(_loops_matmul(dY.tolist(), W.T.tolist()), dtype=np.float64))
    assert np.array_equal(Gr, np.array(_loops_matmul(S.T.tolist(), dY.tolist()), dtype=np.float64))
    want_dW = _loops_matmul(_loops_matmul(X.T.tolist(), S.tolist()), _loops_matmul(S.T.tolist(), dY.tolist()))
    assert np.array_equal(dW, np.array(want_dW, dtype=np.float64))


def test_identity_special_cases():
    rng = np.random.default_rng(1)
    n, d_in, d_out = 6, 6, 4
    W = rng.standard_normal((d_in, d_out))
    dY = rng.standard_normal((n, d_out))
    X = rng.standard_normal((n, d_in))
    Y, _ = orc.linear_fwd(np.eye(n), W, S=np.eye(n))
    assert np.array_equal(Y, W)                                   # X = I  ->  Y = W
    _, Xs = orc.linear_fwd(X, W, S=np.eye(n))
    assert np.array_equal(Xs, X.T)                                # S = I  ->  Xs = X^T
    dX, Gr, dW = orc.linear_bwd(dY, W, Xs, S=np.eye(n))
    assert np.array_equal(Gr, dY)                                 # S = I  ->  Gr = dY
    assert np.allclose(dW, X.T @ dY, rtol=1e-13)                  # and dW is the dense gradient
    # a single non-zero in dY picks one row of W^T
    e = np.zeros((n, d_out)); e[2, 3] = 2.0
    dX1, _, _ = orc.linear_bwd(e, W, Xs, S=np.eye(n), want_dW=False)
    assert np.array_equal(dX1[2], 2.0 * W[:, 3]) and not dX1[[0, 1, 3, 4, 5]].any()


def test_exact_with_orthogonal_sketch_at_full_rank():
    """With r = n and S orthogonal, S S^T = I: the factored gradient is the dense one."""
    rng = np.random.default_rng(2)
    n, d_in, d_out = 64, 24, 40
    X, W, dY = rng.standard_normal((n, d_in)), rng.standard_normal((d_in, d_out)), rng.standard_normal((n, d_out))
    Q, _ = np.linalg.qr(rng.standard_normal((n, n)))
    _, Xs = orc.linear_fwd(X, W, S=Q)
    _, _, dW = orc.linear_bwd(dY, W, Xs, S=Q)
    dense = X.T @ dY
    assert np.linalg.norm(dW - dense) / np.linalg.norm(dense) < 1e-13
    assert np.allclose(orc.reconstruct_activation(Xs, 0, n, n, S=Q), X, atol=1e-12)


def test_factorisation_adds_no_error_and_rank_bound():
    """Xs Gr equals (S S^T X)^T dY formed the long way (paper Sec. 4), and has rank <= r."""
    rng = np.random.default_rng(3)
    n, d_in, d_out, r, seed = 96, 40, 56, 8, 11
    X, W, dY = rng.standard_normal((n, d_in)), rng.standard_normal((d_in, d_out)), rng.standard_normal((n, d_out))
    _, Xs = orc.linear_fwd(X, W, seed, r)
    _, Gr, dW = orc.linear_bwd(dY, W, Xs, seed, r)
    Xhat = orc.reconstruct_activation(Xs, seed, n, r)
    long_way = Xhat.T @ dY
    assert np.linalg.norm(dW - long_way) / np.linalg.norm(long_way) < 1e-13
    sv = np.linalg.svd(dW, compute_uv=False)
    assert sv[r - 1] > 1e-6 * sv[0] and sv[r] < 1e-12 * sv[0]
    # rank(G_W) <= rank(X): a rank-2 activation gives a rank-2 dense gradient
    X2 = rng.standard_normal((n, 2)) @ rng.standard_normal((2, d_in))
    sv2 = np.linalg.svd(X2.T @ dY, compute_uv=False)
    assert sv2[2] < 1e-12 * sv2[0]


def test_input_gradient_is_exact_and_independent_of_compression():
    """Thm 3.2.2(a): dX does not depend on seed, rank or the stored factor."""
    rng = np.random.default_rng(4)
    n, d_in, d_out = 32, 12, 20
    W, dY = rng.standard_normal((d_in, d_out)), rng.standard_normal((n, d_out))
    ref = None
    for seed, r in [(0, 4), (1, 4), (5, 16), (9, 32)]:
        Xs = rng.standard_normal((d_in, r))
        dX, _, _ = orc.linear_bwd(dY, W, Xs, seed, r)
        ref = dX if ref is None else ref
        assert np.array_equal(dX, ref)
    assert np.allclose(ref, np.einsum("no,io->ni", dY, W), rtol=1e-13)


def test_row_offset_makes_shards_add_up():
    """Token shards with global row offsets sum to the unsharded factors (data-parallel reading)."""
    rng = np.random.default_rng(5)
    n, d_in, d_out, r, seed = 48, 10, 14, 8, 3
    X, W, dY = rng.standard_normal((n, d_in)), rng.standard_normal((d_in, d_out)), rng.standard_normal((n, d_out))
    _, Xs = orc.linear_fwd(X, W, seed, r)
    _, Xs_a = orc.linear_fwd(X[:20], W, seed, r, row_offset=0)
    _, Xs_b = orc.linear_fwd(X[20:], W, seed, r, row_offset=20)
    assert np.allclose(Xs_a + Xs_b, Xs, atol=1e-13)
    _, Gr, _ = orc.linear_bwd(dY, W, Xs, seed, r)
    _, Gr_a, _ = orc.linear_bwd(dY[:20], W, Xs, seed, r, row_offset=0)
    _, Gr_b, _ = orc.linear_bwd(dY[20:], W, Xs, seed, r, row_offset=20)
    assert np.allclose(Gr_a + Gr_b, Gr, atol=1e-13)


def test_bf16_rounding_helper():
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 3.0e38, 1e-40], dtype=np.float64)
    got = orc.round_to_bf16(vals)
    assert got[0] == 1.0
    assert got[1] == 1.0                       # tie -> even mantissa
    assert got[2] == 1.0 + 2.0 ** -6           # tie -> even mantissa (rounds up)
    assert got[3] == -2.5
    assert np.all(np.abs(got[:4] - vals[:4]) <= 2.0 ** -8 * np.abs(vals[:4]))


def test_paper_orientation_against_index_loops():
    """w_out_in: W [d_out, d_in] as in Def. 3.1 (Z = X W^T); factor and weight gradient as in Sec. 4.

    Written as index sums straight from the definitions, with Python integers.
    """
    rng = np.random.default_rng(3)
    n, d_in, d_out, r = 6, 4, 5, 3
    X, W, dY, S = _ints(rng, (n, d_in)), _ints(rng, (d_out, d_in)), _ints(rng, (n, d_out)), _ints(rng, (n, r))
    Sf = S.astype(np.float64)
    Y, Xs = orc.linear_fwd(X, W, S=Sf, w_out_in=True)
    dX, Gr, dW = orc.linear_bwd(dY, W, Xs, S=Sf, w_out_in=True)
    assert Y.shape == (n, d_out) and dX.shape == (n, d_in) and Gr.shape == (d_out, r) and dW.shape == (d_out, d_in)
    for i in range(n):
        for o in range(d_out):
            assert Y[i, o] == sum(int(X[i, c]) * int(W[o, c]) for c in range(d_in))
        for c in range(d_in):
            assert dX[i, c] == sum(int(dY[i, o]) * int(W[o, c]) for o in range(d_out))
    for o in range(d_out):
        for j in range(r):
            assert Gr[o, j] == sum(int(dY[i, o]) * int(S[i, j]) for i in range(n))
        for c in range(d_in):
            want = sum(sum(int(dY[i, o]) * int(S[i, j]) for i in range(n)) *
                       sum(int(X[i, c]) * int(S[i, j]) for i in range(n)) for j in range(r))
            assert dW[o, c] == want
    # the two orientations describe the same layer
    Y2, Xs2 = orc.linear_fwd(X, W.T, S=Sf)
    dX2, Gr2, dW2 = orc.linear_bwd(dY, W.T, Xs2, S=Sf)
    assert np.array_equal(Y, Y2) and np.array_equal(Xs, Xs2) and np.array_equal(dX, dX2)
    assert np.array_equal(Gr, Gr2.T) and np.array_equal(dW, dW2.T)


def test_bias_gradient_is_the_derivative_of_the_affine_layer():
    """Proof of Thm 3.2.2 (bias term): for Z = X W + 1 b^T and a loss whose gradient w.r.t. Z is dY,
    dL/db is the column sum of dY, whatever X is.  Checked against a central finite difference of the
    linear loss L(b) = <dY, X W + 1 b^T> (exact for a linear function up to rounding) and against
    integer loops."""
    rng = np.random.default_rng(4)
    n, d_in, d_out = 9, 4, 6
    X, W = rng.standard_normal((n, d_in)), rng.standard_normal((d_in, d_out))
    dY = rng.standard_normal((n, d_out))
    b = rng.standard_normal(d_out)
    dB = orc.bias_grad(dY)
    assert dB.shape == (d_out,)
    loss = lambda bb: float(np.sum(dY * (X @ W + bb[None, :])))
    h = 0.5
    for o in range(d_out):
        e = np.zeros(d_out); e[o] = h
        fd = (loss(b + e) - loss(b - e)) / (2 * h)
        assert abs(fd - dB[o]) < 1e-9 * (1 + abs(dB[o]))
    # independent of the activation: a different X gives the same gradient (it never enters)
    Di = _ints(rng, (5, 3))
    assert orc.bias_grad(Di).tolist() == [sum(int(Di[i, o]) for i in range(5)) for o in range(3)]
    assert orc.bias_grad(np.zeros((0, 4))).tolist() == [0.0] * 4


def test_accumulated_gradient_equals_the_product_of_stacked_factors():
    """Two micro-batches accumulated on the dense gradient: dW_1 + dW_2 = [Xs_1 Xs_2] . [Gr_1; Gr_2],
    the rank-2r factorisation of the summed estimate (Sec. 4), exact on integers."""
    rng = np.random.default_rng(5)
    d_in, d_out, r = 5, 4, 3
    total = None
    xs_all, gr_all = [], []
    for n in (6, 9):
        X, dY, S = _ints(rng, (n, d_in)), _ints(rng, (n, d_out)), _ints(rng, (n, r)).astype(np.float64)
        W = _ints(rng, (d_in, d_out))
        _, Xs = orc.linear_fwd(X, W, S=S)
        _, Gr, total = orc.linear_bwd(dY, W, Xs, S=S, dW_prev=total)
        xs_all.append(Xs); gr_all.append(Gr)
    stacked = np.array(_loops_matmul(np.hstack(xs_all).astype(np.int64).tolist(),
                                     np.vstack(gr_all).astype(np.int64).tolist()), dtype=np.float64)
    assert np.array_equal(total, stacked)
