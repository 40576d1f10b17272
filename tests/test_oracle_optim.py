"""Pins of the oracle's low-rank optimizer step (Sec. 4, update strategy (ii)) against things other than itself:
torch's own AdamW, a closed form, and the dense optimizer it must reduce to."""
import numpy as np
import torch

from oracle import acc_oracle as orc


def _factors(seed, d_in=24, d_out=40, r=8):
    g = np.random.default_rng(seed)
    return (g.standard_normal((d_in, d_out)) * 0.05, g.standard_normal((d_in, r)), g.standard_normal((r, d_out)))


def test_moments_and_normalised_step_match_torch_adamw_on_the_small_factor():
    # torch.optim.AdamW on a zero parameter of Gr's shape, no weight decay: after each step the parameter has
    # moved by -lr * N, so N is read off the library's own arithmetic for five consecutive gradients.
    r, d_out, lr = 8, 40, 1e-2
    g = np.random.default_rng(3)
    p = torch.zeros(r, d_out, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=lr, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.0)
    M = np.zeros((r, d_out)); V = np.zeros((r, d_out))
    W = np.zeros((4, d_out)); left = np.zeros((4, r))
    for t in range(1, 6):
        Gr = g.standard_normal((r, d_out)) * (0.3 ** t)       # shrinking gradients: the history matters
        before = p.detach().clone().numpy()
        p.grad = torch.from_numpy(Gr.copy())
        opt.step()
        n_lib = -(p.detach().numpy() - before) / lr
        _, M, V, N = orc.lowrank_adamw_step(W, left, Gr, M, V, step=t, lr=lr, beta1=0.8, beta2=0.95, eps=1e-6)
        st = opt.state[p]
        np.testing.assert_allclose(M, st["exp_avg"].numpy(), rtol=1e-12, atol=0)
        np.testing.assert_allclose(V, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=0)
        np.testing.assert_allclose(N, n_lib, rtol=1e-9, atol=1e-12)


def test_first_step_from_zero_state_is_sign_descent_through_the_left_factor():
    # step 1, zero moments, eps = 0: M^ = Gr, V^ = Gr^2, so N = sign(Gr) and W moves by -lr * scale * left . sign(Gr)
    W, left, Gr = _factors(5)
    z = np.zeros_like(Gr)
    W1, M1, V1, N = orc.lowrank_adamw_step(W, left, Gr, z, z, step=1, lr=0.01, beta1=0.9, beta2=0.999, eps=0.0,
                                           scale=0.25)
    np.testing.assert_allclose(N, np.sign(Gr), rtol=1e-12)
    want = np.empty_like(W)
    for i in range(W.shape[0]):            # index loops: the orientation of left . N
        for o in range(W.shape[1]):
            want[i, o] = W[i, o] - 0.01 * 0.25 * sum(left[i, k] * np.sign(Gr[k, o]) for k in range(left.shape[1]))
    np.testing.assert_allclose(W1, want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(M1, 0.1 * Gr, rtol=1e-12)
    np.testing.assert_allclose(V1, 0.001 * Gr * Gr, rtol=1e-9)


def test_identity_left_factor_reduces_to_dense_adamw_with_decoupled_weight_decay():
    # r = d_in and left = I: the factored gradient is the dense one, so three steps must follow torch's AdamW
    # on W itself, weight decay included.
    d, d_out, lr, wd = 12, 20, 3e-3, 0.1
    g = np.random.default_rng(11)
    W = g.standard_normal((d, d_out))
    p = torch.tensor(W.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=lr, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
    M = np.zeros((d, d_out)); V = np.zeros((d, d_out))
    for t in range(1, 4):
        G = g.standard_normal((d, d_out))
        p.grad = torch.from_numpy(G.copy())
        opt.step()
        W, M, V, _ = orc.lowrank_adamw_step(W, np.eye(d), G, M, V, step=t, lr=lr, weight_decay=wd)
        np.testing.assert_allclose(W, p.detach().numpy(), rtol=1e-10, atol=1e-13)


def test_square_orthogonal_projector_is_adamw_in_rotated_coordinates():
    # P = Q square orthogonal: Z = Q^T W follows dense AdamW with gradients Q^T G (weight decay commutes with Q),
    # and W = Q Z.  The gradient arrives factored, G = left . Gr, and is never formed by the oracle call.
    d, d_out, r, lr, wd = 10, 14, 6, 5e-3, 0.05
    g = np.random.default_rng(21)
    Q, _ = np.linalg.qr(g.standard_normal((d, d)))
    W = g.standard_normal((d, d_out))
    z = torch.tensor(Q.T @ W, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([z], lr=lr, betas=(0.9, 0.99), eps=1e-7, weight_decay=wd)
    M = np.zeros((d, d_out)); V = np.zeros((d, d_out))
    for t in range(1, 5):
        left, Gr = g.standard_normal((d, r)), g.standard_normal((r, d_out))
        z.grad = torch.from_numpy(Q.T @ (left @ Gr))
        opt.step()
        W, M, V, _ = orc.lowrank_adamw_step(W, left, Gr, M, V, step=t, lr=lr, beta1=0.9, beta2=0.99, eps=1e-7,
                                            weight_decay=wd, P=Q)
        np.testing.assert_allclose(W, Q @ z.detach().numpy(), rtol=1e-9, atol=1e-12)


def test_thin_projector_moves_the_weight_only_inside_its_range():
    # k < d_in: the update lies in range(P), and the projected gradient is P^T (left . Gr) entry by entry
    d, d_out, r, k = 12, 9, 6, 3
    g = np.random.default_rng(22)
    P, _ = np.linalg.qr(g.standard_normal((d, k)))
    W, left, Gr = g.standard_normal((d, d_out)), g.standard_normal((d, r)), g.standard_normal((r, d_out))
    z = np.zeros((k, d_out))
    W1, M1, _, _ = orc.lowrank_adamw_step(W, left, Gr, z, z, step=1, lr=0.01, beta1=0.5, P=P)
    dWt = W1 - W
    np.testing.assert_allclose(P @ (P.T @ dWt), dWt, rtol=1e-10, atol=1e-14)
    want_R = np.array([[sum(P[c, a] * sum(left[c, j] * Gr[j, o] for j in range(r)) for c in range(d))
                        for o in range(d_out)] for a in range(k)])
    np.testing.assert_allclose(M1, 0.5 * want_R, rtol=1e-10, atol=1e-14)


def test_gradient_projector_spans_the_gradients_range():
    g = np.random.default_rng(23)
    d, d_out, r = 40, 30, 8
    left, Gr = g.standard_normal((d, r)), g.standard_normal((r, d_out))
    G = left @ Gr
    # k = r: exactly the range of the factored gradient, which is also what its r leading singular vectors span
    P = orc.gradient_projector(left, Gr, seed=5, k=r)
    np.testing.assert_allclose(P.T @ P, np.eye(r), atol=1e-12)
    np.testing.assert_allclose(P @ (P.T @ G), G, rtol=1e-9, atol=1e-11)
    U = np.linalg.svd(G)[0][:, :r]
    np.testing.assert_allclose(P @ P.T, U @ U.T, atol=1e-10)
    # rank(G) = 3 < k = 4 <= r: still the whole range
    Gr3 = g.standard_normal((r, 3)) @ g.standard_normal((3, d_out))
    P4 = orc.gradient_projector(left, Gr3, seed=5, k=4)
    np.testing.assert_allclose(P4[:, :3] @ (P4[:, :3].T @ (left @ Gr3)), left @ Gr3, rtol=1e-8, atol=1e-10)
    # k < rank: orthonormal, inside the range, first column along G . Omega[:, 0] with a positive coefficient
    P2 = orc.gradient_projector(left, Gr, seed=5, k=2)
    np.testing.assert_allclose(P2.T @ P2, np.eye(2), atol=1e-12)
    np.testing.assert_allclose(U @ (U.T @ P2), P2, atol=1e-10)
    Om = orc.range_finder_matrix(5, d_out, 2)
    y0 = G @ Om[:, 0]
    np.testing.assert_allclose(P2[:, 0], y0 / np.linalg.norm(y0), rtol=1e-10, atol=1e-13)
    # the paper's orientation of Gr gives the same projector
    np.testing.assert_allclose(orc.gradient_projector(left, Gr.T, seed=5, k=2, w_out_in=True), P2, atol=1e-14)
    # an explicit Omega replaces the seeded one
    np.testing.assert_allclose(orc.gradient_projector(left, Gr, seed=0, k=2, Omega=Om), P2, atol=1e-14)


def test_paper_orientation_is_the_transpose():
    W, left, Gr = _factors(7)
    g = np.random.default_rng(8)
    M = g.standard_normal(Gr.shape) * 0.1
    V = g.random(Gr.shape) * 0.1
    kw = dict(step=4, lr=0.02, beta1=0.7, beta2=0.9, eps=1e-5, weight_decay=0.05, scale=2.0)
    a = orc.lowrank_adamw_step(W, left, Gr, M, V, **kw)
    b = orc.lowrank_adamw_step(W.T, left, Gr.T, M.T, V.T, w_out_in=True, **kw)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y.T, rtol=1e-13, atol=1e-15)
    P, _ = np.linalg.qr(g.standard_normal((left.shape[0], 4)))
    Mk, Vk = M[:4], V[:4]
    a = orc.lowrank_adamw_step(W, left, Gr, Mk, Vk, P=P, **kw)
    b = orc.lowrank_adamw_step(W.T, left, Gr.T, Mk.T, Vk.T, w_out_in=True, P=P, **kw)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y.T, rtol=1e-13, atol=1e-15)


def test_a_rescaled_gradient_leaves_the_first_step_unchanged():
    # Adam's normalisation: with eps = 0 the first step does not depend on the gradient's scale
    W, left, Gr = _factors(9)
    z = np.zeros_like(Gr)
    a = orc.lowrank_adamw_step(W, left, Gr, z, z, step=1, lr=0.01, eps=0.0)[0]
    b = orc.lowrank_adamw_step(W, left, 1e3 * Gr, z, z, step=1, lr=0.01, eps=0.0)[0]
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-15)
