"""Plain CPU fp64 oracle of the compressed linear layer.  TEST INFRASTRUCTURE ONLY.

What it computes (spec notation; the paper's is in brackets):

  forward   Y  = X . W                exact output            [Def. 3.1: Z = X W^T]
            Xs = X^T . S              stored low-rank factor  [Sec. 4: V of X^ = U V^T, with U = S]
  backward  dX = dY . W^T             exact input gradient    [Def. 3.1: G_X = (grad_Z L) W; Thm 3.2.2(a)]
            Gr = S^T . dY             small gradient factor   [Sec. 4: ((grad_Z L)^T U)^T]
            dW = Xs . Gr              factored weight grad    [Sec. 4: G^_W = ((grad_Z L)^T U) V^T, transposed]
            dB = 1^T . dY             bias gradient, exact    [proof of Thm 3.2.2, bias term]
  update    W <- W - lr P . Adam(P^T left Gr)   optimizer strategy (ii), states at the projected size  [Sec. 4]
  With w_out_in=True W, Gr and dW are in the paper's own orientation ([d_out, d_in], [d_out, r]).

S is the n x r random-projection compressor (the paper's "RP" option, Experimental
Setup) taken along the token axis with i.i.d. N(0, 1/r) entries, so that
E[S S^T] = I and the reconstructed activation S S^T X is unbiased, the premise of
Thm 3.2.1(a).  The paper does not define RP's matrix, axis, scaling or random
number generator; the readings used here are:

  * integers: Philox4x32-10 (Salmon et al., SC'11), key = (seed low word, seed high word),
    counter = (g >> 2 low word, column j, stream id 0, g >> 34) with g = row_offset + i
    the global token index; the four output words belong to tokens 4q..4q+3 of column j;
  * uniform:  u = ((x >> 9) + 0.5) * 2^-23, exactly representable in fp32 and fp64;
  * normal:   Box-Muller on the word pairs (x0, x1) and (x2, x3):
              z_even = R cos(theta), z_odd = R sin(theta), R = sqrt(-2 ln u_first),
              theta = 2 pi u_second;  S[i, j] = z / sqrt(r).

Everything after the integer stream is fp64 and unrounded.  Matrix products are
numpy's matmul on float64 (a library primitive used as one step); nothing is
blocked, fused or reordered.  The optional *_rounded helpers round S, Xs and Gr to
bfloat16 where the GPU path does, to separate quantisation from mistakes.

Pins (tests/test_oracle_*.py): published Philox known answers; Box-Muller polar
identities and normal moments / KS distance; integer matrices against pure-Python
loops; exactness with an orthogonal S at r = n; Monte-Carlo unbiasedness
(Thm 3.2.1(a)); the Gaussian-sketch variance closed form (Thm 3.3.1 per-layer
term); the 1/sqrt(r) error law matching the paper's RP error table; dX independent
of seed and rank (Thm 3.2.2(a)); the bias gradient against a finite difference of the
affine layer's loss; the [d_out, d_in] orientation against index loops in the paper's form;
the RSVD factors against exact-fraction Gram-Schmidt, exact recovery of low-rank inputs, the
Eckart-Young lower bound and the projection identities; the low-rank optimizer step against torch's AdamW
run on a parameter of the small factor's shape, the sign-descent closed form of its first step, dense
AdamW when the left factor is the identity and AdamW in rotated coordinates when the projector is a square
orthogonal matrix; the gradient projector through orthonormality, the range identities at full and at
deficient rank, and the sign convention.  No function here is "parity unpinned"; what the pins of
lowrank_adamw_step fix is the arithmetic of the stated reading, the reading itself is not in the paper.
"""
from __future__ import annotations

import numpy as np

PHILOX_M0 = 0xD2511F53
PHILOX_M1 = 0xCD9E8D57
PHILOX_W0 = 0x9E3779B9
PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds (Salmon et al., SC'11).

    counter: uint32 array [..., 4]; key: uint32 array broadcastable to [..., 2].
    Returns uint32 array [..., 4].
    """
    c = np.asarray(counter, dtype=np.uint64)
    k = np.asarray(key, dtype=np.uint64)
    c0, c1, c2, c3 = (c[..., t] for t in range(4))
    k0 = np.broadcast_to(k[..., 0], c0.shape).copy()
    k1 = np.broadcast_to(k[..., 1], c0.shape).copy()
    for _ in range(10):
        p0 = np.uint64(PHILOX_M0) * c0          # 32 x 32 -> 64 bit products
        p1 = np.uint64(PHILOX_M1) * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + np.uint64(PHILOX_W0)) & _MASK32
        k1 = (k1 + np.uint64(PHILOX_W1)) & _MASK32
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def sketch_words(seed: int, row_offset: int, n: int, r: int, stream: int = 0):
    """The integer stream behind S: uint32 [ceil(n/4), r, 4].

    Entry [q, j, w] is output word w of the Philox call for token group q
    (global tokens row_offset + 4q .. +3) and sketch column j.
    """
    if row_offset % 4:
        raise ValueError("row_offset must be a multiple of 4")
    nq = (n + 3) // 4
    g4 = (np.uint64(row_offset) >> np.uint64(2)) + np.arange(nq, dtype=np.uint64)
    ctr = np.zeros((nq, r, 4), dtype=np.uint64)
    ctr[..., 0] = (g4 & _MASK32)[:, None]
    ctr[..., 1] = np.arange(r, dtype=np.uint64)[None, :]
    ctr[..., 2] = np.uint64(stream)
    ctr[..., 3] = (g4 >> np.uint64(32))[:, None]          # (g >> 34) of the token index
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint64)
    return philox4x32_10(ctr, key)


def uniform_from_word(x):
    """u = ((x >> 9) + 0.5) 2^-23, strictly inside (0, 1)."""
    x = np.asarray(x, dtype=np.uint32)
    return ((x >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def normals_from_words(words):
    """Box-Muller on word pairs: uint32 [..., 4] -> float64 [..., 4] standard normals."""
    u = uniform_from_word(words)
    z = np.empty(u.shape, dtype=np.float64)
    for a in (0, 2):
        radius = np.sqrt(-2.0 * np.log(u[..., a]))
        theta = 2.0 * np.pi * u[..., a + 1]
        z[..., a] = radius * np.cos(theta)
        z[..., a + 1] = radius * np.sin(theta)
    return z


def sketch_matrix(seed: int, n: int, r: int, row_offset: int = 0):
    """S: float64 [n, r], entries N(0, 1/r)."""
    z = normals_from_words(sketch_words(seed, row_offset, n, r))      # [nq, r, 4]
    z = np.transpose(z, (0, 2, 1)).reshape(-1, r)[:n]                 # token = 4q + w
    return z / np.sqrt(float(r))


def linear_fwd(X, W, seed: int = 0, r: int = 0, row_offset: int = 0, S=None, w_out_in: bool = False):
    """Y = X W (exact), Xs = X^T S (the stored factor).

    w_out_in: W is given as [d_out, d_in], the paper's own orientation (Def. 3.1: Z = X W^T).
    """
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    if S is None:
        S = sketch_matrix(seed, X.shape[0], r, row_offset)
    Y = np.matmul(X, W.T) if w_out_in else np.matmul(X, W)
    Xs = np.matmul(X.T, S)
    return Y, Xs


def linear_bwd(dY, W, Xs, seed: int = 0, r: int = 0, row_offset: int = 0, S=None,
               want_dW: bool = True, w_out_in: bool = False, dW_prev=None):
    """dX = dY W^T (exact), Gr = S^T dY, dW = Xs Gr (optional).

    dW_prev: a dense gradient accumulated over earlier micro-batches (Sec. 4, update strategy (i):
    the full gradient is reconstructed before the optimizer sees it); the new product is added to it.

    w_out_in: W is [d_out, d_in] and the gradient side follows the paper's orientation (Sec. 4):
    the factor is (grad_Z L)^T U = dY^T S, [d_out, r], and the weight gradient is
    G^_W = (dY^T S) (X^T S)^T, [d_out, d_in] like W.
    """
    dY = np.asarray(dY, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Xs = np.asarray(Xs, dtype=np.float64)
    if S is None:
        S = sketch_matrix(seed, dY.shape[0], r, row_offset)
    if w_out_in:
        dX = np.matmul(dY, W)
        Gr = np.matmul(dY.T, S)
        dW = np.matmul(Gr, Xs.T) if want_dW else None
    else:
        dX = np.matmul(dY, W.T)
        Gr = np.matmul(S.T, dY)
        dW = np.matmul(Xs, Gr) if want_dW else None
    if dW is not None and dW_prev is not None:
        dW = np.asarray(dW_prev, dtype=np.float64) + dW
    return dX, Gr, dW


# ---------------------------------------------------------------------------------------------
# RSVD compressor (Experimental Setup: randomized SVD of Halko, Martinsson and Tropp; Sec. 4: the
# compressed activation is stored as two factors, X^ = U V^T with U [n, k] and V [d_in, k]).
# The paper gives no parameters beyond the rank; the reading used here is the basic randomized range
# finder followed by the projection onto it, with no oversampling, no power iteration and no final
# rotation to singular vectors (a rotation inside the k-dimensional subspace changes neither X^ nor
# the gradient estimate); optional rounds of subspace iteration sharpen the range (rsvd_factors):
#   Omega [d_in, k] Gaussian (same Philox map as S, the channel index in place of the token index),
#   Yr = X Omega,  Yr = U R with U^T U = I and diag(R) > 0 (thin QR, unique for full column rank),
#   V = X^T U,     X^ = U V^T = U U^T X,
#   Gr = U^T dY,   dW = V Gr = X^^T dY.
# Unlike S S^T X this estimator is a projection, not unbiased; its error is bounded below by the
# best rank-k approximation error.
# ---------------------------------------------------------------------------------------------
def range_finder_matrix(seed: int, d_in: int, k: int):
    """Omega [d_in, k]: i.i.d. normals addressed by (seed, channel, column); the scale is irrelevant."""
    return sketch_matrix(seed, d_in, k, 0)


def orthonormal_basis(Yr):
    """Thin QR with positive diagonal of R (numpy's Householder QR as the library step, signs fixed)."""
    Q, R = np.linalg.qr(np.asarray(Yr, dtype=np.float64), mode="reduced")
    sign = np.where(np.diag(R) < 0, -1.0, 1.0)
    return Q * sign[None, :], R * sign[:, None]


def rsvd_factors(X, seed: int, k: int, Omega=None, power_iters: int = 0):
    """U [n, k], V [d_in, k] of the RSVD-compressed activation X^ = U V^T.

    power_iters = q > 0 adds q rounds of subspace iteration (Halko et al., randomized subspace
    iteration: the basis is re-orthonormalised after every product, which is what keeps the small
    singular directions from being lost to rounding):  Z = orth(X^T U),  U = orth(X Z).
    The range approaches the dominant k-dimensional left singular subspace of X as q grows.
    """
    X = np.asarray(X, dtype=np.float64)
    if Omega is None:
        Omega = range_finder_matrix(seed, X.shape[1], k)
    U, _ = orthonormal_basis(np.matmul(X, Omega))
    for _ in range(power_iters):
        Z, _ = orthonormal_basis(np.matmul(X.T, U))
        U, _ = orthonormal_basis(np.matmul(X, Z))
    V = np.matmul(X.T, U)
    return U, V


def linear_fwd_rsvd(X, W, seed: int = 0, k: int = 0, Omega=None, w_out_in: bool = False, power_iters: int = 0):
    """Y = X W (exact) and the stored factors U, V of the RSVD-compressed input."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Y = np.matmul(X, W.T) if w_out_in else np.matmul(X, W)
    U, V = rsvd_factors(X, seed, k, Omega, power_iters)
    return Y, U, V


def linear_bwd_rsvd(dY, W, U, V, want_dW: bool = True, w_out_in: bool = False):
    """dX = dY W^T (exact), Gr = U^T dY [k, d_out], dW = V Gr (Sec. 4: ((grad_Z L)^T U) V^T, transposed)."""
    dY = np.asarray(dY, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dX = np.matmul(dY, W) if w_out_in else np.matmul(dY, W.T)
    Gr = np.matmul(U.T, dY)
    dW = np.matmul(V, Gr) if want_dW else None
    if w_out_in:
        Gr = Gr.T
        dW = dW.T if dW is not None else None
    return dX, Gr, dW


def bias_grad(dY):
    """Gradient of a bias b [d_out] broadcast over tokens, Z = X W^T + 1 b^T (proof of Thm 3.2.2,
    bias term): the loss gradient w.r.t. the added term is grad_Z L itself, independent of X and
    therefore exact under compression; summed over the tokens that share b it is the column sum of dY.
    """
    return np.sum(np.asarray(dY, dtype=np.float64), axis=0)


def gradient_projector(left, Gr, seed: int, k: int, Omega=None, w_out_in: bool = False):
    """Projector P [d_in, k] of the low-rank optimizer (Sec. 4, update strategy (ii)): an orthonormal basis
    of a k-dimensional subspace of the range of the factored gradient G^_W = left . Gr [d_in, d_out], found
    without forming it: randomized range finder (Halko et al.) on the factors,

        Yp = left . (Gr . Omega),  Omega [d_out, k] i.i.d. normals addressed by (seed, output channel, column),
        P  = the orthonormal factor of the thin QR of Yp, diagonal of the triangular factor positive.

    The scheme the paper points to takes the leading k left singular vectors of the gradient; for k = r (and in
    general whenever rank(G^_W) <= k) both span exactly range(G^_W), otherwise the range finder's subspace
    captures it up to the usual randomized-SVD error.  The basis within the subspace differs (QR instead of
    singular vectors); the paper fixes neither.
    """
    left, Gr = np.asarray(left, dtype=np.float64), np.asarray(Gr, dtype=np.float64)
    if w_out_in:
        Gr = Gr.T
    if Omega is None:
        Omega = range_finder_matrix(seed, Gr.shape[1], k)
    P, _ = orthonormal_basis(np.matmul(left, np.matmul(Gr, Omega)))
    return P


def lowrank_adamw_step(W, left, Gr, M, V, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999,
                       eps: float = 1e-8, weight_decay: float = 0.0, scale: float = 1.0, w_out_in: bool = False,
                       P=None):
    """Optimizer strategy (ii) of Sec. 4: the update is taken from the factored gradient, with the optimizer
    states kept in a compressed low-rank form.  The paper names the scheme (the low-rank projected Adam of
    Zhao et al., ICML 2024) and gives no formulas; the reading used here is that scheme applied to the two
    factors the backward pass returns, G^_W = left . Gr, never forming their product:

        R  = P^T G^_W = (P^T left) . Gr                  projected gradient, [k, d_out]; P [d_in, k] is held
                                                         fixed between refreshes (gradient_projector)
        M <- beta1 M + (1 - beta1) R                     first moment,  [k, d_out]
        V <- beta2 V + (1 - beta2) R o R                 second moment, [k, d_out]
        N  = (M / (1 - beta1^step)) / (sqrt(V / (1 - beta2^step)) + eps)      step counted from 1
        W <- (1 - lr weight_decay) W - lr scale (P . N)                       decoupled weight decay

    P=None takes the left factor itself as the projector (k = r, R = Gr, step direction left . N): the cheapest
    form, whose moments live in the basis of the current batch's compressor.
    With w_out_in the operands are in the paper's orientation: W [d_out, d_in], Gr [d_out, r], M / V / N
    [d_out, k], and the last line reads W <- (1 - lr weight_decay) W - lr scale (N . P^T).
    Returns (W_new, M_new, V_new, N), all float64.
    """
    W, left, Gr, M, V = (np.asarray(a, dtype=np.float64) for a in (W, left, Gr, M, V))
    if w_out_in:
        W, Gr, M, V = W.T, Gr.T, M.T, V.T
    if P is None:
        back, R = left, Gr
    else:
        back = np.asarray(P, dtype=np.float64)
        R = np.matmul(np.matmul(back.T, left), Gr)
    M_new = beta1 * M + (1.0 - beta1) * R
    V_new = beta2 * V + (1.0 - beta2) * R * R
    m_hat = M_new / (1.0 - beta1 ** step)
    v_hat = V_new / (1.0 - beta2 ** step)
    N = m_hat / (np.sqrt(v_hat) + eps)
    W_new = (1.0 - lr * weight_decay) * W - lr * scale * np.matmul(back, N)
    if w_out_in:
        return W_new.T, M_new.T, V_new.T, N.T
    return W_new, M_new, V_new, N


def reconstruct_activation(Xs, seed: int, n: int, r: int, row_offset: int = 0, S=None):
    """X^ = U V^T = S Xs^T (Def. 3.1), only used by the invariants."""
    if S is None:
        S = sketch_matrix(seed, n, r, row_offset)
    return np.matmul(S, np.asarray(Xs, dtype=np.float64).T)


def round_to_bf16(a):
    """Round-to-nearest-even to bfloat16, returned as float64 (diagnostic mode only)."""
    f = np.asarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def linear_fwd_rounded(X, W, seed: int, r: int, row_offset: int = 0):
    """Diagnostic: as linear_fwd, with S and Xs rounded to bf16 where the bf16 GPU path rounds."""
    S = round_to_bf16(sketch_matrix(seed, np.asarray(X).shape[0], r, row_offset))
    Y, Xs = linear_fwd(X, W, S=S)
    return round_to_bf16(Y), round_to_bf16(Xs)


def closed_form_variance(X, dY, r: int):
    """E||Xs Gr - X^T dY||_F^2 for a Gaussian sketch: (||X||^2 ||dY||^2 + ||X^T dY||^2) / r.

    This is the per-layer compression term of Thm 3.3.1 evaluated for the RP compressor.
    """
    X = np.asarray(X, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    G = np.matmul(X.T, dY)
    return (np.sum(X * X) * np.sum(dY * dY) + np.sum(G * G)) / float(r)
