"""GPU path vs oracle at the benchmark configurations' full sizes, in the launch configuration
bench.py times: whole outputs where the oracle finishes in seconds (the 3B-shaped projection),
otherwise on sampled rows / channels / columns the oracle computes one by one (fixed sample seed)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2605_01255_amd import inputs
from oracle import acc_oracle as orc
import gpu_util as gu


@pytest.fixture(scope="module")
def acc():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_01255_amd import binding
    return binding


def test_c2_full_outputs(acc):
    """LLaMA-3B-shaped attention projection, every element of every output."""
    lin = inputs.config("c2")[0]
    data = inputs.make(lin)
    got = gu.run_layer(acc, lin, data)
    want = gu.run_oracle(lin, data)
    gu.check_outputs(got, want, 1e-2, lin.name)
    # the x20 outlier channels dominate ||Xs||: check them and the ordinary channels separately
    out_ch = inputs.outlier_channels(lin.d_in, lin.n_outliers)
    rest = np.setdiff1d(np.arange(lin.d_in), out_ch)
    assert gu.rel(got["Xs"][out_ch], want["Xs"][out_ch]) <= 1e-2
    assert gu.rel(got["Xs"][rest], want["Xs"][rest]) <= 1e-2
    assert gu.rel(got["dW"][rest], want["dW"][rest]) <= 1e-2


def _sampled_check(acc, lin, rng):
    """Outputs the oracle can compute piece by piece: 256 random token rows of Y and dX plus three whole
    256 x 256 output tiles of each (the first, a random one, the last: the unit a work-group writes), 64 random
    and the last 64 channels of Xs, 64 random and the last 64 columns of Gr, and the matching block of dW.  Every
    piece is held to the full bar (whole piece, every 32 x 32 block, every element)."""
    data = inputs.make(lin)
    got = gu.run_layer(acc, lin, data)
    X, W, dY = (inputs.as_f64(data[k]) for k in ("X", "W", "dY"))
    S = orc.sketch_matrix(lin.seed, lin.n, lin.r)
    rows = np.sort(rng.choice(lin.n, size=min(256, lin.n), replace=False))
    chs = np.union1d(rng.choice(lin.d_in - 64, size=64, replace=False), np.arange(lin.d_in - 64, lin.d_in))
    cols = np.union1d(rng.choice(lin.d_out - 64, size=64, replace=False), np.arange(lin.d_out - 64, lin.d_out))
    Y_rows, _ = orc.linear_fwd(X[rows], W, S=S[rows])
    dX_rows, _, _ = orc.linear_bwd(dY[rows], W, np.zeros((lin.d_in, lin.r)), S=S[rows], want_dW=False)
    _, Xs_ch = orc.linear_fwd(X[:, chs], W[chs][:, :8], S=S)                       # [128, r]
    _, Gr_cols, dW_blk = orc.linear_bwd(dY[:, cols], W[:8][:, cols], Xs_ch, S=S)   # [r, 128], [128, 128]
    have = {"Y": got["Y"][rows], "dX": got["dX"][rows], "Xs": got["Xs"][chs], "Gr": got["Gr"][:, cols],
            "dW": got["dW"][np.ix_(chs, cols)]}
    want = {"Y": Y_rows, "dX": dX_rows, "Xs": Xs_ch, "Gr": Gr_cols, "dW": dW_blk}

    def tile_slices(extent_m, extent_n):
        tm, tn = -(-extent_m // 256), -(-extent_n // 256)
        picks = {(0, 0), (int(rng.integers(tm)), int(rng.integers(tn))), (tm - 1, tn - 1)}
        return [(slice(a * 256, min(extent_m, a * 256 + 256)), slice(b * 256, min(extent_n, b * 256 + 256)))
                for a, b in sorted(picks)]
    for i, (rs, cs) in enumerate(tile_slices(lin.n, lin.d_out)):
        have[f"Y.tile{i}"], want[f"Y.tile{i}"] = got["Y"][rs, cs], X[rs] @ W[:, cs]
    for i, (rs, cs) in enumerate(tile_slices(lin.n, lin.d_in)):
        have[f"dX.tile{i}"], want[f"dX.tile{i}"] = got["dX"][rs, cs], dY[rs] @ W[cs].T
    gu.check_outputs(have, want, 1e-2, f"{lin.name} r={lin.r}")
    # invariants that hold at any size: S^T S structure shows up as ||Gr||^2 ~ ||dY||^2 (1/r per column pair)
    ratio = np.sum(got["Gr"] ** 2) / np.sum(dY ** 2)
    assert 0.9 < ratio < 1.1, ratio


@pytest.mark.parametrize("name", ["c4.k", "c4.gate", "c4.down"])
def test_c4_linears_sampled(acc, name):
    """Decoder-layer linears of the 3B shape (k/v 3072->1024, gate/up 3072->8192, down 8192->3072)."""
    lin = [l for l in inputs.config("c4") if l.name == name][0]
    _sampled_check(acc, lin, np.random.default_rng(1))


@pytest.mark.parametrize("r", [64, 128, 512])
def test_c3_down_ranks_sampled(acc, r):
    """MLP down-projection (SwiGLU input) at the other ranks of the rank sweep."""
    lin = [l for l in inputs.config(f"c3_r{r}") if l.name == "c3.down"][0]
    _sampled_check(acc, lin, np.random.default_rng(2))


@pytest.mark.parametrize("r", [64, 512])
def test_c3_gate_ranks_sampled(acc, r):
    """MLP gate projection (3072 -> 8192) at the ends of the rank sweep."""
    lin = [l for l in inputs.config(f"c3_r{r}") if l.name == "c3.gate"][0]
    _sampled_check(acc, lin, np.random.default_rng(6))


@pytest.mark.parametrize("name", ["c5.q", "c5.k", "c5.gate", "c5.down"])
def test_c5_linears_sampled(acc, name):
    """8B-shaped layer, n = 65536 tokens, r = 512, low-rank-plus-noise activations; the MLP linears have an
    intermediate width of 14336 (the down projection's input is 1.88 GB)."""
    lin = [l for l in inputs.config("c5") if l.name == name][0]
    _sampled_check(acc, lin, np.random.default_rng(3))


def test_operands_beyond_two_gib_sampled(acc):
    """X and dX of 2.3 GB each: byte offsets inside one operand exceed 2^31 (the kernels address with
    per-tile 64-bit bases plus unsigned 32-bit offsets); ragged token count."""
    lin = inputs.Linear("big_x", 140003, 8192, 1024, 128, x_kind="plain")
    assert lin.n * lin.d_in * 2 > 2 ** 31
    _sampled_check(acc, lin, np.random.default_rng(4))


def test_c5_q_rsvd_rank32_sampled(acc):
    """RSVD compressor at the 8B-shaped q projection (n = 65536, 4096 -> 4096) and the paper's rank 32: the
    factors U, V, Gr and dW whole (their oracle products are thin), the exact products Y and dX on sampled rows."""
    import dataclasses
    import torch
    lin = dataclasses.replace([l for l in inputs.config("c5") if l.name == "c5.q"][0], r=32)
    data = inputs.make(lin)
    dev = "cuda:0"
    X, W, dY = (acc.to_device(data[k], dev) for k in ("X", "W", "dY"))
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed)
    bf = torch.bfloat16
    Y = torch.empty(lin.n, lin.d_out, dtype=bf, device=dev); dX = torch.empty(lin.n, lin.d_in, dtype=bf, device=dev)
    U = torch.empty(lin.n, lin.r, dtype=bf, device=dev); V = torch.empty(lin.d_in, lin.r, dtype=bf, device=dev)
    Gr = torch.empty(lin.r, lin.d_out, dtype=bf, device=dev); dW = torch.empty(lin.d_in, lin.d_out, dtype=bf, device=dev)
    acc.acc_linear_fwd_rsvd(desc, X, W, Y, U, V, acc.alloc_workspace(desc, False, dev, rsvd=True))
    acc.acc_linear_bwd_rsvd(desc, dY, W, U, V, dX, Gr, dW, acc.alloc_workspace(desc, True, dev, rsvd=True))
    torch.cuda.synchronize()
    Xo, Wo, dYo = (inputs.as_f64(data[k]) for k in ("X", "W", "dY"))
    Uo, Vo = orc.rsvd_factors(Xo, lin.seed, lin.r)
    Gro = Uo.T @ dYo
    rows = np.sort(np.random.default_rng(5).choice(lin.n, size=256, replace=False))
    errs = {"U": gu.rel(acc.to_host_f64(U), Uo), "V": gu.rel(acc.to_host_f64(V), Vo),
            "Gr": gu.rel(acc.to_host_f64(Gr), Gro), "dW": gu.rel(acc.to_host_f64(dW), Vo @ Gro),
            "Y": gu.rel(acc.to_host_f64(Y[rows]), Xo[rows] @ Wo), "dX": gu.rel(acc.to_host_f64(dX[rows]), dYo[rows] @ Wo.T)}
    print(lin.name, "rsvd k=32", " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= 1e-2 for v in errs.values()), errs
