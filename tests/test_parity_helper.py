"""The GPU parity tests' comparison helper, checked on the CPU: a stand-in for a GPU result (the oracle's value
with the roundings the bf16 kernels make) passes; the same result with one read-out unit, one row, one ragged
edge block or one element replaced by wrong values fails, although the whole-tensor norm still passes."""
import numpy as np
import pytest

from paper_2605_01255_amd import inputs
from oracle import acc_oracle as orc
import gpu_util as gu


def _bf16(a):
    return inputs.as_f64(inputs.f32_to_bf16_bits(np.asarray(a, dtype=np.float32)))


@pytest.fixture(scope="module")
def layer():
    lin = inputs.Linear("helper", 2100, 1024, 1544, 64, dtype="bf16")   # ragged last block row and column
    data = inputs.make(lin)
    X, W, dY = (inputs.as_f64(data[k]) for k in ("X", "W", "dY"))
    S = orc.sketch_matrix(lin.seed, lin.n, lin.r)
    Y, Xs = orc.linear_fwd(X, W, S=S)
    _, Gr, dW = orc.linear_bwd(dY, W, Xs, S=S)
    # what a correct bf16 kernel returns: S rounded to bf16 before the product, outputs rounded once
    Sb = _bf16(S)
    got = {"Y": _bf16(Y), "Xs": _bf16(X.T @ Sb), "Gr": _bf16(Sb.T @ dY)}
    got["dW"] = _bf16(got["Xs"] @ got["Gr"])
    return {"want": {"Y": Y, "Xs": Xs, "Gr": Gr, "dW": dW}, "got": got}


def test_a_correctly_rounded_result_passes(layer):
    for k, want in layer["want"].items():
        whole = gu.assert_close(layer["got"][k], want, 1e-2, k)
        worst_blk, worst_el, _ = gu.local_errors(layer["got"][k], want, 1e-2)
        print(k, f"whole={whole:.2e} worst block={worst_blk:.2e} worst element={worst_el:.2f}")
        assert worst_blk < 1e-2 and worst_el < 0.7   # headroom: the bounds are not at the edge of the noise


@pytest.fixture(scope="module")
def big():
    """An output of the 3B-shaped projection's size (16384 x 3072) and its correctly rounded bf16 image."""
    want = np.random.default_rng(7).standard_normal((16384, 3072), dtype=np.float32).astype(np.float64)
    return want, _bf16(want)


@pytest.mark.parametrize("what", ["unit_32x64", "row", "ragged_corner", "element", "stale_unit", "shifted_unit"])
def test_local_corruption_fails_where_the_whole_norm_passes(big, what):
    want, got = big[0], big[1].copy()
    rng = np.random.default_rng(0)
    if what == "unit_32x64":      # a read-out unit filled with unrelated values of the right size
        got[256:288, 640:704] = rng.standard_normal((32, 64))
    elif what == "row":
        got[10031] = 0.0
    elif what == "ragged_corner":  # the last block row x block column
        got[-32:, -32:] = 0.0
    elif what == "element":
        got[77, 1201] += 1.0
    elif what == "stale_unit":     # a unit that kept the value of the neighbouring tile
        got[512:544, 256:320] = got[512:544, 320:384]
    elif what == "shifted_unit":   # right values, one column off
        got[96:128, 64:128] = np.roll(got[96:128, 64:128], 1, axis=1)
    assert gu.rel(got, want) <= 1e-2, "the whole-tensor norm alone does not see this"
    # the local checks work block by block, so a band of block rows around the damage is enough to show them fail
    lo = {"row": 9984, "ragged_corner": 16384 - 256}.get(what, 0)
    worst_blk, worst_el, blk_tol = gu.local_errors(got[lo:lo + 1024], want[lo:lo + 1024], 1e-2)
    assert worst_blk > blk_tol or worst_el > 1.0, (worst_blk, worst_el)
    clean_blk, clean_el, _ = gu.local_errors(big[1][lo:lo + 1024], want[lo:lo + 1024], 1e-2)
    assert clean_blk <= blk_tol and clean_el <= 1.0


def test_float32_bounds(layer):
    want = layer["want"]["Y"][:300, :200]
    got = want.astype(np.float32).astype(np.float64)      # one fp32 rounding
    gu.assert_close(got, want, 1e-5, "f32")
    bad = got.copy()
    bad[40, 50] *= 1.0 + 1e-3
    with pytest.raises(AssertionError):
        gu.assert_close(bad, want, 1e-5, "f32 element")


def test_zero_blocks_and_vectors():
    want = np.zeros((70, 40))
    gu.assert_close(want.copy(), want, 1e-2, "zeros")
    bad = want.copy()
    bad[69, 39] = 1e-30
    with pytest.raises(AssertionError):
        gu.assert_close(bad, want, 1e-2, "zeros with one non-zero")
    v = np.linspace(1.0, 2.0, 100)
    gu.assert_close(_bf16(v), v, 1e-2, "vector")
