"""GPU vs oracle: the Philox integer stream is bit-exact; the regenerated S agrees to fp32 rounding."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import acc_oracle as orc


@pytest.fixture(scope="module")
def acc():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_01255_amd import binding
    return binding


def _dump_words(acc, seed, row_offset, n, r):
    import torch
    nq = (n + 3) // 4
    out = torch.zeros(nq * r * 4, dtype=torch.int32, device="cuda:0")
    acc.acc_philox_dump_u32(seed, row_offset, n, r, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint32).reshape(nq, r, 4)


@pytest.mark.parametrize("seed,row_offset,n,r", [
    (0, 0, 256, 16),                                  # the tiny configuration, whole range
    (0x0123456789ABCDEF, 0, 1001, 48),                # ragged token count, both key words
    (42, 4 * 12345, 515, 32),                         # a shard that starts mid-stream
    (7, (1 << 34) - 8, 64, 16),                       # token indices crossing into counter word 3
    (3, 65536 - 512, 512, 512),                       # the tail of the 65536-token, rank-512 shape
])
def test_philox_stream_bit_exact(acc, seed, row_offset, n, r):
    got = _dump_words(acc, seed, row_offset, n, r)
    want = orc.sketch_words(seed, row_offset, n, r)
    assert got.dtype == want.dtype and got.shape == want.shape
    assert np.array_equal(got, want)


@pytest.mark.parametrize("n,r,row_offset", [(256, 16, 0), (1003, 64, 8), (4096, 256, 0)])
def test_sketch_matrix_fp32(acc, n, r, row_offset):
    import torch
    S = torch.full((n, r), 9.0, dtype=torch.float32, device="cuda:0")
    desc = acc.make_desc(n, 8, 8, r, seed=5, io_dtype=acc.ACC_F32, row_offset=row_offset)
    acc.acc_sketch_dump(desc, S)
    torch.cuda.synchronize()
    got = S.cpu().numpy().astype(np.float64)
    want = orc.sketch_matrix(5, n, r, row_offset)
    scale = 1.0 / np.sqrt(r)
    # fp32 libm after exact uniforms: a few ulp of values of size ~scale
    assert np.max(np.abs(got - want)) < 4e-6 * scale
    assert np.linalg.norm(got - want) / np.linalg.norm(want) < 3e-7


@pytest.mark.parametrize("n,r", [(256, 16), (4096, 256)])
def test_sketch_matrix_bf16_generator(acc, n, r):
    """The fast generator (hardware log/sqrt/sin/cos) rounded to bf16: error is bf16 rounding."""
    import torch
    S = torch.zeros((n, r), dtype=torch.float32, device="cuda:0")
    desc = acc.make_desc(n, 8, 8, r, seed=5, io_dtype=acc.ACC_BF16)
    acc.acc_sketch_dump(desc, S)
    torch.cuda.synchronize()
    got = S.cpu().numpy().astype(np.float64)
    want = orc.sketch_matrix(5, n, r)
    assert np.array_equal(orc.round_to_bf16(got), got)           # values are bf16-representable
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 3e-6 / np.sqrt(r))
    rounded = orc.round_to_bf16(want)
    assert np.mean(rounded != got) < 2e-3                        # nearly always the same bf16 value


def _identity_like(acc, n, d):
    """[n, d] bf16 device matrix with ones on the main diagonal (d >= n)."""
    import torch
    m = torch.zeros(n, d, dtype=torch.bfloat16, device="cuda:0")
    m[torch.arange(n), torch.arange(n)] = 1.0
    return m


@pytest.mark.parametrize("n,d,r,row_offset,one_launch", [
    (512, 512, 64, 0, False),                      # one channel slab, one column slice, two token splits
    (512, 512, 256, 0, False),                     # four column slices
    (1030, 1088, 64, 4 * 33, False),               # ragged token count (not even a multiple of 4), ragged slab
    (1030, 1088, 256, 0, False),
    (1030, 1032, 48, 0, False),                    # rank below the tile's 64 columns (surplus columns masked)
    (1024, 1024, 128, 0, True),                    # the 512 x 128 tile
    (1024, 1024, 256, 8, True),
    (1024, 1024, 64, (1 << 34) - 512, False),      # token indices crossing 2^34 inside the range
    (1024, 1024, 128, (1 << 34) - 512, True),
    (8192, 8192, 256, 0, False),                   # 16 channel slabs, 2048 tokens (64 stages) per split
    (4096, 4096, 512, 4096, True),                 # eight column slices of the narrow tile's width, wide tile
])
def test_layer_kernels_regenerate_s_entry_by_entry(acc, n, d, r, row_offset, one_launch):
    """The sketch kernels' own generator (their Philox rounds, counter arithmetic, Box-Muller and the exchange of
    generated pieces between waves), pinned through the layer calls: with X = I the forward's factor is
    Xs = X^T.S = S itself, with dY = I the backward's factor is Gr = S^T, each product having one non-zero term,
    so every entry of the factors is one entry of S as the kernel generated and rounded it."""
    import torch
    seed = 0xC0FFEE123456789
    flags = acc.ACC_FLAG_ONE_LAUNCH if one_launch else 0
    desc = acc.make_desc(n, d, d, r, seed=seed, io_dtype=acc.ACC_BF16, row_offset=row_offset, flags=flags)
    eye = _identity_like(acc, n, d)
    W = torch.zeros(d, d, dtype=torch.bfloat16, device="cuda:0")
    Y = torch.empty(n, d, dtype=torch.bfloat16, device="cuda:0")
    dX = torch.empty(n, d, dtype=torch.bfloat16, device="cuda:0")
    Xs = torch.full((d, r), 7.0, dtype=torch.bfloat16, device="cuda:0")
    Gr = torch.full((r, d), 7.0, dtype=torch.bfloat16, device="cuda:0")
    acc.acc_linear_fwd(desc, eye, W, Y, Xs, acc.alloc_workspace(desc, False))
    acc.acc_linear_bwd(desc, eye, W, Xs, dX, Gr, None, acc.alloc_workspace(desc, True))
    torch.cuda.synchronize()
    want = orc.sketch_matrix(seed, n, r, row_offset)
    rounded = orc.round_to_bf16(want)
    for name, got in (("Xs", acc.to_host_f64(Xs)), ("Gr", acc.to_host_f64(Gr).T)):
        assert np.all(got[n:] == 0.0), name                          # channels no token touches
        got = got[:n]
        # hardware log / sqrt / sin / cos against libm: a few 1e-6 of 1/sqrt(r) before the rounding to bf16
        assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 3e-6 / np.sqrt(r)), name
        mismatch = float(np.mean(rounded != got))
        print(name, n, r, "fraction of entries one bf16 step off:", mismatch, flush=True)
        assert mismatch < 2e-3, (name, mismatch)                     # nearly always the very same bf16 value
