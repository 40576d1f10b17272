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
