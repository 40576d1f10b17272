"""The 8-bit float bit helpers of the input module against PyTorch's own casts (an independent implementation)."""
import numpy as np
import pytest
import torch

from paper_2605_01255_amd import inputs

FORMATS = [("e4m3", torch.float8_e4m3fn), ("e5m2", torch.float8_e5m2)]


@pytest.mark.parametrize("fmt,tdt", FORMATS)
def test_decode_of_every_finite_pattern(fmt, tdt):
    bits = np.arange(256, dtype=np.uint8)
    ours = inputs.fp8_bits_to_f64(bits, fmt)
    theirs = torch.from_numpy(bits).view(tdt).to(torch.float64).numpy()
    finite = np.isfinite(theirs)
    assert np.array_equal(np.isfinite(ours), finite)
    assert np.array_equal(ours[finite], theirs[finite])


@pytest.mark.parametrize("fmt,tdt", FORMATS)
def test_encode_rounds_to_nearest_even_and_saturates(fmt, tdt):
    rng = np.random.default_rng(3)
    top = inputs.fp8_max(fmt)
    a = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(top / 4),
        rng.standard_normal(50000).astype(np.float32) * np.float32(2.0 ** -8),      # subnormal range
        np.array([0.0, -0.0, top, -top, top * 0.999, 2.0 ** -9, 2.0 ** -10, 2.0 ** -17], dtype=np.float32),
    ])
    # midpoints between neighbouring patterns: the tie rule
    tab = inputs.fp8_bits_to_f64(np.arange(0x70, dtype=np.uint8), fmt)
    a = np.concatenate([a, ((tab[:-1] + tab[1:]) / 2).astype(np.float32)])
    ours = inputs.f32_to_fp8_bits(a, fmt)
    inside = np.abs(a) <= top                               # torch's cast does not saturate; ours does
    theirs = torch.from_numpy(a[inside]).to(tdt).view(torch.uint8).numpy()
    assert np.array_equal(ours[inside], theirs)
    sat = inputs.fp8_bits_to_f64(ours[~inside], fmt)
    assert np.array_equal(np.abs(sat), np.full(sat.shape, top)) and np.array_equal(np.sign(sat), np.sign(a[~inside]))
