"""The dense weight gradient from the two factors alone (acc_linear_dw: Sec. 4, update strategy (i)) against the
oracle's product, over the shapes that choose between its kernels: the three-stage small-K kernel (at most 256
tiles of 192 x 192), the pipelined kernel (more tiles), the generic kernels (fp32 factors, K % 64 != 0); ragged
edges in both dimensions, both orientations, both output types, plain and accumulating."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2605_01255_amd import inputs
import gpu_util as gu


@pytest.fixture(scope="module")
def acc():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_01255_amd import binding
    return binding


def _factors(d_in, d_out, r, dtype, seed):
    rng = np.random.default_rng(seed)
    xs = rng.standard_normal((d_in, r)).astype(np.float32) * 8.0
    xs[5 % d_in] *= 20.0                                   # an outlier channel, as the sketch of X has
    gr = rng.standard_normal((r, d_out)).astype(np.float32) * 0.08
    return inputs.store(xs, dtype), inputs.store(gr, dtype)


CASES = [
    # d_in, d_out, r, factor dtype, dW dtype
    (3072, 3072, 256, "bf16", "bf16"),     # the benchmark's gradient: 16 x 16 tiles, one round
    (200, 392, 64, "bf16", "bf16"),        # ragged in both dimensions, one K tile
    (1000, 1160, 128, "bf16", "f32"),      # ragged, fp32 output
    (3000, 3080, 512, "bf16", "bf16"),     # eight K tiles: the ring of three stages wraps twice
    (3072, 8192, 192, "bf16", "bf16"),     # 688 tiles: the pipelined kernel
    (520, 264, 40, "bf16", "bf16"),        # K % 64 != 0: generic kernel
    (264, 520, 32, "f32", "f32"),          # fp32 factors: generic kernel
]


@pytest.mark.parametrize("w_out_in", [False, True])
@pytest.mark.parametrize("d_in,d_out,r,fdt,ddt", CASES)
def test_dense_gradient_from_factors(acc, d_in, d_out, r, fdt, ddt, w_out_in):
    import torch
    dev = "cuda:0"
    xs_h, gr_h = _factors(d_in, d_out, r, fdt, seed=d_in + r)
    xs64, gr64 = inputs.as_f64(xs_h), inputs.as_f64(gr_h)
    want = xs64 @ gr64
    fcode = acc.ACC_BF16 if fdt == "bf16" else acc.ACC_F32
    dcode = acc.ACC_BF16 if ddt == "bf16" else acc.ACC_F32
    flags = acc.ACC_FLAG_W_OUT_IN if w_out_in else 0
    Xs = acc.to_device(xs_h, dev)
    Gr = acc.to_device(np.ascontiguousarray(gr_h.T) if w_out_in else gr_h, dev)
    shape = (d_out, d_in) if w_out_in else (d_in, d_out)
    start = np.random.default_rng(1).standard_normal(shape).astype(np.float32)
    start_h = inputs.store(start, ddt)
    dW = acc.to_device(start_h, dev)
    desc = acc.make_desc(256, d_in, d_out, r, io_dtype=fcode, factor_dtype=fcode, dw_dtype=dcode, flags=flags)
    print(f"dW case {d_in}x{d_out} r={r} {fdt}->{ddt} w_out_in={w_out_in} write", flush=True)
    acc.acc_linear_dw(desc, Xs, Gr, dW)
    torch.cuda.synchronize()
    tol = 1e-2 if "bf16" in (fdt, ddt) else 1e-5
    w = want.T if w_out_in else want
    gu.assert_close(acc.to_host_f64(dW), w, tol, "dW")
    # accumulate onto what is there
    desc_a = acc.make_desc(256, d_in, d_out, r, io_dtype=fcode, factor_dtype=fcode, dw_dtype=dcode,
                           flags=flags | acc.ACC_FLAG_DW_ACCUMULATE)
    dW2 = acc.to_device(start_h, dev)
    print(f"dW case {d_in}x{d_out} r={r} {fdt}->{ddt} w_out_in={w_out_in} accumulate", flush=True)
    acc.acc_linear_dw(desc_a, Xs, Gr, dW2)
    torch.cuda.synchronize()
    gu.assert_close(acc.to_host_f64(dW2), inputs.as_f64(start_h) + w, tol, "dW accumulated")
