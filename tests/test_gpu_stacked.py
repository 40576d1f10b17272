"""Accumulation of the factored gradient over micro-batches without a dense gradient (Sec. 4: the gradient is
kept as two factors; a sum of factored gradients is the product of the stacked factors), GPU vs the oracle.

Each micro-batch writes its Xs into a column block of one stacked left factor (descriptor field ldf) and its Gr
into a row block of one stacked small factor; acc_linear_dw then forms the dense sum from the stacked pair in one
pass.  Checked: the stacked factors block by block against the oracle's per-batch factors, the dense product
against the oracle's sum of per-batch gradients, and against the GPU's own dense accumulation
(ACC_FLAG_DW_ACCUMULATE), which must agree to rounding."""
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


def _run(acc, n, d_in, d_out, r, M, dtype, w_out_in=False, dev="cuda:0"):
    import torch
    code = acc.ACC_BF16 if dtype == "bf16" else acc.ACC_F32
    tdt = acc.torch_dtype(code)
    flags = acc.ACC_FLAG_W_OUT_IN if w_out_in else 0
    R = M * r
    xs_stack = torch.full((d_in, R), 7.0, dtype=tdt, device=dev)
    gr_stack = torch.full((d_out, R) if w_out_in else (R, d_out), 7.0, dtype=tdt, device=dev)
    dw_acc = torch.zeros((d_out, d_in) if w_out_in else (d_in, d_out), dtype=torch.float32, device=dev)
    esz = xs_stack.element_size()
    want_xs, want_gr, want_dw = [], [], None
    lin0 = inputs.Linear(f"stack_{dtype}", n, d_in, d_out, r, dtype=dtype, x_kind="plain" if dtype == "f32" else "outlier")
    W_host = inputs.store(inputs.make_w(lin0), dtype)
    Wf = inputs.as_f64(W_host)
    W = acc.to_device(np.ascontiguousarray(W_host.T) if w_out_in else W_host, dev)
    for m in range(M):
        lin = inputs.Linear(f"stack_{dtype}_{m}", n, d_in, d_out, r, dtype=dtype, data_seed=inputs.DATA_SEED + 1 + m,
                            x_kind="plain" if dtype == "f32" else "outlier")
        data = inputs.make(lin)
        row_offset = 4 * ((m * n + 3) // 4)          # every micro-batch draws its own rows of S
        X, dY = acc.to_device(data["X"], dev), acc.to_device(data["dY"], dev)
        desc = acc.make_desc(n, d_in, d_out, r, seed=5, io_dtype=code, dw_dtype=acc.ACC_F32, row_offset=row_offset,
                             flags=flags, ldf=R)
        Y = torch.empty(n, d_out, dtype=tdt, device=dev)
        dX = torch.empty(n, d_in, dtype=tdt, device=dev)
        xs_ptr = xs_stack.data_ptr() + m * r * esz
        gr_ptr = gr_stack.data_ptr() + (m * r * esz if w_out_in else m * r * d_out * esz)
        print(f"stacked case {lin.name} w_out_in={w_out_in} micro-batch {m}", flush=True)
        acc.acc_linear_fwd(desc, X, W, Y, xs_ptr, acc.alloc_workspace(desc, False, dev))
        acc.acc_linear_bwd(desc, dY, W, xs_ptr, dX, gr_ptr, None, acc.alloc_workspace(desc, True, dev))
        # the same micro-batch accumulated on a dense fp32 gradient
        adesc = acc.make_desc(n, d_in, d_out, r, seed=5, io_dtype=code, dw_dtype=acc.ACC_F32, row_offset=row_offset,
                              flags=flags | acc.ACC_FLAG_DW_ACCUMULATE, ldf=R)
        acc.acc_linear_dw(adesc, xs_ptr, gr_ptr, dw_acc)
        torch.cuda.synchronize()
        Xf, dYf = inputs.as_f64(data["X"]), inputs.as_f64(data["dY"])
        S = orc.sketch_matrix(5, n, r, row_offset)
        _, oXs = orc.linear_fwd(Xf, Wf, S=S)
        _, oGr, want_dw = orc.linear_bwd(dYf, Wf, oXs, S=S, dW_prev=want_dw)
        want_xs.append(oXs); want_gr.append(oGr)
    # one pass over dW from the stacked pair (rank M r, dense factors)
    sdesc = acc.make_desc(n, d_in, d_out, R, io_dtype=code, dw_dtype=acc.ACC_F32, flags=flags)
    dw_stack = torch.full_like(dw_acc, 7.0)
    acc.acc_linear_dw(sdesc, xs_stack, gr_stack, dw_stack)
    torch.cuda.synchronize()
    tol = gu.tolerance(code)
    got = {"Xs_stack": acc.to_host_f64(xs_stack), "Gr_stack": acc.to_host_f64(gr_stack),
           "dW_stack": acc.to_host_f64(dw_stack), "dW_accumulated": acc.to_host_f64(dw_acc)}
    want_gr_stack = np.vstack(want_gr)
    want_dw_o = want_dw
    if w_out_in:
        want_gr_stack, want_dw_o = np.ascontiguousarray(want_gr_stack.T), np.ascontiguousarray(want_dw.T)
    want = {"Xs_stack": np.hstack(want_xs), "Gr_stack": want_gr_stack, "dW_stack": want_dw_o,
            "dW_accumulated": want_dw_o}
    gu.check_outputs(got, want, tol, f"stacked {dtype} n={n} {d_in}x{d_out} r={r} M={M} oi={w_out_in}")
    # stacked product and dense accumulation are the same sum in a different order
    assert gu.rel(got["dW_stack"], got["dW_accumulated"]) <= (2e-3 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("w_out_in", [False, True])
def test_stacked_factors_bf16_tuned_kernels(acc, w_out_in):
    _run(acc, 1030, 1032, 776, 64, 3, "bf16", w_out_in)


@pytest.mark.parametrize("w_out_in", [False, True])
def test_stacked_factors_fp32_generic_kernels(acc, w_out_in):
    _run(acc, 130, 72, 40, 16, 2, "f32", w_out_in)


def test_stacked_factors_bf16_small_rank_generic_sketch(acc):
    _run(acc, 515, 264, 136, 8, 4, "bf16")
