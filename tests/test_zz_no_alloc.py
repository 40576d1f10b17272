"""acc_linear_fwd_static (the forward entry point that allocates nothing: the sketch's split-token partial
tiles live in a static device array inside the library) against acc_linear_fwd with a caller's workspace.

Both run the same kernels in the same order, so every output must agree bit for bit; beside that the static
call's outputs are held to the oracle at the usual bar.  Two calls in a row share the array, the second with
a smaller input, so stale partial tiles of the first call would show."""
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


def _forward_both(acc, lin, data, flags=0, dev="cuda:0"):
    import torch
    code = acc.ACC_BF16 if lin.dtype == "bf16" else acc.ACC_F32
    tdt = acc.torch_dtype(code)
    X, W = acc.to_device(data["X"], dev), acc.to_device(data["W"], dev)
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=code, flags=flags)
    out = []
    for static in (False, True):
        Y = torch.full((lin.n, lin.d_out), 7.0, dtype=tdt, device=dev)
        Xs = torch.full((lin.d_in, lin.r), 7.0, dtype=tdt, device=dev)
        print(f"no-alloc case {lin.name} static={static}", flush=True)
        if static:
            acc.acc_linear_fwd_static(desc, X, W, Y, Xs)
        else:
            acc.acc_linear_fwd(desc, X, W, Y, Xs, acc.alloc_workspace(desc, False, dev))
        torch.cuda.synchronize()
        out.append((Y.cpu(), Xs.cpu(), acc.to_host_f64(Y), acc.to_host_f64(Xs)))
    return out


def test_static_scratch_forward_matches_the_workspace_forward_twice_in_a_row(acc):
    import torch
    # first call: tuned kernels, several token splits, ragged tails; second call: smaller in every dimension
    # (fewer splits, fewer channels, smaller rank), so it reads only what it wrote itself if it is correct
    cases = [inputs.Linear("static_a", 2049, 1032, 776, 128, dtype="bf16"),
             inputs.Linear("static_b", 777, 520, 264, 48, dtype="bf16"),
             inputs.Linear("static_c_f32", 130, 72, 40, 16, dtype="f32", x_kind="plain")]
    for lin in cases:
        data = inputs.make(lin)
        (y0, xs0, _, _), (y1, xs1, yf, xsf) = _forward_both(acc, lin, data)
        assert torch.equal(y0, y1), lin.name
        assert torch.equal(xs0, xs1), lin.name
        Xf, Wf = inputs.as_f64(data["X"]), inputs.as_f64(data["W"])
        oY, oXs = orc.linear_fwd(Xf, Wf, lin.seed, lin.r)
        tol = gu.tolerance(acc.ACC_BF16 if lin.dtype == "bf16" else acc.ACC_F32)
        gu.check_outputs({"Y": yf, "Xs": xsf}, {"Y": oY, "Xs": oXs}, tol, lin.name)


def test_static_scratch_forward_refuses_what_does_not_fit(acc):
    import ctypes
    import torch
    # 8B-shaped projection: the partial tiles need more than the static array holds
    desc = acc.make_desc(65536, 4096, 4096, 512, io_dtype=acc.ACC_BF16)
    assert acc.acc_linear_workspace_bytes(desc, False) > acc.ACC_STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    rc = acc._lib.acc_linear_fwd_static(ctypes.byref(desc), t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), None)
    assert rc == -5
    # the 3B-shaped projection at r = 256 fits
    desc = acc.make_desc(16384, 3072, 3072, 256, io_dtype=acc.ACC_BF16)
    assert 0 < acc.acc_linear_workspace_bytes(desc, False) <= acc.ACC_STATIC_SCRATCH_BYTES
