"""Optimizer step on the factored gradient (Sec. 4, update strategy (ii)) on the GPU vs the CPU fp64 oracle,
through the C ABI.  Several consecutive steps, each side carrying its own state from zero.

Tolerances.  M and V are fp32 running sums of exactly representable inputs: 1e-5 relative Frobenius.  W is
stored in io_dtype: 1e-5 (float32) or 1e-2 (bfloat16) like every other output.  Because the weight dwarfs one
update, the update itself is checked too, dW_step = W_after - W_before: in float32 its error is the rounding of
W (6e-8 |W|) plus 1e-5 of the step, bounded here by 1e-3 of the step since the inputs are sized so that a step
is at least 1e-3 of the weight; in bfloat16 the step is sized comparable to the weight, so rounding W to
bfloat16 (2^-9 |W|) plus the bfloat16 roundings of N and of the product stay below 1e-2 of the step."""
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


def run_steps(acc, lin, steps, hyper, flags=0, factor_dtype=None, pad_w=0, k=0):
    """Returns per step (W, M, V, W_before) from the GPU and from the oracle.  k > 0: through a projector
    [d_in, k], the oracle's for the first step's factors, stored in the factor type and given to both sides."""
    import torch
    dev = "cuda:0"
    code = acc.ACC_BF16 if lin.dtype == "bf16" else acc.ACC_F32
    fname = factor_dtype or lin.dtype
    fcode = acc.ACC_BF16 if fname == "bf16" else acc.ACC_F32
    w_oi = bool(flags & acc.ACC_FLAG_W_OUT_IN)
    left_h, grs_h = inputs.make_gradient_factors(lin, steps, fname)
    w_h = inputs.store(inputs.make_w(lin), lin.dtype)
    w_dev_h = np.ascontiguousarray(w_h.T) if w_oi else w_h
    cols = w_dev_h.shape[1]
    W = torch.full((w_dev_h.shape[0], cols + pad_w), float("nan"), dtype=acc.torch_dtype(code), device=dev)
    W[:, :cols] = acc.to_device(w_dev_h, dev)
    left = acc.to_device(left_h, dev)
    kk = k or lin.r
    shape = (lin.d_out, kk) if w_oi else (kk, lin.d_out)
    P = P_o = None
    if k:
        P_h = inputs.store(orc.gradient_projector(inputs.as_f64(left_h), inputs.as_f64(grs_h[0]), lin.seed, k)
                           .astype(np.float32), fname)
        P, P_o = acc.to_device(P_h, dev), inputs.as_f64(P_h)
    M = torch.zeros(shape, dtype=torch.float32, device=dev)
    V = torch.zeros(shape, dtype=torch.float32, device=dev)
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, io_dtype=code, factor_dtype=fcode, flags=flags,
                         ldw=cols + pad_w if pad_w else 0)
    ws = acc.alloc_lowrank_workspace(desc, k, dev)
    got, want = [], []
    Wo = inputs.as_f64(w_h)
    Mo = np.zeros((kk, lin.d_out)); Vo = np.zeros((kk, lin.d_out))
    lo = inputs.as_f64(left_h)
    for t in range(1, steps + 1):
        g_h = grs_h[t - 1]
        Gr = acc.to_device(np.ascontiguousarray(g_h.T) if w_oi else g_h, dev)
        before = acc.to_host_f64(W[:, :cols])
        acc.acc_lowrank_adamw_step(desc, acc.make_hyper(t, **hyper), P, k, left, Gr, M, V, W, ws)
        torch.cuda.synchronize()
        after = acc.to_host_f64(W[:, :cols])
        if pad_w:
            assert bool(torch.isnan(W[:, cols:]).all()), "padding columns of W were written"
        tr = (lambda a: a.T) if w_oi else (lambda a: a)
        got.append((tr(after), tr(acc.to_host_f64(M)), tr(acc.to_host_f64(V)), tr(before)))
        Wprev = Wo
        Wo, Mo, Vo, _ = orc.lowrank_adamw_step(Wo, lo, inputs.as_f64(g_h), Mo, Vo, step=t, P=P_o, **hyper)
        want.append((Wo, Mo, Vo, Wprev))
    return got, want


def check(got, want, w_tol, step_tol, name):
    for t, (g, w) in enumerate(zip(got, want), start=1):
        e_w, e_m, e_v = gu.rel(g[0], w[0]), gu.rel(g[1], w[1]), gu.rel(g[2], w[2])
        # the step each side took from its own previous weight
        e_step = gu.rel(g[0] - g[3], w[0] - w[3])
        size = np.linalg.norm(w[0] - w[3]) / np.linalg.norm(w[3])
        print(f"{name} step {t}: W={e_w:.2e} M={e_m:.2e} V={e_v:.2e} step={e_step:.2e} |step|/|W|={size:.2e}",
              flush=True)
        assert e_m <= 1e-5 and e_v <= 1e-5, (t, e_m, e_v)
        assert e_w <= w_tol, (t, e_w)
        assert e_step <= step_tol, (t, e_step)


HYPER = dict(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, scale=0.5)


@pytest.mark.parametrize("flags_name", ["default", "w_out_in"])
def test_f32_ragged_three_steps(acc, flags_name):
    flags = acc.ACC_FLAG_W_OUT_IN if flags_name == "w_out_in" else 0
    lin = inputs.Linear("opt.f32", 320, 200, 328, 24, dtype="f32", x_kind="plain")
    got, want = run_steps(acc, lin, 3, HYPER, flags=flags, pad_w=8)
    check(got, want, 1e-5, 1e-3, f"f32 {flags_name}")


@pytest.mark.parametrize("flags_name", ["default", "w_out_in"])
def test_bf16_tuned_kernel_three_steps(acc, flags_name):
    # r % 64 == 0: the tuned GEMM's accumulate epilogue; several tiles and a ragged last tile in both directions
    flags = acc.ACC_FLAG_W_OUT_IN if flags_name == "w_out_in" else 0
    lin = inputs.Linear("opt.bf16", 2048, 1096, 840, 128, dtype="bf16", x_kind="plain")
    got, want = run_steps(acc, lin, 3, HYPER, flags=flags, pad_w=16)
    check(got, want, 1e-2, 1e-2, f"bf16 {flags_name}")


@pytest.mark.parametrize("flags_name", ["default", "w_out_in"])
@pytest.mark.parametrize("dtype,k,w_tol,step_tol", [("f32", 16, 1e-5, 1e-3), ("bf16", 64, 1e-2, 1e-2),
                                                    ("bf16", 24, 1e-2, 1e-2)])
def test_projected_three_steps(acc, flags_name, dtype, k, w_tol, step_tol):
    """Through a fixed projector P [d_in, k]: R = (P^T left) Gr, moments [k, d_out], W moves inside range(P).
    k = 64 takes the tuned GEMM's accumulate epilogue for P . N, k = 24 and float32 the generic kernel."""
    flags = acc.ACC_FLAG_W_OUT_IN if flags_name == "w_out_in" else 0
    lin = inputs.Linear("opt.proj." + dtype, 2048, 712, 840, 128, dtype=dtype, x_kind="plain")
    # an orthonormal projector gives steps of size lr * scale * sqrt(k / d_in) per entry: lr is sized so that the
    # step stays comparable to the weight (0.02 per entry), as the step tolerance in bfloat16 assumes
    got, want = run_steps(acc, lin, 3, {**HYPER, "lr": 0.2}, flags=flags, pad_w=8, k=k)
    check(got, want, w_tol, step_tol, f"projected {dtype} k={k} {flags_name}")


@pytest.mark.parametrize("flags_name", ["default", "w_out_in"])
@pytest.mark.parametrize("dtype,k", [("f32", 8), ("f32", 40), ("bf16", 32), ("bf16", 64),
                                     ("f32", 72), ("bf16", 128)])   # above 64: the blocked factorisation
def test_projector_matches_oracle(acc, flags_name, dtype, k):
    """P = orthonormal basis (positive-diagonal QR) of left . (Gr . Omega).  Tolerance: the basis inherits the
    conditioning of Yp, so the bar is cond(Yp) times the output type's (1e-5 float32, 1e-2 bfloat16 capped at
    what bfloat16 storage of P itself costs, 2^-9), evaluated from the oracle's Yp."""
    import torch
    dev = "cuda:0"
    flags = acc.ACC_FLAG_W_OUT_IN if flags_name == "w_out_in" else 0
    lin = inputs.Linear("opt.P." + dtype, 1024, 520, 328, max(72, k + 8), dtype=dtype, x_kind="plain")
    code = acc.ACC_BF16 if dtype == "bf16" else acc.ACC_F32
    left_h, (gr_h,) = inputs.make_gradient_factors(lin, 1)
    left = acc.to_device(left_h, dev)
    Gr = acc.to_device(np.ascontiguousarray(gr_h.T) if flags else gr_h, dev)
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=code, flags=flags)
    P = torch.full((lin.d_in, k), 7.0, dtype=acc.torch_dtype(code), device=dev)
    acc.acc_lowrank_projector(desc, k, left, Gr, P, acc.alloc_lowrank_workspace(desc, k, dev))
    torch.cuda.synchronize()
    got = acc.to_host_f64(P)
    lo, go = inputs.as_f64(left_h), inputs.as_f64(gr_h)
    want = orc.gradient_projector(lo, go, lin.seed, k)
    cond = np.linalg.cond(lo @ (go @ orc.range_finder_matrix(lin.seed, lin.d_out, k)))
    tol = cond * (1e-5 if dtype == "f32" else 1e-2 / 4)
    err = gu.rel(got, want)
    orth = np.linalg.norm(got.T @ got - np.eye(k))
    print(f"projector {dtype} k={k} {flags_name}: rel={err:.2e} cond={cond:.1f} |P^T P - I|={orth:.2e}", flush=True)
    assert err <= tol, (err, tol)
    assert orth <= (1e-4 if dtype == "f32" else 2e-2)
    # inside the gradient's range: P = left . C for some C
    resid = got - lo @ np.linalg.lstsq(lo, got, rcond=None)[0]
    assert np.linalg.norm(resid) <= (1e-4 if dtype == "f32" else 1e-2) * np.sqrt(k)


def test_projector_then_step_on_the_gpu_moves_the_weight_inside_the_gradients_range(acc):
    """The two calls chained as a training loop chains them, checked through properties that need no oracle input
    from the GPU: the update W_after - W_before lies in range(left) (it is P . N with range(P) in range(left))."""
    import torch
    dev = "cuda:0"
    lin = inputs.Linear("opt.chain", 1024, 520, 328, 72, dtype="f32", x_kind="plain")
    left_h, (gr_h,) = inputs.make_gradient_factors(lin, 1)
    w_h = inputs.store(inputs.make_w(lin), "f32")
    left, Gr, W = acc.to_device(left_h, dev), acc.to_device(gr_h, dev), acc.to_device(w_h, dev)
    k = 24
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=acc.ACC_F32)
    ws = acc.alloc_lowrank_workspace(desc, k, dev)
    P = torch.empty(lin.d_in, k, device=dev)
    M = torch.zeros(k, lin.d_out, device=dev); V = torch.zeros(k, lin.d_out, device=dev)
    acc.acc_lowrank_projector(desc, k, left, Gr, P, ws)
    acc.acc_lowrank_adamw_step(desc, acc.make_hyper(1, lr=1e-2), P, k, left, Gr, M, V, W, ws)
    torch.cuda.synchronize()
    step = acc.to_host_f64(W) - inputs.as_f64(w_h)
    lo = inputs.as_f64(left_h)
    resid = step - lo @ np.linalg.lstsq(lo, step, rcond=None)[0]
    assert np.linalg.norm(step) > 0
    assert np.linalg.norm(resid) <= 1e-4 * np.linalg.norm(step)
    # first step from zero state: |N| = 1 up to eps, so the step has norm lr * sqrt(k * d_out) (P orthonormal)
    np.testing.assert_allclose(np.linalg.norm(step), 1e-2 * np.sqrt(k * lin.d_out), rtol=1e-3)


def test_bf16_small_rank_generic_kernel(acc):
    lin = inputs.Linear("opt.bf16.r8", 512, 264, 136, 8, dtype="bf16", x_kind="plain")
    got, want = run_steps(acc, lin, 2, HYPER)
    check(got, want, 1e-2, 1e-2, "bf16 r8")


def test_f32_weight_bf16_factors(acc):
    # master weights in float32, factors as the bf16 backward pass stores them
    lin = inputs.Linear("opt.mixed", 1024, 512, 768, 64, dtype="f32", x_kind="plain")
    got, want = run_steps(acc, lin, 3, HYPER, factor_dtype="bf16")
    # N goes through a bfloat16 MFMA operand: the step carries its 2^-9 roundings, and the step is about as large
    # as the weight here, so W inherits them (about 1e-3)
    check(got, want, 3e-3, 1e-2, "f32 W, bf16 factors")


def test_c2_shape_one_step_sampled(acc):
    """The benchmark's projection shape (3072 x 3072, r = 256), one step, whole outputs (the oracle's product is
    a 3072 x 256 x 3072 matmul)."""
    lin = inputs.config("c2")[0]
    got, want = run_steps(acc, lin, 1, HYPER, flags=acc.ACC_FLAG_W_OUT_IN)
    check(got, want, 1e-2, 1e-2, "c2")


def test_c5_gate_shape_projected_step(acc):
    """The 8B-shaped gate projection (4096 x 14336, r = 512) through a rank-64 projector, one step, whole outputs."""
    lin = [l for l in inputs.config("c5") if l.name == "c5.gate"][0]
    got, want = run_steps(acc, lin, 1, {**HYPER, "lr": 0.2}, k=64)
    check(got, want, 1e-2, 1e-2, "c5.gate k=64")


def test_invalid_hyperparameters_are_refused(acc):
    import torch
    lin = inputs.Linear("opt.bad", 256, 64, 64, 8, dtype="f32", x_kind="plain")
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, io_dtype=acc.ACC_F32)
    z = torch.zeros(64, 64, device="cuda:0")
    ws = acc.alloc_workspace(desc, True)
    for bad in (dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0), dict(lr=float("nan"))):
        kw = {**dict(step=1, lr=1e-3), **bad}
        with pytest.raises(acc.AccError) as e:
            acc.acc_lowrank_adamw_step(desc, acc.make_hyper(**kw), None, 0, z, z, z, z, z, ws)
        assert e.value.status == -1, bad
    with pytest.raises(acc.AccError) as e:
        acc.acc_lowrank_adamw_step(desc, acc.make_hyper(1, 1e-3), None, 0, z, z, z, z, z, ws, ws_bytes=64)
    assert e.value.status == -5
    for k in (4, 72, 12):      # not a multiple of 8; above d_in; not a multiple of 8
        with pytest.raises(acc.AccError) as e:
            acc.acc_lowrank_adamw_step(desc, acc.make_hyper(1, 1e-3), z, k, z, z, z, z, z, ws)
        assert e.value.status == -2, k
    for k in (0, 16, 128):     # projector rank: 8..64 and at most r = 8
        with pytest.raises(acc.AccError) as e:
            acc.acc_lowrank_projector(desc, k, z, z, z, ws)
        assert e.value.status == -2, k
    assert acc.acc_lowrank_workspace_bytes(desc, 12) == 0
    torch.cuda.synchronize()
    assert float(z.abs().sum()) == 0.0


def test_rsvd_pass_and_optimizer_step_replay_from_a_hip_graph(acc):
    """A whole training step of update strategy (ii) with the RSVD compressor (forward, backward with the gradient
    left factored, projector refresh, optimizer step) captured once and replayed: the calls only enqueue kernels.
    Every replay starts from the same weight and moments (restored by eager copies between replays) and must
    reproduce the eager result bit for bit."""
    import torch
    dev = "cuda:0"
    lin = inputs.Linear("graph.opt", 2100, 1024, 1544, 32, dtype="bf16")
    data = inputs.make(lin)
    X, W0, dY = (acc.to_device(data[k], dev) for k in ("X", "W", "dY"))
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=7)
    k = 16
    bf = torch.bfloat16
    W = W0.clone()
    Y = torch.empty(lin.n, lin.d_out, dtype=bf, device=dev); dX = torch.empty(lin.n, lin.d_in, dtype=bf, device=dev)
    U = torch.empty(lin.n, lin.r, dtype=bf, device=dev); V = torch.empty(lin.d_in, lin.r, dtype=bf, device=dev)
    Gr = torch.empty(lin.r, lin.d_out, dtype=bf, device=dev); P = torch.empty(lin.d_in, k, dtype=bf, device=dev)
    M = torch.zeros(k, lin.d_out, device=dev); Vm = torch.zeros(k, lin.d_out, device=dev)
    ws_f = acc.alloc_workspace(desc, False, dev, rsvd=True)
    ws_b = acc.alloc_workspace(desc, True, dev, rsvd=True)
    ws_o = acc.alloc_lowrank_workspace(desc, k, dev)
    hyper = acc.make_hyper(1, lr=0.05, weight_decay=0.01)

    def enqueue():
        acc.acc_linear_fwd_rsvd(desc, X, W, Y, U, V, ws_f)
        acc.acc_linear_bwd_rsvd(desc, dY, W, U, V, dX, Gr, None, ws_b)
        acc.acc_lowrank_projector(desc, k, V, Gr, P, ws_o)
        acc.acc_lowrank_adamw_step(desc, hyper, P, k, V, Gr, M, Vm, W, ws_o)

    def reset():
        W.copy_(W0); M.zero_(); Vm.zero_()

    enqueue()
    torch.cuda.synchronize()
    eager = {n_: t.clone() for n_, t in (("W", W), ("M", M), ("V", Vm), ("P", P), ("Y", Y), ("dX", dX))}
    assert not torch.equal(W, W0)
    reset()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for rep in range(3):
        reset()
        for t in (P, Y, dX):
            t.fill_(3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n_, t in (("W", W), ("M", M), ("V", Vm), ("P", P), ("Y", Y), ("dX", dX)):
            assert torch.equal(t, eager[n_]), (rep, n_)
