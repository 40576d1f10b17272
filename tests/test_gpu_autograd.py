"""The autograd wrapper (operator workflow of Def. 3.1) against the oracle and against exact PyTorch autograd."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import acc_oracle as orc


@pytest.fixture(scope="module")
def mods():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_01255_amd import autograd as ag
    return torch, ag


def _f64(t):
    return t.detach().to("cpu").double().numpy()


def _rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


@pytest.mark.parametrize("compressor,rank", [("rp", 64), ("rsvd", 16)])
def test_module_matches_oracle_and_saves_only_the_factors(mods, compressor, rank):
    torch, ag = mods
    torch.manual_seed(0)
    b, t, d_in, d_out = 4, 300, 512, 384
    lin = ag.CompressedLinear(d_in, d_out, rank, bias=True, compressor=compressor, seed=3, device="cuda")
    with torch.no_grad():
        lin.bias.normal_(std=0.1)
    x = torch.randn(b, t, d_in, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    saved = []
    with torch.autograd.graph.saved_tensors_hooks(lambda z: (saved.append(tuple(z.shape)), z)[1], lambda z: z):
        y = lin(x)
    g = (torch.randn_like(y) * 0.01)
    y.backward(g)
    # what autograd keeps: the weight and the rank-r factors, never the [tokens, d_in] activation
    assert (b * t, d_in) not in saved and (b, t, d_in) not in saved, saved
    assert (d_in, rank) in saved

    X, W, B, dY = _f64(x).reshape(-1, d_in), _f64(lin.weight), _f64(lin.bias), _f64(g).reshape(-1, d_out)
    seed = 3 << 20
    if compressor == "rp":
        Y, Xs = orc.linear_fwd(X, W, seed, rank, w_out_in=True)
        dX, _, dW = orc.linear_bwd(dY, W, Xs, seed, rank, w_out_in=True)
    else:
        Y, U, V = orc.linear_fwd_rsvd(X, W, seed, rank, w_out_in=True)
        dX, _, dW = orc.linear_bwd_rsvd(dY, W, U, V, w_out_in=True)
    assert _rel(_f64(y).reshape(-1, d_out), Y + B) <= 1e-2
    assert _rel(_f64(x.grad).reshape(-1, d_in), dX) <= 1e-2
    assert _rel(_f64(lin.weight.grad), dW) <= 1e-2
    assert _rel(_f64(lin.bias.grad), orc.bias_grad(dY)) <= 1e-2


def test_input_gradient_equals_exact_autograd_and_weight_gradient_is_unbiased(mods):
    """dX is the exact layer's (Thm 3.2.2(a)); the mean of the weight gradient over fresh seeds approaches
    the exact one (Thm 3.2.1(a))."""
    torch, ag = mods
    torch.manual_seed(1)
    n, d_in, d_out, rank = 2048, 256, 128, 64
    lin = ag.CompressedLinear(d_in, d_out, rank, bias=False, seed=7, device="cuda", dtype=torch.float32)
    x = torch.randn(n, d_in, device="cuda", requires_grad=True)
    g = torch.randn(n, d_out, device="cuda") * 0.01
    xe = x.detach().clone().requires_grad_(True)
    we = lin.weight.detach().clone().requires_grad_(True)
    torch.nn.functional.linear(xe, we).backward(g)
    acc_dw = torch.zeros_like(lin.weight)
    reps = 200
    for i in range(reps):
        lin.weight.grad = None
        x.grad = None
        lin(x).backward(g)
        acc_dw += lin.weight.grad
        if i == 0:
            assert _rel(_f64(x.grad), _f64(xe.grad)) <= 1e-5
            single = _rel(_f64(lin.weight.grad), _f64(we.grad))
    mean_err = _rel(_f64(acc_dw / reps), _f64(we.grad))
    assert mean_err < single / 8, (single, mean_err)      # 1/sqrt(200) = 1/14 expected


def test_state_dict_is_interchangeable_with_nn_linear(mods):
    torch, ag = mods
    ref = torch.nn.Linear(64, 48, bias=True, device="cuda", dtype=torch.bfloat16)
    lin = ag.CompressedLinear(64, 48, 16, bias=True, device="cuda")
    lin.load_state_dict(ref.state_dict())
    x = torch.randn(100, 64, device="cuda", dtype=torch.bfloat16)
    assert torch.allclose(lin(x).float(), ref(x).float(), atol=2e-2, rtol=2e-2)


def test_a_small_network_trains_with_compressed_linears(mods):
    """End to end: a two-layer network on a synthetic regression task, AdamW, compressed vs exact linears.
    The paper's point (Thm 3.2.1(a), Sec. 5.1): unbiased compression of linear-layer activations barely
    changes the optimisation.  Loose thresholds: both runs must learn, and end within 2x of each other."""
    torch, ag = mods

    def run(make_linear):
        torch.manual_seed(0)
        d, h, n = 128, 256, 4096
        teacher = torch.nn.Sequential(torch.nn.Linear(d, h), torch.nn.SiLU(), torch.nn.Linear(h, d)).cuda()
        net = torch.nn.Sequential(make_linear(d, h), torch.nn.SiLU(), make_linear(h, d)).cuda()
        opt = torch.optim.AdamW(net.parameters(), lr=2e-3, weight_decay=0.0)
        losses = []
        for step in range(150):
            x = torch.randn(n, d, device="cuda")
            with torch.no_grad():
                y = teacher(x)
            loss = torch.nn.functional.mse_loss(net(x), y)
            opt.zero_grad(set_to_none=True)
            loss.backward()
            opt.step()
            losses.append(float(loss.detach()))
        return losses

    exact = run(lambda i, o: torch.nn.Linear(i, o))
    comp = run(lambda i, o: ag.CompressedLinear(i, o, rank=64, bias=True, dtype=torch.float32, seed=5))
    print("exact", exact[0], exact[-1], "compressed", comp[0], comp[-1], flush=True)
    assert exact[-1] < exact[0] / 5 and comp[-1] < comp[0] / 5
    assert comp[-1] < 2.0 * exact[-1] + 1e-4


def test_factored_gradient_reaches_the_low_rank_optimizer(mods):
    """factored_grad=True: backward leaves weight.grad empty and hands (left, Gr) to the module; one LowRankAdamW
    step equals the oracle's step from the same factors (read back from the module: they are the optimizer's
    inputs here, their own parity is the backward tests')."""
    torch, ag = mods
    torch.manual_seed(1)
    d_in, d_out, rank = 256, 192, 64
    lin = ag.CompressedLinear(d_in, d_out, rank, bias=False, seed=2, device="cuda", dtype=torch.float32,
                              factored_grad=True)
    w0 = _f64(lin.weight)
    x = torch.randn(512, d_in, device="cuda", requires_grad=True)
    y = lin(x)
    y.backward(torch.randn_like(y) * 0.01)
    assert lin.weight.grad is None and x.grad is not None
    left, gr = (_f64(t) for t in lin.grad_factors)
    assert left.shape == (d_in, rank) and gr.shape == (d_out, rank)
    opt = ag.LowRankAdamW([lin], lr=1e-2, betas=(0.9, 0.99), eps=1e-8, weight_decay=0.1, scale=0.5)
    opt.step()
    torch.cuda.synchronize()
    assert lin.grad_factors is None
    z = np.zeros((d_out, rank))
    want = orc.lowrank_adamw_step(w0, left, gr, z, z, step=1, lr=1e-2, beta1=0.9, beta2=0.99, eps=1e-8,
                                  weight_decay=0.1, scale=0.5, w_out_in=True)[0]
    assert _rel(_f64(lin.weight) - w0, want - w0) <= 1e-3


@pytest.mark.parametrize("compressor,rank,proj_rank", [("rsvd", 32, 32), ("rp", 64, 32)])
def test_a_small_network_trains_with_the_low_rank_optimizer(mods, compressor, rank, proj_rank):
    """End to end with update strategy (ii): projected moments, projector refreshed every 20 steps, no dense
    gradient anywhere.  Loose threshold: the loss must fall by at least a factor of three.  The paper reports
    this strategy somewhat below strategy (i) in accuracy; nothing tighter is claimed here."""
    torch, ag = mods
    torch.manual_seed(0)
    d, h, n = 128, 256, 4096
    teacher = torch.nn.Sequential(torch.nn.Linear(d, h), torch.nn.SiLU(), torch.nn.Linear(h, d)).cuda()
    mk = lambda i, o, s: ag.CompressedLinear(i, o, rank=rank, bias=False, compressor=compressor, dtype=torch.float32,
                                             seed=s, factored_grad=True)
    net = torch.nn.Sequential(mk(d, h, 5), torch.nn.SiLU(), mk(h, d, 6)).cuda()
    opt = ag.LowRankAdamW(list(net), lr=3e-3, proj_rank=proj_rank, proj_gap=20, seed=1)
    losses = []
    for step in range(200):
        x = torch.randn(n, d, device="cuda")
        with torch.no_grad():
            y = teacher(x)
        loss = torch.nn.functional.mse_loss(net(x), y)
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    print(compressor, "low-rank AdamW", losses[0], losses[-1], flush=True)
    assert all(p.grad is None for p in net.parameters())
    assert losses[-1] < losses[0] / 3
