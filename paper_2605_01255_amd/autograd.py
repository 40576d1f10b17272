"""The operator-level workflow of Def. 3.1 as a PyTorch autograd function and module.

Forward: the output is exact, the input is compressed and only the compressed form is saved for the
backward pass.  Backward: the input gradient is exact (Thm 3.2.2(a)), the weight gradient is the factored
estimate of Sec. 4, materialised because `weight.grad` is a dense tensor (update strategy (i)), or, with
`factored_grad=True`, left as its two factors for `LowRankAdamW` (update strategy (ii)).

Everything numerical happens in libacc's kernels through `binding`; this file only allocates the output
tensors with torch and keeps the saved factors on the autograd context.  There is no fallback: without the
library, importing `binding` raises.
"""
from __future__ import annotations

import itertools

import torch

from . import binding as acc

_CODES = {torch.bfloat16: acc.ACC_BF16, torch.float32: acc.ACC_F32}


def _workspace(nbytes: int, device):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


class CompressedLinearFunction(torch.autograd.Function):
    """y = x @ weight.T (+ bias) with `weight` in torch.nn.Linear's [out_features, in_features] layout.

    compressor "rp": the seeded Gaussian token sketch (unbiased; keeps Xs [in_features, rank] + the seed);
    compressor "rsvd": randomized range finder + projection (keeps U [tokens, rank] and V [in_features, rank]).
    `seed` must differ from call to call for the random projection to be unbiased over a training run.
    Linears that share an input (q/k/v, gate/up; Sec. 5.1) are compressed once by stacking their weights
    into one call.
    """

    @staticmethod
    def forward(ctx, x, weight, bias, rank: int, seed: int, compressor: str = "rp", power_iters: int = 0,
                factor_sink=None):
        if x.dtype not in _CODES or weight.dtype != x.dtype:
            raise TypeError("x and weight must both be bfloat16 or both float32")
        d_out, d_in = weight.shape
        x2 = x.reshape(-1, d_in)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        w = weight if weight.is_contiguous() else weight.contiguous()
        n, code, dev = x2.shape[0], _CODES[x.dtype], x.device
        flags = acc.ACC_FLAG_W_OUT_IN
        y = torch.empty(n, d_out, dtype=x.dtype, device=dev)
        if compressor == "rp":
            desc = acc.make_desc(n, d_in, d_out, rank, seed=seed, io_dtype=code, flags=flags)
            xs = torch.empty(d_in, rank, dtype=x.dtype, device=dev)
            acc.acc_linear_fwd(desc, x2, w, y, xs, _workspace(acc.acc_linear_workspace_bytes(desc, False), dev))
            ctx.save_for_backward(w, xs)
        elif compressor == "rsvd":
            desc = acc.make_desc(n, d_in, d_out, rank, seed=seed, io_dtype=code,
                                 flags=flags | (int(power_iters) << acc.ACC_FLAG_RSVD_POWER_SHIFT))
            u = torch.empty(n, rank, dtype=x.dtype, device=dev)
            v = torch.empty(d_in, rank, dtype=x.dtype, device=dev)
            acc.acc_linear_fwd_rsvd(desc, x2, w, y, u, v, _workspace(acc.acc_rsvd_workspace_bytes(desc, False), dev))
            ctx.save_for_backward(w, u, v)
        else:
            raise ValueError("compressor must be 'rp' or 'rsvd'")
        if bias is not None:
            y += bias
        ctx.meta = (compressor, n, d_in, d_out, rank, seed, code, bias is not None, x.shape)
        ctx.factor_sink = factor_sink
        return y.reshape(*x.shape[:-1], d_out)

    @staticmethod
    def backward(ctx, dy):
        compressor, n, d_in, d_out, rank, seed, code, has_bias, x_shape = ctx.meta
        dy2 = dy.reshape(n, d_out)
        if not dy2.is_contiguous():
            dy2 = dy2.contiguous()
        dev, dt = dy.device, dy.dtype
        dx = torch.empty(n, d_in, dtype=dt, device=dev)
        gr = torch.empty(d_out, rank, dtype=dt, device=dev)
        sink = ctx.factor_sink
        dw = None if sink is not None else torch.empty(d_out, d_in, dtype=dt, device=dev)
        desc = acc.make_desc(n, d_in, d_out, rank, seed=seed, io_dtype=code, flags=acc.ACC_FLAG_W_OUT_IN)
        if compressor == "rp":
            w, xs = ctx.saved_tensors
            ws = _workspace(acc.acc_linear_workspace_bytes(desc, True), dev)
            acc.acc_linear_bwd(desc, dy2, w, xs, dx, gr, dw, ws)
            left = xs
        else:
            w, u, v = ctx.saved_tensors
            ws = _workspace(max(acc.acc_rsvd_workspace_bytes(desc, True), acc.acc_linear_workspace_bytes(desc, True)), dev)
            acc.acc_linear_bwd_rsvd(desc, dy2, w, u, v, dx, gr, dw, ws)
            left = v
        if sink is not None:   # the weight gradient stays factored: left [d_in, r], gr [d_out, r]
            sink.grad_factors = (left, gr)
        db = None
        if has_bias:
            db = torch.empty(d_out, dtype=dt, device=dev)
            bdesc = acc.make_desc(n, d_in, d_out, rank, seed=seed, io_dtype=code)
            acc.acc_linear_bias_grad(bdesc, dy2, db, _workspace(acc.acc_linear_workspace_bytes(bdesc, True), dev))
        return dx.reshape(x_shape), dw, db, None, None, None, None, None


class CompressedLinear(torch.nn.Module):
    """Drop-in for torch.nn.Linear (same parameter names and layout) that keeps only the compressed input
    for the backward pass.  Each forward call draws a fresh sketch seed from a per-module counter."""

    def __init__(self, in_features: int, out_features: int, rank: int, bias: bool = True, compressor: str = "rp",
                 seed: int = 0, power_iters: int = 0, device=None, dtype=torch.bfloat16, factored_grad: bool = False):
        super().__init__()
        self.factored_grad = factored_grad
        self.grad_factors = None   # (left [in, rank], gr [out, rank]) of the last backward pass when factored_grad
        self.in_features, self.out_features, self.rank = in_features, out_features, rank
        self.compressor, self.power_iters = compressor, power_iters
        self.weight = torch.nn.Parameter(torch.empty(out_features, in_features, device=device, dtype=dtype))
        if bias:
            self.bias = torch.nn.Parameter(torch.zeros(out_features, device=device, dtype=dtype))
        else:
            self.register_parameter("bias", None)
        torch.nn.init.normal_(self.weight, std=0.02)
        self._seeds = itertools.count(int(seed) << 20)

    def forward(self, x):
        return CompressedLinearFunction.apply(x, self.weight, self.bias, self.rank, next(self._seeds),
                                              self.compressor, self.power_iters,
                                              self if self.factored_grad else None)

    def extra_repr(self):
        return (f"in_features={self.in_features}, out_features={self.out_features}, rank={self.rank}, "
                f"compressor={self.compressor}, bias={self.bias is not None}")


class LowRankAdamW:
    """Update strategy (ii) of Sec. 4 for `CompressedLinear(..., factored_grad=True)` modules: AdamW whose moments
    have the shape [out_features, proj_rank]; the weights are updated in place by acc_lowrank_adamw_step, and no
    dense gradient or dense optimizer state is ever allocated.

    proj_rank > 0: moments live in the range of a projector [in_features, proj_rank] computed from the factored
    gradient by acc_lowrank_projector and refreshed every `proj_gap` steps (the moments are kept across a
    refresh).  proj_rank = 0: the left factor of each step is its own projector.  One backward pass per step
    (factors of several micro-batches cannot be summed).  Biases are left to an ordinary optimizer.
    """

    def __init__(self, modules, lr: float = 1e-3, betas=(0.9, 0.999), eps: float = 1e-8, weight_decay: float = 0.0,
                 scale: float = 1.0, proj_rank: int = 0, proj_gap: int = 200, seed: int = 0):
        self.modules = [m for m in modules if isinstance(m, CompressedLinear) and m.factored_grad]
        if not self.modules:
            raise ValueError("no CompressedLinear module with factored_grad=True")
        self.lr, self.betas, self.eps, self.weight_decay, self.scale = lr, betas, eps, weight_decay, scale
        self.proj_rank, self.proj_gap, self.seed = int(proj_rank), int(proj_gap), int(seed)
        self.state = {}

    @torch.no_grad()
    def step(self):
        k = self.proj_rank
        for idx, m in enumerate(self.modules):
            if m.grad_factors is None:
                continue
            left, gr = m.grad_factors
            w = m.weight.data
            if not w.is_contiguous():
                raise ValueError("weight must be contiguous to be updated in place")
            st = self.state.get(m)
            if st is None:
                rows = k if k else m.rank
                st = self.state[m] = {
                    "step": 0,
                    "exp_avg": torch.zeros(m.out_features, rows, dtype=torch.float32, device=gr.device),
                    "exp_avg_sq": torch.zeros(m.out_features, rows, dtype=torch.float32, device=gr.device),
                    "projector": torch.empty(m.in_features, k, dtype=gr.dtype, device=gr.device) if k else None}
            refresh = k and st["step"] % self.proj_gap == 0
            st["step"] += 1
            # a fresh range-finder seed per module and refresh
            desc = acc.make_desc(1, m.in_features, m.out_features, m.rank, io_dtype=_CODES[w.dtype],
                                 factor_dtype=_CODES[gr.dtype], flags=acc.ACC_FLAG_W_OUT_IN,
                                 seed=(self.seed << 40) + (idx << 24) + st["step"] // max(self.proj_gap, 1))
            ws = _workspace(acc.acc_lowrank_workspace_bytes(desc, k), gr.device)
            if refresh:
                acc.acc_lowrank_projector(desc, k, left, gr, st["projector"], ws)
            hyper = acc.make_hyper(st["step"], self.lr, self.betas[0], self.betas[1], self.eps, self.weight_decay,
                                   self.scale)
            acc.acc_lowrank_adamw_step(desc, hyper, st["projector"], k, left, gr, st["exp_avg"], st["exp_avg_sq"],
                                       w, ws)
            m.grad_factors = None

    def zero_grad(self):
        for m in self.modules:
            m.grad_factors = None
