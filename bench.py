#!/usr/bin/env python3
"""Benchmark of the compressed linear layer on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: forward
(Y = X.W, Xs = X^T.S) and backward (dX = dY.W^T, Gr = S^T.dY, dense dW = Xs.Gr), S regenerated
from the Philox seed in both.  Inputs are resident in HBM before the timed region.
Prints ONE JSON line (metric: algorithmic TFLOP/s of fwd+bwd; S generation counts zero flops).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5000.0      # MI355X dense fp8 MFMA, published
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)  # the clocks settle over about 0.1 s of load
    ap.add_argument("--config", default="c2", help="c1 | c2 | c3_r256 | c4 | c5 (a named linear: c4.k)")
    ap.add_argument("--layer", default=None, help="c4 | c5: time all linears of a decoder layer instead (own JSON line)")
    ap.add_argument("--no-dw", action="store_true", help="leave the dense dW out of the step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--buffer-sets", type=int, default=3, help="rotated so no tensor stays in the 256 MB cache")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy 5 times (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="instead of the layer: time the register-only bf16 MFMA loop (acc_probe_mfma) on zero and on "
                         "random operands, both instruction shapes, one and two waves per SIMD (own JSON line)")
    ap.add_argument("--traffic-mb", type=float, default=None,
                    help="HBM-side MB per launch of the dominant kernel, from rocprofv3 --pmc runs; default: the figure "
                         "stored beside the counter summary of this workload under profiles/, null if there is none")
    return ap.parse_args()


def stored_traffic(workload):
    """HBM-side bytes per launch of the dominant kernel for `workload`, as measured with rocprofv3 --pmc and
    recorded beside the counter summary (a line `traffic_bytes_per_launch[<workload>] = <bytes>` in
    profiles/*_counters.md); None when no profile of this workload is stored."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*counters*.md"))):
        m = re.search(r"traffic_bytes_per_launch\[" + re.escape(workload) + r"\]\s*=\s*([0-9.eE+]+)", open(path).read())
        if m:
            return float(m.group(1))
    return None


class Buffers:
    """Device tensors of one linear layer (one rotation slot)."""

    def __init__(self, acc, torch, lin, data, dev, with_dw):
        code = acc.ACC_BF16 if lin.dtype == "bf16" else acc.ACC_F32
        tdt = acc.torch_dtype(code)
        self.X, self.W, self.dY = (acc.to_device(data[k], dev) for k in ("X", "W", "dY"))
        self.Y = torch.empty(lin.n, lin.d_out, dtype=tdt, device=dev)
        self.dX = torch.empty(lin.n, lin.d_in, dtype=tdt, device=dev)
        self.Xs = torch.empty(lin.d_in, lin.r, dtype=tdt, device=dev)
        self.Gr = torch.empty(lin.r, lin.d_out, dtype=tdt, device=dev)
        self.dW = torch.empty(lin.d_in, lin.d_out, dtype=tdt, device=dev) if with_dw else None


def time_events(torch, fn, iters):
    """Average milliseconds of fn() over iters calls, HIP events on the launch stream."""
    st = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for i in range(iters):
        fn(i)
    e1.record(st)
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def time_each(torch, fn, iters):
    """Milliseconds of every single call of fn(i), one pair of HIP events per call: (median, min)."""
    st = torch.cuda.current_stream()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for i, (a, b) in enumerate(evs):
        a.record(st)
        fn(i)
        b.record(st)
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2], ts[0]


def run_layer(args, torch, acc, inputs, dev):
    """All linears of a decoder-layer configuration (c4, c5), the linears that share an input sketched once
    (ACC_FLAG_SKIP_SKETCH on the others; Sec. 5.1: q/k/v see the same activation, so do gate/up).  Prints one
    JSON line for the layer: algorithmic TFLOP/s over all linears and the activation bytes kept."""
    linears = inputs.config(args.layer)
    groups = {}                              # distinct input tensors: q,k,v | o | gate,up | down
    for l in linears:
        key = {"q": "attn_in", "k": "attn_in", "v": "attn_in", "gate": "mlp_in", "up": "mlp_in"}.get(
            l.name.split(".")[-1], l.name)
        groups.setdefault(key, []).append(l)
    bf, items = torch.bfloat16, []
    torch.manual_seed(inputs.DATA_SEED)      # dY is drawn on the device: N(0, 0.01^2), seeded
    for key, ls in groups.items():
        first = ls[0]
        X = acc.to_device(inputs.store(inputs.make_x(first), first.dtype), dev)
        Xs = torch.empty(first.d_in, first.r, dtype=bf, device=dev)
        for i, l in enumerate(ls):
            W = acc.to_device(inputs.store(inputs.make_w(l), l.dtype), dev)
            dY = torch.randn(l.n, l.d_out, device=dev, dtype=torch.float32).mul_(0.01).to(bf)
            fl = acc.ACC_FLAG_SKIP_SKETCH if i else 0
            fd = acc.make_desc(l.n, l.d_in, l.d_out, l.r, seed=first.seed, flags=fl)
            bd = acc.make_desc(l.n, l.d_in, l.d_out, l.r, seed=first.seed)
            items.append(dict(l=l, X=X, W=W, dY=dY, Xs=Xs, fd=fd, bd=bd, sketch=(i == 0),
                              Y=torch.empty(l.n, l.d_out, dtype=bf, device=dev),
                              dX=torch.empty(l.n, l.d_in, dtype=bf, device=dev),
                              Gr=torch.empty(l.r, l.d_out, dtype=bf, device=dev),
                              dW=torch.empty(l.d_in, l.d_out, dtype=bf, device=dev),
                              ws_f=acc.alloc_workspace(bd, False, dev), ws_b=acc.alloc_workspace(bd, True, dev)))

    def step(_):
        for it in items:
            acc.acc_linear_fwd(it["fd"], it["X"], it["W"], it["Y"], it["Xs"], it["ws_f"] if it["sketch"] else None)
        for it in reversed(items):
            acc.acc_linear_bwd(it["bd"], it["dY"], it["W"], it["Xs"], it["dX"], it["Gr"], it["dW"], it["ws_b"])

    steps, warm = max(3, args.steps // 5), max(1, args.warmup // 5)
    for i in range(warm):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flops = 0
    for it in items:
        l = it["l"]
        flops += 4 * l.n * l.d_in * l.d_out + 2 * l.n * l.r * l.d_out + 2 * l.d_in * l.r * l.d_out
        if it["sketch"]:
            flops += 2 * l.n * l.d_in * l.r
    dense = sum(ls[0].n * ls[0].d_in * 2 for ls in groups.values())
    kept = sum(ls[0].d_in * ls[0].r * 2 + 8 for ls in groups.values())
    n = linears[0].n
    print(json.dumps({
        "metric": "compressed decoder-layer linears fwd+bwd TFLOP/s", "value": round(flops / (ms * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.layer}: {len(items)} linears, n={n}, shared sketches for q/k/v and gate/up",
                   "with_dw": True},
        "activation_bytes": {"dense_per_distinct_input": dense, "kept": kept, "ratio": round(dense / kept, 2),
                             "dense_per_token": dense / n, "kept_per_token": round(kept / n, 3)}}), flush=True)


def run_mfma_ceiling(args, torch, acc, dev):
    """What the matrix pipe sustains with nothing else running: the practical ceiling of the MFMA-bound steps."""
    sink = torch.empty(256 * 512, dtype=torch.float32, device=dev)
    iters, rows = 20000, []
    for shape, name in ((0, "32x32x16 bf16"), (1, "16x16x32 bf16"), (2, "16x16x128 fp8")):
        for waves in (1, 2):
            for rnd in (0, 1):
                def launch(_):
                    return acc.acc_probe_mfma(shape, waves, rnd, iters, sink)
                flops = launch(0)
                for i in range(max(2, args.warmup // 20)):     # ~1 ms per launch: the clocks settle under load
                    launch(i)
                ms = time_events(torch, launch, max(5, args.steps // 10))
                rows.append({"mfma": name, "waves_per_simd": waves, "operands": "random" if rnd else "zeros",
                             "ms_per_launch": round(ms, 4), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                             "frac_of_peak": round(flops / (ms * 1e-3) / 1e12 / (PEAK_BF16_TFLOPS * (2 if shape == 2 else 1)), 4)})
    print(json.dumps({"metric": "register-only MFMA loop TFLOP/s (peaks: bf16 2500, fp8 5000)", "unit": "TFLOP/s", "n_gpus": 1,
                      "config": {"workload": f"256 work-groups, {iters} x 4 matrix instructions per wave"},
                      "rows": rows}), flush=True)


def cpu_baseline(lin, data, with_dw, budget_tokens):
    """The oracle, as it stands, timed on a bounded token sample of the same workload."""
    import numpy as np
    from oracle import acc_oracle as orc
    from paper_2605_01255_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    ns = min(lin.n, budget_tokens)
    X = inputs.as_f64(data["X"][:ns]); W = inputs.as_f64(data["W"]); dY = inputs.as_f64(data["dY"][:ns])
    # whole passes of the oracle over the sample until about 10 s of CPU work are spent (at most 12 passes)
    times = []
    while len(times) < 12 and sum(times) < 10.0:
        t0 = time.perf_counter()
        Y, Xs = orc.linear_fwd(X, W, lin.seed, lin.r)
        dX, Gr, dW = orc.linear_bwd(dY, W, Xs, lin.seed, lin.r, want_dW=with_dw)
        times.append(time.perf_counter() - t0)
    dt = sum(times) / len(times)
    flops = 4 * ns * lin.d_in * lin.d_out + 2 * ns * lin.r * (lin.d_in + lin.d_out)
    if with_dw:
        flops += 2 * lin.d_in * lin.r * lin.d_out
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {ns} of {lin.n} tokens, fp64 numpy fwd+bwd{'+dW' if with_dw else ''}, "
                      f"mean of {len(times)} passes, {dt:.2f} s each"}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_01255_amd import binding as acc, inputs

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.mfma_ceiling:
        run_mfma_ceiling(args, torch, acc, dev)
        return
    if args.layer:
        run_layer(args, torch, acc, inputs, dev)
        return
    cfg, _, which = args.config.partition(".")
    linears = inputs.config(cfg)
    if which:
        linears = [l for l in linears if l.name in (args.config, which)]
    with_dw = not args.no_dw
    lin = linears[0]                       # the benchmark line is quoted on the first linear of the config
    data = inputs.make(lin)
    code = acc.ACC_BF16 if lin.dtype == "bf16" else acc.ACC_F32
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=code)
    sets = [Buffers(acc, torch, lin, data, dev, with_dw) for _ in range(max(1, args.buffer_sets))]
    ws_f = acc.alloc_workspace(desc, False, dev)
    ws_b = acc.alloc_workspace(desc, True, dev)

    def fwd(i):
        b = sets[i % len(sets)]
        acc.acc_linear_fwd(desc, b.X, b.W, b.Y, b.Xs, ws_f)

    def bwd(i):
        b = sets[i % len(sets)]
        acc.acc_linear_bwd(desc, b.dY, b.W, b.Xs, b.dX, b.Gr, b.dW, ws_b)

    def step(i):
        fwd(i)
        bwd(i)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Order of the legs: the rows beside the headline run first (small kernels, then the layer in the other weight
    # orientation and single steps), then the headline region (warm-up, timed steps), then the per-phase and
    # single-kernel timings.  The part raises its clocks over the first 20-30 ms of heavy load after idling or after
    # a run of small kernels (measured: single steps 0.77, 0.75, 0.72, ... 0.60 ms when the region starts 3 ms after
    # idle, 0.58 ms once settled), and host-side input generation leaves it idle for seconds, so a region that came
    # first with a short warm-up would time that ramp; `timed_region` shows the single steps of the region either way.
    flops = lin.flops(with_dw)
    step(0)
    # rows added after the hot path: bias gradient (HBM-bound column sum of dY) and the layer with W in
    # the [d_out, d_in] orientation; reported beside the headline, not part of `value`
    tdt = acc.torch_dtype(code)
    dB = torch.empty(lin.d_out, dtype=tdt, device=dev)

    def bias_grad(i):
        acc.acc_linear_bias_grad(desc, sets[i % len(sets)].dY, dB, ws_b)

    bias_grad(0)
    ms_db = time_events(torch, bias_grad, args.steps)
    db_bytes = lin.n * lin.d_out * (2 if lin.dtype == "bf16" else 4)
    desc_oi = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=code,
                            flags=acc.ACC_FLAG_W_OUT_IN)
    w_oi = [b.W.t().contiguous() for b in sets]
    gr_oi = torch.empty(lin.d_out, lin.r, dtype=tdt, device=dev)
    dw_oi = torch.empty(lin.d_out, lin.d_in, dtype=tdt, device=dev) if with_dw else None

    def step_oi(i):
        b = sets[i % len(sets)]
        acc.acc_linear_fwd(desc_oi, b.X, w_oi[i % len(sets)], b.Y, b.Xs, ws_f)
        acc.acc_linear_bwd(desc_oi, b.dY, w_oi[i % len(sets)], b.Xs, b.dX, gr_oi, dw_oi, ws_b)

    step_oi(0)
    # RSVD compressor at the paper's rank 32 on the same layer (U [n, 32] + V [d_in, 32] kept)
    k_rsvd = 32
    desc_rs = acc.make_desc(lin.n, lin.d_in, lin.d_out, k_rsvd, seed=lin.seed, io_dtype=code)
    ws_rf = acc.alloc_workspace(desc_rs, False, dev, rsvd=True)
    ws_rb = acc.alloc_workspace(desc_rs, True, dev, rsvd=True)
    U_rs = torch.empty(lin.n, k_rsvd, dtype=tdt, device=dev)
    V_rs = torch.empty(lin.d_in, k_rsvd, dtype=tdt, device=dev)
    Gr_rs = torch.empty(k_rsvd, lin.d_out, dtype=tdt, device=dev)

    def fwd_rsvd(i):
        b = sets[i % len(sets)]
        acc.acc_linear_fwd_rsvd(desc_rs, b.X, b.W, b.Y, U_rs, V_rs, ws_rf)

    def bwd_rsvd(i):
        b = sets[i % len(sets)]
        acc.acc_linear_bwd_rsvd(desc_rs, b.dY, b.W, U_rs, V_rs, b.dX, Gr_rs, b.dW, ws_rb)

    fwd_rsvd(0); bwd_rsvd(0)
    n_rs = max(5, args.steps // 4)
    ms_rf = time_events(torch, fwd_rsvd, n_rs)
    ms_rb = time_events(torch, bwd_rsvd, n_rs)
    # the same forward with two rounds of subspace iteration (four more passes over X)
    desc_rs2 = acc.make_desc(lin.n, lin.d_in, lin.d_out, k_rsvd, seed=lin.seed, io_dtype=code,
                             flags=2 << acc.ACC_FLAG_RSVD_POWER_SHIFT)
    ws_rf2 = acc.alloc_workspace(desc_rs2, False, dev, rsvd=True)

    def fwd_rsvd2(i):
        b = sets[i % len(sets)]
        acc.acc_linear_fwd_rsvd(desc_rs2, b.X, b.W, b.Y, U_rs, V_rs, ws_rf2)

    fwd_rsvd2(0)
    ms_rf2 = time_events(torch, fwd_rsvd2, n_rs)
    # optimizer step on the factored gradient (update strategy (ii)): the weight is updated from Xs and Gr of the
    # backward pass; no dense gradient, moments [k, d_out].  The weight is a scratch copy: the step count is pinned
    # at 1 and lr at 0 so that the timed repetitions leave it finite.
    k_opt = 64
    w_opt = sets[0].W.clone()
    ws_opt = acc.alloc_lowrank_workspace(desc, k_opt, dev)
    P_opt = torch.empty(lin.d_in, k_opt, dtype=tdt, device=dev)
    m_k = torch.zeros(k_opt, lin.d_out, dtype=torch.float32, device=dev)
    v_k = torch.zeros(k_opt, lin.d_out, dtype=torch.float32, device=dev)
    m_r = torch.zeros(lin.r, lin.d_out, dtype=torch.float32, device=dev)
    v_r = torch.zeros(lin.r, lin.d_out, dtype=torch.float32, device=dev)
    hyper = acc.make_hyper(1, lr=0.0, weight_decay=0.0)
    xs0, gr0 = sets[0].Xs, sets[0].Gr

    def opt_projector(i):
        acc.acc_lowrank_projector(desc, k_opt, xs0, gr0, P_opt, ws_opt)

    def opt_step_projected(i):
        acc.acc_lowrank_adamw_step(desc, hyper, P_opt, k_opt, xs0, gr0, m_k, v_k, w_opt, ws_opt)

    def opt_step_left(i):
        acc.acc_lowrank_adamw_step(desc, hyper, None, 0, xs0, gr0, m_r, v_r, w_opt, ws_opt)

    opt_projector(0); opt_step_projected(0); opt_step_left(0)
    ms_proj = time_events(torch, opt_projector, n_rs)
    ms_optk = time_events(torch, opt_step_projected, args.steps)
    ms_optr = time_events(torch, opt_step_left, args.steps)
    w_bytes = 2 * lin.d_in * lin.d_out * (2 if lin.dtype == "bf16" else 4)   # W read and written once
    # the exact products on 8-bit copies of the operands (fp8 e4m3 for X and W, e5m2 for dY; per-tensor power-of-two
    # scales, cast here on the device: input preparation), everything else of the step unchanged
    fp8_ok = (lin.dtype == "bf16" and lin.d_in % 128 == 0 and lin.d_out % 128 == 0 and min(lin.d_in, lin.d_out) >= 384)
    ms_fp8 = ms_fp8_gemm = None
    if fp8_ok:
        def cast8(t, tdtype, top):
            q = 2.0 ** math.floor(math.log2(top / float(t.abs().max())))
            return (t.float() * q).to(tdtype).view(torch.uint8), 1.0 / q
        x8 = [cast8(b.X, torch.float8_e4m3fn, 448.0) for b in sets]
        dy8 = [cast8(b.dY, torch.float8_e5m2, 57344.0) for b in sets]
        w8, sw8 = cast8(sets[0].W, torch.float8_e4m3fn, 448.0)
        desc_ns = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=code,
                                flags=acc.ACC_FLAG_SKIP_SKETCH)

        def step_fp8(i):
            k = i % len(sets)
            b = sets[k]
            acc.acc_linear_fwd_fp8(desc, b.X, x8[k][0], w8, x8[k][1] * sw8, b.Y, b.Xs, ws_f)
            acc.acc_linear_bwd_fp8(desc, b.dY, dy8[k][0], acc.ACC_FP8_E5M2, w8, dy8[k][1] * sw8, b.Xs, b.dX, b.Gr,
                                   b.dW, ws_b)

        def gemm_fp8(i):
            k = i % len(sets)
            acc.acc_linear_fwd_fp8(desc_ns, None, x8[k][0], w8, x8[k][1] * sw8, sets[k].Y, None, None)

        step_fp8(0); gemm_fp8(0)
    # the heavy legs last: the small kernels above let the clocks fall again
    if fp8_ok:
        ms_fp8_gemm = time_events(torch, gemm_fp8, args.steps)
        ms_fp8 = time_events(torch, step_fp8, args.steps)
    ms_oi = time_events(torch, step_oi, args.steps)
    step_median, step_min = time_each(torch, step, args.steps)
    widened = {
        "lowrank_adamw": {"projector_rank": k_opt, "ms_step_projected": round(ms_optk, 4),
                          "ms_step_left_factor_as_projector": round(ms_optr, 4),
                          "ms_projector_refresh": round(ms_proj, 4), "bound": "hbm",
                          "achieved": round(w_bytes / (ms_optk * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                          "unit": "GB/s", "frac": round(w_bytes / (ms_optk * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                          "state_bytes": 2 * k_opt * lin.d_out * 4 + lin.d_in * k_opt * 2,
                          "dense_adamw_state_bytes": 2 * lin.d_in * lin.d_out * 4},
        "rsvd_rank32": {"ms_fwd": round(ms_rf, 4), "ms_bwd": round(ms_rb, 4), "ms_fwd_2_subspace_iterations": round(ms_rf2, 4),
                        "kept_bytes_per_token": round((lin.n + lin.d_in) * k_rsvd * 2 / lin.n, 2)},
        "bias_grad": {"ms": round(ms_db, 4), "bound": "hbm", "achieved": round(db_bytes / (ms_db * 1e-3) / 1e9, 1),
                      "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(db_bytes / (ms_db * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "w_out_in": {"ms_per_step": round(ms_oi, 4), "value": round(flops / (ms_oi * 1e-3) / 1e12, 2), "unit": "TFLOP/s"},
    }
    if fp8_ok:
        gemm_flops = 2.0 * lin.n * lin.d_in * lin.d_out
        widened["fp8_exact_products"] = {
            "ms_per_step": round(ms_fp8, 4), "value": round(flops / (ms_fp8 * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
            "operands": "X8, W8 fp8 e4m3, dY8 fp8 e5m2; bf16 sketches, factors and outputs",
            "gemm_alone": {"ms": round(ms_fp8_gemm, 4), "bound": "mfma",
                           "achieved": round(gemm_flops / (ms_fp8_gemm * 1e-3) / 1e12, 1), "peak": PEAK_FP8_TFLOPS,
                           "unit": "TFLOP/s",
                           "frac": round(gemm_flops / (ms_fp8_gemm * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 4)}}
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # The timed region: exactly args.steps steps between two synchronisations, host clock.  One HIP event after
    # every step (on the launch stream; recording costs about a microsecond of host time and nothing on the GPU)
    # shows afterwards where inside the region the time went.
    st = torch.cuda.current_stream()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(st)
    for i in range(args.steps):
        step(i)
        marks[i + 1].record(st)
    t_enqueued = time.perf_counter()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    timed_region = {
        "wall_ms": round(wall * 1e3, 4), "host_enqueue_ms": round((t_enqueued - t0) * 1e3, 4),
        "first_to_last_event_ms": round(marks[0].elapsed_time(marks[-1]), 4),
        "step_ms_first5": [round(t, 4) for t in per_step[:5]],
        "step_ms_last5": [round(t, 4) for t in per_step[-5:]],
        "step_ms_median": round(sorted(per_step)[len(per_step) // 2], 4)}

    value = flops / (ms_per_step * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if lin.dtype == "bf16" else PEAK_F32_TFLOPS

    # per-phase event timings (same launches, HIP events on the launch stream)
    for i in range(len(sets)):             # every buffer set holds an Xs before a backward leg reads it
        fwd(i)
    ms_fwd = time_events(torch, fwd, args.steps)
    ms_bwd = time_events(torch, bwd, args.steps)
    # the same step with the weight gradient left in factored form (no dense dW)
    ms_bwd_nodw = None
    if with_dw:
        def bwd_nodw(i):
            b = sets[i % len(sets)]
            acc.acc_linear_bwd(desc, b.dY, b.W, b.Xs, b.dX, b.Gr, None, ws_b)
        bwd_nodw(0)
        ms_bwd_nodw = time_events(torch, bwd_nodw, args.steps)
    # dominant kernel: the exact-output GEMM Y = X.W, launched alone by a forward with the
    # sketch skipped (that call enqueues exactly one kernel)
    desc_gemm = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, io_dtype=code,
                              flags=acc.ACC_FLAG_SKIP_SKETCH)

    def gemm_only(i):
        b = sets[i % len(sets)]
        acc.acc_linear_fwd(desc_gemm, b.X, b.W, b.Y, None, None)

    gemm_only(0)
    ms_gemm = time_events(torch, gemm_only, args.steps)
    gemm_flops = 2 * lin.n * lin.d_in * lin.d_out
    achieved = gemm_flops / (ms_gemm * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "Y = X.W GEMM (acc_linear_fwd, sketch skipped)",
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "avg_kernel_ms": round(ms_gemm, 4),
                "traffic": args.traffic_mb * 1e6 if args.traffic_mb else stored_traffic(lin.name),
                "algorithmic_bytes": (lin.n * lin.d_in + lin.d_in * lin.d_out + lin.n * lin.d_out) * 2}

    dense_b, kept_b = lin.activation_bytes(2 if lin.dtype == "bf16" else 4)
    out = {
        "metric": "compressed-linear fwd+bwd TFLOP/s", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if lin.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{lin.name}: n={lin.n} tokens, {lin.d_in}->{lin.d_out}, r={lin.r}, "
                               f"{lin.dtype}, X with {lin.n_outliers} outlier channels x20"
                               if lin.x_kind == "outlier" else f"{lin.name}: n={lin.n}, {lin.d_in}->{lin.d_out}, r={lin.r}, {lin.dtype}",
                   "with_dw": with_dw, "buffer_sets": len(sets)},
        "pct_of_bf16_mfma_peak": round(100.0 * value / peak, 2),
        "ms_per_step_median": round(step_median, 4), "ms_per_step_min": round(step_min, 4),
        "timed_region": timed_region,
        "ms_fwd": round(ms_fwd, 4), "ms_bwd": round(ms_bwd, 4),
        "factored_only": None if ms_bwd_nodw is None else {
            "ms_bwd": round(ms_bwd_nodw, 4),
            "value": round(lin.flops(False) / ((ms_fwd + ms_bwd_nodw) * 1e-3) / 1e12, 2), "unit": "TFLOP/s"},
        "activation_bytes_per_token": {"dense": dense_b / lin.n, "kept": round(kept_b / lin.n, 4),
                                       "saved": round((dense_b - kept_b) / lin.n, 4),
                                       "ratio": round(dense_b / kept_b, 2)},
        "roofline": roofline,
        "widened": widened,
    }
    if not args.no_cpu_baseline:
        # the whole 3B-shaped projection is ~1-2 s of fp64 BLAS on the machine's cores; larger shapes are sampled
        budget = lin.n if lin.flops(with_dw) <= 1.5e12 else max(1024, int(lin.n * 1.5e12 / lin.flops(with_dw)) // 256 * 256)
        out["cpu_baseline"] = cpu_baseline(lin, data, with_dw, budget)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
