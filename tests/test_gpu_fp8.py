"""The exact products on 8-bit operands (acc_linear_fwd_fp8 / acc_linear_bwd_fp8) against the oracle.

The inputs are the seeded workloads, cast on the host to fp8 with a per-tensor scale (the cast an fp8 training
recipe applies); the oracle receives the dequantised values in fp64, so what is compared is the arithmetic of the
layer on exactly those operands: Y = scale (X8 . W8), dX = scale (dY8 . W8^T), bf16 outputs, the spec bar
plus the per-block and per-element companions.  The sketches are taken from the bf16 tensors as in the bf16 path."""
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


def _cast(a_bits, fmt):
    """bf16 bit patterns -> (fp8 bits, dequantisation scale): the tensor's largest magnitude lands on the format's."""
    a = inputs.bf16_bits_to_f32(a_bits)
    amax = float(max(np.max(a), -np.min(a)))
    q = inputs.fp8_max(fmt) / amax if amax > 0 else 1.0
    q = 2.0 ** np.floor(np.log2(q))                       # power-of-two scale: the cast itself adds no rounding of its own
    a *= np.float32(q)
    return inputs.f32_to_fp8_bits(a, fmt), 1.0 / q


def _device_pass(acc, lin, data, w_out_in, dy_fmt, want_dw=True):
    """Forward + backward through the fp8 entry points.  Returns (outputs as float64, the 8-bit casts and scales)."""
    import torch
    dev = "cuda:0"
    flags = acc.ACC_FLAG_W_OUT_IN if w_out_in else 0
    x8, sx = _cast(data["X"], "e4m3")
    w8, sw = _cast(data["W"], "e4m3")
    dy8, sdy = _cast(data["dY"], dy_fmt)
    w_bits = np.ascontiguousarray(w8.T) if w_out_in else w8
    X, dY = acc.to_device(data["X"], dev), acc.to_device(data["dY"], dev)
    X8, W8, dY8 = (torch.from_numpy(a).to(dev) for a in (x8, w_bits, dy8))
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed, flags=flags)
    Y = torch.full((lin.n, lin.d_out), 7.0, dtype=torch.bfloat16, device=dev)
    dX = torch.full((lin.n, lin.d_in), 7.0, dtype=torch.bfloat16, device=dev)
    Xs = torch.full((lin.d_in, lin.r), 7.0, dtype=torch.bfloat16, device=dev)
    Gr = torch.full((lin.d_out, lin.r) if w_out_in else (lin.r, lin.d_out), 7.0, dtype=torch.bfloat16, device=dev)
    dW = torch.full((lin.d_out, lin.d_in) if w_out_in else (lin.d_in, lin.d_out), 7.0, dtype=torch.bfloat16,
                    device=dev) if want_dw else None
    acc.acc_linear_fwd_fp8(desc, X, X8, W8, sx * sw, Y, Xs, acc.alloc_workspace(desc, False, dev))
    fmt_code = acc.ACC_FP8_E4M3 if dy_fmt == "e4m3" else acc.ACC_FP8_E5M2
    acc.acc_linear_bwd_fp8(desc, dY, dY8, fmt_code, W8, sdy * sw, Xs, dX, Gr, dW, acc.alloc_workspace(desc, True, dev))
    torch.cuda.synchronize()
    got = {"Y": acc.to_host_f64(Y), "Xs": acc.to_host_f64(Xs), "dX": acc.to_host_f64(dX), "Gr": acc.to_host_f64(Gr)}
    if want_dw:
        got["dW"] = acc.to_host_f64(dW)
    return got, {"x8": x8, "w8": w8, "dy8": dy8, "sx": sx, "sw": sw, "sdy": sdy}


def _run(acc, lin, data, w_out_in, dy_fmt, want_dw=True):
    got, q = _device_pass(acc, lin, data, w_out_in, dy_fmt, want_dw)
    # the oracle on the dequantised operands (exact products) and on the bf16 tensors (sketches)
    Xq = inputs.fp8_bits_to_f64(q["x8"], "e4m3") * q["sx"]
    Wq = inputs.fp8_bits_to_f64(q["w8"], "e4m3") * q["sw"]
    dYq = inputs.fp8_bits_to_f64(q["dy8"], dy_fmt) * q["sdy"]
    S = orc.sketch_matrix(lin.seed, lin.n, lin.r, 0)
    Wo = np.ascontiguousarray(Wq.T) if w_out_in else Wq
    Yq, _ = orc.linear_fwd(Xq, Wo, S=S, w_out_in=w_out_in)
    _, Xs_o = orc.linear_fwd(inputs.as_f64(data["X"]), Wo, S=S, w_out_in=w_out_in)
    dXq, _, _ = orc.linear_bwd(dYq, Wo, Xs_o, S=S, want_dW=False, w_out_in=w_out_in)
    _, Gr_o, dW_o = orc.linear_bwd(inputs.as_f64(data["dY"]), Wo, Xs_o, S=S, want_dW=want_dw, w_out_in=w_out_in)
    want = {"Y": Yq, "Xs": Xs_o, "dX": dXq, "Gr": Gr_o}
    if want_dw:
        want["dW"] = dW_o
    return got, want


@pytest.mark.parametrize("w_out_in", [False, True])
@pytest.mark.parametrize("n,d_in,d_out,r,dy_fmt", [
    (700, 512, 640, 64, "e4m3"),      # 3 x 3 and 3 x 2 tiles with ragged last rows, four and five K tiles
    (1000, 384, 1152, 32, "e5m2"),    # the shortest contraction the path takes (three K tiles), half a tile of columns
    (256, 1024, 384, 64, "e5m2"),     # one row of tiles
])
def test_fp8_exact_products_small(acc, n, d_in, d_out, r, dy_fmt, w_out_in):
    lin = inputs.Linear(f"fp8_{n}_{d_in}_{d_out}", n, d_in, d_out, r, seed=11)
    data = inputs.make(lin)
    print(f"fp8 case n={n} {d_in}->{d_out} r={r} dY8={dy_fmt} w_out_in={w_out_in}", flush=True)
    got, want = _run(acc, lin, data, w_out_in, dy_fmt)
    gu.check_outputs(got, want, 1e-2, lin.name)


def test_fp8_c2_every_element(acc):
    """The benchmark's projection (n = 16384, 3072 -> 3072, r = 256) in the launch configuration bench.py times:
    every element of every output."""
    lin = inputs.config("c2")[0]
    data = inputs.make(lin)
    print("fp8 c2 whole outputs", flush=True)
    got, want = _run(acc, lin, data, False, "e5m2")
    gu.check_outputs(got, want, 1e-2, lin.name + ".fp8")


def test_fp8_factors_equal_the_bf16_path_bit_for_bit(acc):
    """The sketches do not depend on the 8-bit operands: Xs, Gr and dW of the fp8 calls are the bits the bf16
    calls produce on the same X and dY."""
    lin = inputs.Linear("fp8_same_factors", 2048, 1024, 768, 64, seed=5)
    data = inputs.make(lin)
    got8, _ = _device_pass(acc, lin, data, False, "e4m3")
    got16 = gu.run_layer(acc, lin, data)
    for k in ("Xs", "Gr", "dW"):
        assert np.array_equal(got8[k], got16[k]), k


@pytest.mark.parametrize("cfg,name", [("c4", "c4.gate"), ("c5", "c5.down")])
def test_fp8_large_linears_sampled(acc, cfg, name):
    """3072 -> 8192 (32 x 64 output tiles) and the 8B-shaped down projection (n = 65536, 14336 -> 4096: 112 K tiles
    per output tile, a 0.94 GB 8-bit input): 256 random token rows of Y and dX and three whole 256 x 256 output
    tiles of each (first, a random one, last) against the oracle on the dequantised operands."""
    lin = [l for l in inputs.config(cfg) if l.name == name][0]
    rng = np.random.default_rng(8)
    data = inputs.make(lin)
    print(f"fp8 sampled {name}", flush=True)
    got, q = _device_pass(acc, lin, data, False, "e5m2", want_dw=False)
    sx, sw, sdy = q["sx"], q["sw"], q["sdy"]
    Wq = inputs.fp8_bits_to_f64(q["w8"], "e4m3") * sw
    rows = np.sort(rng.choice(lin.n, size=256, replace=False))
    have = {"Y": got["Y"][rows], "dX": got["dX"][rows]}
    want = {"Y": orc.linear_fwd(inputs.fp8_bits_to_f64(q["x8"][rows], "e4m3") * sx, Wq, S=np.zeros((256, lin.r)))[0],
            "dX": orc.linear_bwd(inputs.fp8_bits_to_f64(q["dy8"][rows], "e5m2") * sdy, Wq, np.zeros((lin.d_in, lin.r)),
                                 S=np.zeros((256, lin.r)), want_dW=False)[0]}

    def tiles(extent_m, extent_n):
        tm, tn = -(-extent_m // 256), -(-extent_n // 256)
        picks = {(0, 0), (int(rng.integers(tm)), int(rng.integers(tn))), (tm - 1, tn - 1)}
        return [(slice(a * 256, min(extent_m, a * 256 + 256)), slice(b * 256, min(extent_n, b * 256 + 256)))
                for a, b in sorted(picks)]
    for i, (rs, cs) in enumerate(tiles(lin.n, lin.d_out)):
        have[f"Y.tile{i}"] = got["Y"][rs, cs]
        want[f"Y.tile{i}"] = orc.linear_fwd(inputs.fp8_bits_to_f64(q["x8"][rs], "e4m3") * sx, Wq[:, cs],
                                            S=np.zeros((rs.stop - rs.start, lin.r)))[0]
    for i, (rs, cs) in enumerate(tiles(lin.n, lin.d_in)):
        have[f"dX.tile{i}"] = got["dX"][rs, cs]
        want[f"dX.tile{i}"] = orc.linear_bwd(inputs.fp8_bits_to_f64(q["dy8"][rs], "e5m2") * sdy, Wq[cs],
                                             np.zeros((cs.stop - cs.start, lin.r)),
                                             S=np.zeros((rs.stop - rs.start, lin.r)), want_dW=False)[0]
    gu.check_outputs(have, want, 1e-2, name + ".fp8")


def test_hot_path_and_its_fp8_form_replay_from_a_hip_graph(acc):
    """Forward + backward + dense dW of the layer, in bf16 and on 8-bit operands, captured once and replayed: the
    calls only enqueue kernels (no allocation, no memset, no synchronisation).  Each replay runs after eager work of
    the program's own and must reproduce the eager results bit for bit."""
    import torch
    dev = "cuda:0"
    lin = inputs.Linear("graph.hot", 2100, 1024, 1536, 64, seed=9)
    data = inputs.make(lin)
    bf = torch.bfloat16
    X, W, dY = (acc.to_device(data[k], dev) for k in ("X", "W", "dY"))
    x8, sx = _cast(data["X"], "e4m3"); w8, sw = _cast(data["W"], "e4m3"); dy8, sdy = _cast(data["dY"], "e5m2")
    X8, W8, dY8 = (torch.from_numpy(a).to(dev) for a in (x8, w8, dy8))
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=lin.seed)
    out = {k: torch.empty(s, dtype=bf, device=dev) for k, s in (
        ("Y", (lin.n, lin.d_out)), ("dX", (lin.n, lin.d_in)), ("Xs", (lin.d_in, lin.r)), ("Gr", (lin.r, lin.d_out)),
        ("dW", (lin.d_in, lin.d_out)), ("Y8", (lin.n, lin.d_out)), ("dX8", (lin.n, lin.d_in)),
        ("Xs8", (lin.d_in, lin.r)), ("Gr8", (lin.r, lin.d_out)), ("dW8", (lin.d_in, lin.d_out)))}
    ws_f, ws_b = acc.alloc_workspace(desc, False, dev), acc.alloc_workspace(desc, True, dev)

    def enqueue():
        acc.acc_linear_fwd(desc, X, W, out["Y"], out["Xs"], ws_f)
        acc.acc_linear_bwd(desc, dY, W, out["Xs"], out["dX"], out["Gr"], out["dW"], ws_b)
        acc.acc_linear_fwd_fp8(desc, X, X8, W8, sx * sw, out["Y8"], out["Xs8"], ws_f)
        acc.acc_linear_bwd_fp8(desc, dY, dY8, acc.ACC_FP8_E5M2, W8, sdy * sw, out["Xs8"], out["dX8"], out["Gr8"],
                               out["dW8"], ws_b)

    enqueue()
    torch.cuda.synchronize()
    eager = {k: t.clone() for k, t in out.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in out.values():
            t.fill_(3.0)
        ws_f.fill_(0xAB); ws_b.fill_(0xCD)          # stale workspace contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, t in out.items():
            assert torch.equal(t, eager[k]), (rep, k)


def _fp8_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        n = int(rng.integers(1, 40)) * 97 + int(rng.integers(1, 97))          # ragged token counts, 98 .. 3900
        d_in = 128 * int(rng.integers(3, 13))
        d_out = 128 * int(rng.integers(3, 13))
        out.append((n, d_in, d_out, int(rng.choice([16, 64])), int(rng.integers(0, 3)) * 16,
                    int(rng.integers(0, 3)) * 16, int(rng.integers(0, 3)) * 16))
    return out


@pytest.mark.parametrize("n,d_in,d_out,r,pad_x,pad_w,pad_y", _fp8_shapes(6, 77))
def test_fp8_seeded_random_shapes_with_row_strides(acc, n, d_in, d_out, r, pad_x, pad_w, pad_y):
    """Seeded random sizes (ragged token counts, every multiple of 128 from 384 to 1536 as contraction length) with
    row strides wider than the rows (multiples of 16 bytes for the 8-bit operands): exact products against the
    oracle, padding columns untouched, in both weight orientations."""
    import torch
    dev = "cuda:0"
    lin = inputs.Linear(f"fp8_rand_{n}_{d_in}_{d_out}", n, d_in, d_out, r, seed=3)
    data = inputs.make(lin)
    x8, sx = _cast(data["X"], "e4m3"); w8, sw = _cast(data["W"], "e4m3"); dy8, sdy = _cast(data["dY"], "e5m2")
    Xq, Wq = inputs.fp8_bits_to_f64(x8, "e4m3") * sx, inputs.fp8_bits_to_f64(w8, "e4m3") * sw
    dYq = inputs.fp8_bits_to_f64(dy8, "e5m2") * sdy
    want = {"Y": orc.linear_fwd(Xq, Wq, S=np.zeros((n, r)))[0],
            "dX": orc.linear_bwd(dYq, Wq, np.zeros((d_in, r)), S=np.zeros((n, r)), want_dW=False)[0]}
    for w_out_in in (False, True):
        print(f"fp8 random case n={n} {d_in}->{d_out} pads={pad_x},{pad_w},{pad_y} w_out_in={w_out_in}", flush=True)
        w_host = np.ascontiguousarray(w8.T) if w_out_in else w8
        ldx, ldw, ldy = d_in + pad_x, w_host.shape[1] + pad_w, d_out + pad_y

        def padded(a, ld, fill):
            buf = torch.full((a.shape[0], ld), fill, dtype=a.dtype, device=dev)
            buf[:, :a.shape[1]] = a
            return buf
        X = padded(acc.to_device(data["X"], dev), ldx, float("nan"))
        dY = padded(acc.to_device(data["dY"], dev), ldy, float("nan"))
        X8 = padded(torch.from_numpy(x8).to(dev), ldx, 0x7F)       # the padding holds the format's NaN pattern
        dY8 = padded(torch.from_numpy(dy8).to(dev), ldy, 0x7F)
        W8 = padded(torch.from_numpy(w_host).to(dev), ldw, 0x7F)
        desc = acc.make_desc(n, d_in, d_out, r, seed=lin.seed, ldx=ldx, ldw=ldw, ldy=ldy,
                             flags=acc.ACC_FLAG_W_OUT_IN if w_out_in else 0)
        Y = torch.full((n, ldy), 7.0, dtype=torch.bfloat16, device=dev)
        dX = torch.full((n, ldx), 7.0, dtype=torch.bfloat16, device=dev)
        Xs = torch.empty(d_in, r, dtype=torch.bfloat16, device=dev)
        Gr = torch.empty((d_out, r) if w_out_in else (r, d_out), dtype=torch.bfloat16, device=dev)
        acc.acc_linear_fwd_fp8(desc, X, X8, W8, sx * sw, Y, Xs, acc.alloc_workspace(desc, False, dev))
        acc.acc_linear_bwd_fp8(desc, dY, dY8, acc.ACC_FP8_E5M2, W8, sdy * sw, None, dX, Gr, None,
                               acc.alloc_workspace(desc, True, dev))
        torch.cuda.synchronize()
        Yh, dXh = acc.to_host_f64(Y), acc.to_host_f64(dX)
        assert np.all(Yh[:, d_out:] == 7.0) and np.all(dXh[:, d_in:] == 7.0)
        gu.check_outputs({"Y": Yh[:, :d_out], "dX": dXh[:, :d_in]}, want, 1e-2, lin.name)
