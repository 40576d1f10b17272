"""Helpers for the GPU parity tests: run the layer through the C ABI, run the oracle, compare."""
import numpy as np

from paper_2605_01255_amd import inputs
from oracle import acc_oracle as orc


def rel(a, b):
    """Relative Frobenius error of a against the oracle value b."""
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def tolerance(dtype_code):
    """The spec bar: 1e-2 for bfloat16 outputs, 1e-5 for float32 outputs."""
    return 1e-2 if dtype_code == 1 else 1e-5


# ---- local companions of the whole-tensor norm ----------------------------------------------------------
# A single Frobenius norm over an output of 50 M elements cannot see a wrong 32 x 64 read-out unit or a wrong
# row (they move it by 6e-3 ... 8e-3, under the bar).  The checks below apply the same bar to every 32 x 32
# block of the output (the matrix instruction's tile, so every unit of every epilogue is a union of blocks; the
# last, ragged row and column of blocks included) and bound every single element.
#
# Bounds for bfloat16 outputs: the exact products round once to bf16 (relative error <= 2^-9 per element,
# measured 1.7e-3 rms); the factors add the bf16 rounding of S (same size, independent per term, so the sum's
# error is that fraction of the sum's own rms) -> 2.4e-3 rms; the dense gradient multiplies two rounded factors ->
# 3.7e-3 rms.  A block averages these over its elements, but a block that holds an outlier channel is in effect
# only that channel's row piece (8 to 32 values, whose errors share the rounding of one row of the factor), so
# block errors spread to a bit more than twice the mean (8.6e-3 seen on a 32 x 8 edge block of dW): the bound per
# block is twice the whole-tensor bar, 2e-2 -- a wrong block errs by 1e-1 or more.  One element can stray by
# several sigma of its surroundings' rms when its own value is small: |got - want| <= rtol |want| + atol scale,
# with rtol = 2^-8 (two roundings) and atol = 4e-2 (over ten sigma of 3.7e-3; the largest of 10^7 Gaussian errors
# is 5.5 sigma).  float32 outputs: 2e-5 per block and (1e-5, 2e-5) per element (accumulation of up to a few
# thousand terms in fp32, libm-grade generator).
# Blocks whose own norm is unusually small (cancellation, few elements) are measured against a quarter of the
# tensor's rms instead.
BLOCK = 32
FLOOR = 0.25


def _block_sums(a2, block=BLOCK):
    ri = np.arange(0, a2.shape[0], block)
    ci = np.arange(0, a2.shape[1], block)
    return np.add.reduceat(np.add.reduceat(a2, ri, axis=0), ci, axis=1)


def block_report(got, want, block=BLOCK):
    """(relative Frobenius error of every block x block tile, got - want, per-element scale).  The block error is
    taken against the floored block norm described above; the per-element scale is the larger of the rms of the
    element's row piece and of its column piece inside the block (an outlier channel's row of Xs or dW is twenty
    times its neighbours, so the block's own rms is the wrong yardstick for both), floored likewise."""
    got = np.atleast_2d(np.asarray(got, dtype=np.float64))
    want = np.atleast_2d(np.asarray(want, dtype=np.float64))
    assert got.shape == want.shape, (got.shape, want.shape)
    rows, cols = want.shape
    d = got - want
    ri, ci = np.arange(0, rows, block), np.arange(0, cols, block)
    nr = np.diff(np.append(ri, rows)).astype(np.float64)               # rows / columns in each block
    nc = np.diff(np.append(ci, cols)).astype(np.float64)
    w2 = want * want
    row_piece = np.add.reduceat(w2, ci, axis=1)                        # [rows, column blocks]
    col_piece = np.add.reduceat(w2, ri, axis=0)                        # [row blocks, cols]
    blk = np.add.reduceat(row_piece, ri, axis=0)                       # [row blocks, column blocks]
    counts = np.outer(nr, nc)
    d2 = _block_sums(d * d, block)
    ms_global = float(np.sum(blk) / want.size) if want.size else 0.0
    ms_block = np.maximum(blk / counts, FLOOR * FLOOR * ms_global)     # mean square per element, floored
    with np.errstate(divide="ignore", invalid="ignore"):
        blk_err = np.where(ms_block > 0, np.sqrt(d2 / (ms_block * counts)), np.sqrt(d2))

    def expand(a, axis, n):
        return np.repeat(a, block, axis=axis)[:n] if axis == 0 else np.repeat(a, block, axis=axis)[:, :n]
    blk_el = expand(expand(ms_block, 0, rows), 1, cols)
    row_el = expand(row_piece / nc[None, :], 1, cols)
    col_el = expand(col_piece / nr[:, None], 0, rows)
    scale_el = np.sqrt(np.maximum(np.maximum(row_el, col_el), FLOOR * FLOOR * blk_el))
    return blk_err, d, scale_el


def local_bounds(tol):
    """(per-block bound, rtol, atol) that go with a whole-tensor bar of `tol` (1e-2: bf16, 1e-5: fp32)."""
    return (2 * tol, 2.0 ** -8, 4e-2) if tol >= 1e-3 else (2 * tol, 1e-5, 2e-5)


def local_errors(got, want, tol):
    """Worst block error and worst per-element excess (<= 1 passes) of one output."""
    blk_tol, rtol, atol = local_bounds(tol)
    blk_err, d, rms_el = block_report(got, want)
    want2 = np.atleast_2d(np.asarray(want, dtype=np.float64))
    allowed = rtol * np.abs(want2) + atol * rms_el
    with np.errstate(divide="ignore", invalid="ignore"):
        excess = np.where(allowed > 0, np.abs(d) / allowed, np.where(d == 0, 0.0, np.inf))
    return (float(blk_err.max()) if blk_err.size else 0.0), (float(excess.max()) if excess.size else 0.0), blk_tol


def assert_close(got, want, tol, name=""):
    """The full bar for one output: whole-tensor relative Frobenius error, every 32 x 32 block, every element.
    Returns the whole-tensor error."""
    whole = rel(np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64))
    worst_blk, worst_el, blk_tol = local_errors(got, want, tol)
    assert whole <= tol, (name, "whole-tensor error", whole, tol)
    if not worst_blk <= blk_tol:
        blk_err = block_report(got, want)[0]
        where = np.unravel_index(int(np.argmax(blk_err)), blk_err.shape)
        raise AssertionError((name, "block error", worst_blk, blk_tol, "block", where,
                              "blocks above the bound", int(np.sum(blk_err > blk_tol))))
    assert worst_el <= 1.0, (name, "element outside rtol |want| + atol scale by a factor of", worst_el)
    return whole


def run_layer(acc, lin, data, factor_dtype=None, dw_dtype=None, want_dw=True, row_offset=0,
              pad=(0, 0, 0), flags=0, seed=None, device="cuda:0", want_db=False):
    """One forward + backward through acc_linear_fwd / acc_linear_bwd.  Returns float64 arrays.

    With ACC_FLAG_W_OUT_IN in flags the weight goes in as [d_out, d_in] and Gr / dW come back in that
    orientation ([d_out, r], [d_out, d_in]).  want_db adds "dB" from acc_linear_bias_grad."""
    import torch
    code = acc.ACC_BF16 if lin.dtype == "bf16" else acc.ACC_F32
    fcode = code if factor_dtype is None else factor_dtype
    dcode = code if dw_dtype is None else dw_dtype
    seed = lin.seed if seed is None else seed
    tdt = acc.torch_dtype(code)
    w_oi = bool(flags & acc.ACC_FLAG_W_OUT_IN)
    w_host = np.ascontiguousarray(data["W"].T) if w_oi else data["W"]
    ldx, ldw, ldy = lin.d_in + pad[0], w_host.shape[1] + pad[1], lin.d_out + pad[2]

    def padded(arr, ld):
        t = acc.to_device(arr, device)
        if ld == arr.shape[1]:
            return t, t
        buf = torch.full((arr.shape[0], ld), float("nan"), dtype=t.dtype, device=device)
        buf[:, :arr.shape[1]] = t
        return buf, buf

    X, _ = padded(data["X"], ldx)
    W, _ = padded(w_host, ldw)
    dY, _ = padded(data["dY"], ldy)
    desc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=seed, io_dtype=code, factor_dtype=fcode,
                         dw_dtype=dcode, row_offset=row_offset, ldx=ldx if pad[0] else 0,
                         ldw=ldw if pad[1] else 0, ldy=ldy if pad[2] else 0, flags=flags)
    Y = torch.full((lin.n, ldy), 7.0, dtype=tdt, device=device)
    dX = torch.full((lin.n, ldx), 7.0, dtype=tdt, device=device)
    Xs = torch.full((lin.d_in, lin.r), 7.0, dtype=acc.torch_dtype(fcode), device=device)
    gr_shape = (lin.d_out, lin.r) if w_oi else (lin.r, lin.d_out)
    dw_shape = (lin.d_out, lin.d_in) if w_oi else (lin.d_in, lin.d_out)
    Gr = torch.full(gr_shape, 7.0, dtype=acc.torch_dtype(fcode), device=device)
    dW = torch.full(dw_shape, 7.0, dtype=acc.torch_dtype(dcode), device=device) if want_dw else None
    acc.acc_linear_fwd(desc, X, W, Y, Xs, acc.alloc_workspace(desc, False, device))
    bdesc = acc.make_desc(lin.n, lin.d_in, lin.d_out, lin.r, seed=seed, io_dtype=code, factor_dtype=fcode,
                          dw_dtype=dcode, row_offset=row_offset, ldx=desc.ldx, ldw=desc.ldw, ldy=desc.ldy,
                          flags=flags & ~acc.ACC_FLAG_SKIP_SKETCH)
    ws_b = acc.alloc_workspace(bdesc, True, device)
    acc.acc_linear_bwd(bdesc, dY, W, Xs, dX, Gr, dW, ws_b)
    if want_db:
        dB = torch.full((lin.d_out,), 7.0, dtype=acc.torch_dtype(dcode), device=device)
        acc.acc_linear_bias_grad(bdesc, dY, dB, ws_b)
    torch.cuda.synchronize()
    out = {"Y": acc.to_host_f64(Y), "Xs": acc.to_host_f64(Xs), "dX": acc.to_host_f64(dX),
           "Gr": acc.to_host_f64(Gr)}
    if want_dw:
        out["dW"] = acc.to_host_f64(dW)
    if want_db:
        out["dB"] = acc.to_host_f64(dB)
    # padding columns must be untouched
    if pad[2]:
        assert np.all(out["Y"][:, lin.d_out:] == 7.0)
        out["Y"] = out["Y"][:, :lin.d_out]
    if pad[0]:
        assert np.all(out["dX"][:, lin.d_in:] == 7.0)
        out["dX"] = out["dX"][:, :lin.d_in]
    return out


def run_oracle(lin, data, want_dw=True, row_offset=0, seed=None, w_out_in=False, want_db=False):
    seed = lin.seed if seed is None else seed
    X, W, dY = (inputs.as_f64(data[k]) for k in ("X", "W", "dY"))
    if w_out_in:
        W = np.ascontiguousarray(W.T)
    S = orc.sketch_matrix(seed, lin.n, lin.r, row_offset)
    Y, Xs = orc.linear_fwd(X, W, S=S, w_out_in=w_out_in)
    dX, Gr, dW = orc.linear_bwd(dY, W, Xs, S=S, want_dW=want_dw, w_out_in=w_out_in)
    out = {"Y": Y, "Xs": Xs, "dX": dX, "Gr": Gr}
    if want_dw:
        out["dW"] = dW
    if want_db:
        out["dB"] = orc.bias_grad(dY)
    return out


def check_outputs(got, want, tol, label="", names=None):
    """Every output in `want` against the full bar (assert_close); prints one line of whole-tensor, worst-block
    and worst-element figures first, so a failing run shows all of them.  tol: a number or {name: number}."""
    names = list(names or want.keys())
    tols = {k: (tol[k] if isinstance(tol, dict) else tol) for k in names}
    stats = {}
    for k in names:
        worst_blk, worst_el, _ = local_errors(got[k], want[k], tols[k])
        stats[k] = (rel(np.asarray(got[k], dtype=np.float64), np.asarray(want[k], dtype=np.float64)), worst_blk, worst_el)
    print(label, " ".join(f"{k}={w:.2e}/blk {b:.2e}/el {e:.2f}" for k, (w, b, e) in stats.items()), flush=True)
    for k in names:
        assert_close(got[k], want[k], tols[k], f"{label}.{k}")
    return {k: v[0] for k, v in stats.items()}
