"""ctypes binding of libacc.so: same names as include/acc.h, argument marshalling only.

PyTorch appears here only as the owner of device memory and of the HIP stream; every step of
the layer runs inside the library's kernels.  There is no CPU fallback: if the library is not
built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libacc.so")

ACC_F32, ACC_BF16 = 0, 1
ACC_FLAG_SKIP_SKETCH = 1
ACC_FLAG_ONE_LAUNCH = 2
ACC_FLAG_W_OUT_IN = 4
ACC_FLAG_DW_ACCUMULATE = 8
ACC_FLAG_RSVD_POWER_SHIFT = 8   # flags bits 8..9: rounds of subspace iteration of the RSVD forward

ACC_STATIC_SCRATCH_BYTES = 32 << 20
ACC_FP8_E4M3, ACC_FP8_E5M2 = 0, 1

EXPORTS = ("acc_linear_workspace_bytes", "acc_linear_fwd", "acc_linear_fwd_static", "acc_linear_bwd", "acc_linear_dw",
           "acc_linear_fwd_fp8", "acc_linear_bwd_fp8",
           "acc_linear_bias_grad",
           "acc_rsvd_workspace_bytes", "acc_linear_fwd_rsvd", "acc_linear_bwd_rsvd", "acc_lowrank_workspace_bytes",
           "acc_lowrank_projector", "acc_lowrank_adamw_step",
           "acc_philox_dump_u32", "acc_probe_mfma",
           "acc_sketch_dump", "acc_status_string", "acc_version")


class AccLinearDesc(ctypes.Structure):
    """Mirror of `acc_linear_desc`."""
    _fields_ = [("n", ctypes.c_int64), ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64),
                ("r", ctypes.c_int64), ("ldx", ctypes.c_int64), ("ldw", ctypes.c_int64),
                ("ldy", ctypes.c_int64), ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
                ("io_dtype", ctypes.c_int32), ("factor_dtype", ctypes.c_int32),
                ("dw_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32), ("ldf", ctypes.c_int64)]


class AccAdamwHyper(ctypes.Structure):
    """Mirror of `acc_adamw_hyper`."""
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("scale", ctypes.c_float),
                ("step", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class AccError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libacc status {status}: {status_string(status)}")


# torch first: libacc.so must bind to the HIP runtime torch has loaded, so that torch's device
# pointers and streams are valid inside the library.
import torch  # noqa: E402,F401

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _sz, _dp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(AccLinearDesc)
_lib.acc_linear_workspace_bytes.restype = _sz
_lib.acc_linear_workspace_bytes.argtypes = [_dp, ctypes.c_int]
_lib.acc_linear_fwd.restype = ctypes.c_int
_lib.acc_linear_fwd.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_linear_fwd_static.restype = ctypes.c_int
_lib.acc_linear_fwd_static.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp]
_lib.acc_linear_bwd.restype = ctypes.c_int
_lib.acc_linear_bwd.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_linear_fwd_fp8.restype = ctypes.c_int
_lib.acc_linear_fwd_fp8.argtypes = [_dp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _sz, _vp]
_lib.acc_linear_bwd_fp8.restype = ctypes.c_int
_lib.acc_linear_bwd_fp8.argtypes = [_dp, _vp, _vp, ctypes.c_int, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_linear_dw.restype = ctypes.c_int
_lib.acc_linear_dw.argtypes = [_dp, _vp, _vp, _vp, _vp]
_lib.acc_linear_bias_grad.restype = ctypes.c_int
_lib.acc_linear_bias_grad.argtypes = [_dp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_rsvd_workspace_bytes.restype = _sz
_lib.acc_rsvd_workspace_bytes.argtypes = [_dp, ctypes.c_int]
_lib.acc_linear_fwd_rsvd.restype = ctypes.c_int
_lib.acc_linear_fwd_rsvd.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_linear_bwd_rsvd.restype = ctypes.c_int
_lib.acc_linear_bwd_rsvd.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_lowrank_adamw_step.restype = ctypes.c_int
_lib.acc_lowrank_adamw_step.argtypes = [_dp, ctypes.POINTER(AccAdamwHyper), _vp, ctypes.c_int64, _vp, _vp, _vp, _vp,
                                        _vp, _vp, _sz, _vp]
_lib.acc_lowrank_workspace_bytes.restype = _sz
_lib.acc_lowrank_workspace_bytes.argtypes = [_dp, ctypes.c_int64]
_lib.acc_lowrank_projector.restype = ctypes.c_int
_lib.acc_lowrank_projector.argtypes = [_dp, ctypes.c_int64, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.acc_philox_dump_u32.restype = ctypes.c_int
_lib.acc_philox_dump_u32.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, _vp, _vp]
_lib.acc_sketch_dump.restype = ctypes.c_int
_lib.acc_sketch_dump.argtypes = [_dp, _vp, _vp]
_lib.acc_probe_mfma.restype = ctypes.c_int
_lib.acc_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64, _vp, _sz,
                                ctypes.POINTER(ctypes.c_double), _vp]
_lib.acc_status_string.restype = ctypes.c_char_p
_lib.acc_status_string.argtypes = [ctypes.c_int]
_lib.acc_version.restype = ctypes.c_int
_lib.acc_version.argtypes = []


def status_string(status: int) -> str:
    return _lib.acc_status_string(int(status)).decode()


def acc_probe_mfma(shape, waves_per_simd, random_data, iters, sink, stream=None) -> float:
    """Enqueue one launch of the register-only MFMA loop; returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _check(_lib.acc_probe_mfma(shape, waves_per_simd, 1 if random_data else 0, iters, _ptr(sink),
                               sink.numel() * sink.element_size(), ctypes.byref(flops), _stream(stream)))
    return flops.value


def acc_version() -> int:
    return int(_lib.acc_version())


def make_desc(n, d_in, d_out, r, seed=0, io_dtype=ACC_BF16, factor_dtype=None, dw_dtype=None,
              row_offset=0, ldx=0, ldw=0, ldy=0, flags=0, ldf=0) -> AccLinearDesc:
    if factor_dtype is None:
        factor_dtype = io_dtype
    if dw_dtype is None:
        dw_dtype = io_dtype
    return AccLinearDesc(n, d_in, d_out, r, ldx, ldw, ldy, seed, row_offset, io_dtype, factor_dtype,
                         dw_dtype, flags, ldf)


def _ptr(t):
    """Device pointer of a torch tensor (or None -> NULL, or a raw int)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int):
    if status != 0:
        raise AccError(status)


def acc_linear_workspace_bytes(desc: AccLinearDesc, is_backward: bool) -> int:
    return int(_lib.acc_linear_workspace_bytes(ctypes.byref(desc), 1 if is_backward else 0))


def acc_linear_fwd(desc, X, W, Y, Xs, workspace, stream=None, ws_bytes=None):
    """Enqueue Y = X.W and Xs = X^T.S.  All tensors are caller-allocated device tensors."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_fwd(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(Y), _ptr(Xs),
                               _ptr(workspace), ws_bytes, _stream(stream)))


def acc_linear_fwd_static(desc, X, W, Y, Xs, stream=None):
    """acc_linear_fwd with the partial tiles in the library's static device array (nothing is allocated)."""
    _check(_lib.acc_linear_fwd_static(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(Y), _ptr(Xs), _stream(stream)))


def acc_linear_bwd(desc, dY, W, Xs, dX, Gr, dW, workspace, stream=None, ws_bytes=None):
    """Enqueue dX = dY.W^T, Gr = S^T.dY and (dW is not None) dW = Xs.Gr."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_bwd(ctypes.byref(desc), _ptr(dY), _ptr(W), _ptr(Xs), _ptr(dX), _ptr(Gr),
                               _ptr(dW), _ptr(workspace), ws_bytes, _stream(stream)))


def acc_linear_fwd_fp8(desc, X, X8, W8, scale, Y, Xs, workspace, stream=None, ws_bytes=None):
    """Enqueue Y = scale * (X8.W8) on 8-bit operands (uint8 tensors of fp8 e4m3 bits) and Xs = X^T.S from the bf16 X."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_fwd_fp8(ctypes.byref(desc), _ptr(X), _ptr(X8), _ptr(W8), float(scale), _ptr(Y), _ptr(Xs),
                                   _ptr(workspace), ws_bytes, _stream(stream)))


def acc_linear_bwd_fp8(desc, dY, dY8, dy8_format, W8, scale, Xs, dX, Gr, dW, workspace, stream=None, ws_bytes=None):
    """Enqueue dX = scale * (dY8.W8^T) on 8-bit operands, Gr = S^T.dY from the bf16 dY and (dW is not None) dW."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_bwd_fp8(ctypes.byref(desc), _ptr(dY), _ptr(dY8), int(dy8_format), _ptr(W8), float(scale),
                                   _ptr(Xs), _ptr(dX), _ptr(Gr), _ptr(dW), _ptr(workspace), ws_bytes,
                                   _stream(stream)))


def acc_linear_dw(desc, Xs, Gr, dW, stream=None):
    """Enqueue dW = Xs.Gr (+= with ACC_FLAG_DW_ACCUMULATE) from the two factors alone."""
    _check(_lib.acc_linear_dw(ctypes.byref(desc), _ptr(Xs), _ptr(Gr), _ptr(dW), _stream(stream)))


def acc_linear_bias_grad(desc, dY, dB, workspace, stream=None, ws_bytes=None):
    """Enqueue dB = column sums of dY (workspace: the backward one)."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_bias_grad(ctypes.byref(desc), _ptr(dY), _ptr(dB), _ptr(workspace), ws_bytes,
                                     _stream(stream)))


def acc_rsvd_workspace_bytes(desc: AccLinearDesc, is_backward: bool) -> int:
    return int(_lib.acc_rsvd_workspace_bytes(ctypes.byref(desc), 1 if is_backward else 0))


def acc_linear_fwd_rsvd(desc, X, W, Y, U, V, workspace, stream=None, ws_bytes=None):
    """Enqueue Y = X.W and the RSVD factors U [n, r], V [d_in, r] of X."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_fwd_rsvd(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(Y), _ptr(U), _ptr(V),
                                    _ptr(workspace), ws_bytes, _stream(stream)))


def acc_linear_bwd_rsvd(desc, dY, W, U, V, dX, Gr, dW, workspace, stream=None, ws_bytes=None):
    """Enqueue dX = dY.W^T, Gr = U^T.dY and (dW is not None) dW = V.Gr."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_linear_bwd_rsvd(ctypes.byref(desc), _ptr(dY), _ptr(W), _ptr(U), _ptr(V), _ptr(dX),
                                    _ptr(Gr), _ptr(dW), _ptr(workspace), ws_bytes, _stream(stream)))


def make_hyper(step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, scale=1.0) -> AccAdamwHyper:
    return AccAdamwHyper(lr, beta1, beta2, eps, weight_decay, scale, step, 0)


def acc_lowrank_workspace_bytes(desc: AccLinearDesc, k: int) -> int:
    return int(_lib.acc_lowrank_workspace_bytes(ctypes.byref(desc), int(k)))


def acc_lowrank_projector(desc, k, left, Gr, P, workspace, stream=None, ws_bytes=None):
    """Enqueue P [d_in, k] = orthonormal basis of a k-dimensional subspace of range(left . Gr)."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_lowrank_projector(ctypes.byref(desc), int(k), _ptr(left), _ptr(Gr), _ptr(P), _ptr(workspace),
                                      ws_bytes, _stream(stream)))


def acc_lowrank_adamw_step(desc, hyper, P, k, left, Gr, M, V, W, workspace, stream=None, ws_bytes=None):
    """Enqueue one AdamW update of W from the gradient factors left [d_in, r] and Gr, through the projector
    P [d_in, k] (None: the left factor is the projector, k = r); M, V fp32 [k, d_out]."""
    if ws_bytes is None:
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.acc_lowrank_adamw_step(ctypes.byref(desc), ctypes.byref(hyper), _ptr(P), int(k), _ptr(left),
                                       _ptr(Gr), _ptr(M), _ptr(V), _ptr(W), _ptr(workspace), ws_bytes,
                                       _stream(stream)))


def alloc_lowrank_workspace(desc, k: int, device="cuda:0"):
    import torch
    return torch.empty(max(acc_lowrank_workspace_bytes(desc, k), 16), dtype=torch.uint8, device=device)


def acc_philox_dump_u32(seed, row_offset, n, r, out, stream=None):
    _check(_lib.acc_philox_dump_u32(seed, row_offset, n, r, _ptr(out), _stream(stream)))


def acc_sketch_dump(desc, S, stream=None):
    _check(_lib.acc_sketch_dump(ctypes.byref(desc), _ptr(S), _stream(stream)))


# ---------------------------------------------------------------------------------------------
# convenience for tests / bench: allocation helpers (torch owns the memory, nothing is computed)
# ---------------------------------------------------------------------------------------------
def torch_dtype(code: int):
    import torch
    return torch.bfloat16 if code == ACC_BF16 else torch.float32


def to_device(arr, device="cuda:0"):
    """numpy float32 array or uint16 bf16-bit array -> device tensor of the matching dtype."""
    import numpy as np
    import torch
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def to_host_f64(t):
    """device tensor -> numpy float64 (exact widening)."""
    import torch
    return t.detach().to("cpu").to(torch.float64).numpy()


def alloc_workspace(desc, is_backward: bool, device="cuda:0", rsvd: bool = False):
    import torch
    nbytes = (acc_rsvd_workspace_bytes if rsvd else acc_linear_workspace_bytes)(desc, is_backward)
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
