"""Host-side checks of the C ABI: the library loads, exports what include/acc.h declares,
the ctypes mirror of the descriptor matches the header, and invalid calls are refused before
anything touches a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "acc.h")

acc = pytest.importorskip("paper_2605_01255_amd.binding", reason="libacc.so not built")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(acc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert set(names) == set(acc.EXPORTS)
    lib = ctypes.CDLL(acc.LIB_PATH)
    for name in names:
        assert getattr(lib, name) is not None


def test_descriptor_layout_matches_header():
    text = open(HEADER).read()
    body = re.search(r"typedef struct acc_linear_desc \{(.*?)\} acc_linear_desc;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(int64_t|uint64_t|int32_t|uint32_t)\s+(\w+)\s*;", body)
    ctype = {"int64_t": ctypes.c_int64, "uint64_t": ctypes.c_uint64, "int32_t": ctypes.c_int32,
             "uint32_t": ctypes.c_uint32}
    assert [(n, ctype[t]) for t, n in fields] == list(acc.AccLinearDesc._fields_)
    assert ctypes.sizeof(acc.AccLinearDesc) == 96


def test_version_and_status_strings():
    assert acc.acc_version() >= 100
    assert acc.status_string(0) == "ACC_OK"
    for code in range(-6, 0):
        assert acc.status_string(code).startswith("ACC_ERR_")
    assert acc.status_string(-99) == "ACC_ERR_UNKNOWN"


def _fwd(desc, X=0x1000, W=0x2000, Y=0x3000, Xs=0x4000, ws=0x5000, ws_bytes=1 << 40):
    return acc._lib.acc_linear_fwd(ctypes.byref(desc), X, W, Y, Xs, ws, ws_bytes, None)


def _bwd(desc, dY=0x1000, W=0x2000, Xs=0x4000, dX=0x3000, Gr=0x6000, dW=0x7000, ws=0x5000, ws_bytes=1 << 40):
    return acc._lib.acc_linear_bwd(ctypes.byref(desc), dY, W, Xs, dX, Gr, dW, ws, ws_bytes, None)


def test_invalid_descriptors_are_refused():
    ok = dict(n=256, d_in=256, d_out=512, r=16)
    assert acc._lib.acc_linear_fwd(None, 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 1 << 30, None) == -1
    for bad in (dict(n=0), dict(d_in=0), dict(r=0), dict(r=20), dict(d_in=252), dict(d_out=516),
                dict(row_offset=2), dict(ldx=128), dict(ldx=260), dict(ldy=8), dict(n=-5),
                dict(n=(1 << 30) + 1), dict(d_in=(1 << 21) + 8), dict(r=(1 << 16) + 16)):
        d = acc.make_desc(**{**ok, **bad})
        assert _fwd(d) == -2, bad
        assert _bwd(d) == -2, bad
        assert acc.acc_linear_workspace_bytes(d, False) == 0
    assert _fwd(acc.make_desc(**ok, io_dtype=7)) == -4
    assert _fwd(acc.make_desc(**ok, factor_dtype=-1)) == -4
    assert _fwd(acc.make_desc(**ok, flags=16)) == -1
    assert _fwd(acc.make_desc(**ok, flags=1 << 8)) == -1      # subspace iterations belong to the RSVD forward
    assert _bwd(acc.make_desc(**ok, flags=acc.ACC_FLAG_SKIP_SKETCH)) == -1
    assert _fwd(acc.make_desc(**ok, flags=acc.ACC_FLAG_ONE_LAUNCH)) in (0, -6)


def test_pointer_and_workspace_checks():
    d = acc.make_desc(256, 256, 512, 16, io_dtype=acc.ACC_F32)
    assert _fwd(d, X=0) == -1 and _fwd(d, Y=0) == -1 and _fwd(d, Xs=0) == -1
    assert _fwd(d, X=0x1004) == -3 and _fwd(d, Xs=0x4008) == -3 and _fwd(d, ws=0x5002) == -3
    need = acc.acc_linear_workspace_bytes(d, False)
    assert need >= 256 * 16 * 4
    assert _fwd(d, ws_bytes=need - 1) == -5 and _fwd(d, ws=0) == -5
    assert _bwd(d, dY=0) == -1 and _bwd(d, Gr=0) == -1 and _bwd(d, Xs=0) == -1
    assert _bwd(d, dW=0x7004) == -3
    needb = acc.acc_linear_workspace_bytes(d, True)
    assert _bwd(d, ws_bytes=needb - 1) == -5
    # Xs may be NULL when no dense dW is requested: passes validation (then needs a device)
    assert _bwd(d, Xs=0, dW=0) in (0, -6)


def test_hooks_validate_arguments():
    assert acc._lib.acc_philox_dump_u32(0, 0, 16, 16, None, None) == -1
    assert acc._lib.acc_philox_dump_u32(0, 2, 16, 16, 0x1000, None) == -2
    assert acc._lib.acc_philox_dump_u32(0, 0, 0, 16, 0x1000, None) == -2
    assert acc._lib.acc_philox_dump_u32(0, 0, 16, 16, 0x1004, None) == -3
    d = acc.make_desc(16, 8, 8, 16)
    assert acc._lib.acc_sketch_dump(ctypes.byref(d), None, None) == -1
    assert acc._lib.acc_sketch_dump(None, 0x1000, None) == -1


def test_without_a_gfx950_device_calls_fail_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    d = acc.make_desc(256, 256, 512, 16, io_dtype=acc.ACC_F32)
    assert _fwd(d) == -6
    with pytest.raises(acc.AccError):
        acc._check(_fwd(d))


def test_workspace_query_is_positive_and_monotone_in_rank():
    a = acc.acc_linear_workspace_bytes(acc.make_desc(16384, 3072, 3072, 64), False)
    b = acc.acc_linear_workspace_bytes(acc.make_desc(16384, 3072, 3072, 256), False)
    assert 0 < a <= b


def test_weight_orientation_flag_changes_the_row_length_of_w():
    ok = dict(n=256, d_in=256, d_out=512, r=16)
    # default orientation: a row of W holds d_out elements; with the flag, d_in
    assert _fwd(acc.make_desc(**ok, ldw=256)) == -2
    assert _fwd(acc.make_desc(**ok, ldw=256, flags=acc.ACC_FLAG_W_OUT_IN)) in (0, -6)
    assert _fwd(acc.make_desc(**ok, ldw=248, flags=acc.ACC_FLAG_W_OUT_IN)) == -2
    assert _bwd(acc.make_desc(**ok, ldw=248, flags=acc.ACC_FLAG_W_OUT_IN)) == -2


def test_bias_gradient_refuses_bad_arguments():
    d = acc.make_desc(n=256, d_in=256, d_out=512, r=16)
    f = acc._lib.acc_linear_bias_grad
    need = acc.acc_linear_workspace_bytes(d, True)
    assert f(None, 0x1000, 0x2000, 0x3000, need, None) == -1
    assert f(ctypes.byref(d), None, 0x2000, 0x3000, need, None) == -1
    assert f(ctypes.byref(d), 0x1000, None, 0x3000, need, None) == -1
    assert f(ctypes.byref(d), 0x1004, 0x2000, 0x3000, need, None) == -3
    assert f(ctypes.byref(d), 0x1000, 0x2000, None, need, None) == -5
    assert f(ctypes.byref(d), 0x1000, 0x2000, 0x3000, need - 1, None) == -5
    assert f(ctypes.byref(acc.make_desc(n=0, d_in=256, d_out=512, r=16)), 0x1000, 0x2000, 0x3000, need, None) == -2


def test_rsvd_entry_points_validate_the_rank():
    f = acc._lib.acc_linear_fwd_rsvd
    args = (0x1000, 0x2000, 0x3000, 0x4000, 0x6000, 0x5000, 1 << 40, None)
    ok = dict(n=256, d_in=256, d_out=512)
    assert f(ctypes.byref(acc.make_desc(**ok, r=8)), *args) in (0, -6)
    for bad_r in (4, 12, 520, 1024):     # not a multiple of 8, above the limit of 512
        assert f(ctypes.byref(acc.make_desc(n=2048, d_in=2048, d_out=512, r=bad_r)), *args) == -2, bad_r
    for good_r in (72, 128, 256):        # ranks above 64 run the blocked factorisation
        assert f(ctypes.byref(acc.make_desc(**ok, r=good_r)), *args) in (0, -6), good_r
    assert f(ctypes.byref(acc.make_desc(**ok, r=512)), *args) == -2                          # n, d_in < rank
    assert f(ctypes.byref(acc.make_desc(n=16, d_in=256, d_out=512, r=32)), *args) == -2      # n < rank
    assert f(ctypes.byref(acc.make_desc(**ok, r=16, flags=acc.ACC_FLAG_SKIP_SKETCH)), *args) == -1
    d = acc.make_desc(**ok, r=16)
    need = acc.acc_rsvd_workspace_bytes(d, False)
    assert need > 0 and acc.acc_rsvd_workspace_bytes(d, True) > 0
    assert f(ctypes.byref(d), 0x1000, 0x2000, 0x3000, 0x4000, 0x6000, 0x5000, need - 1, None) == -5
    assert f(ctypes.byref(d), 0x1000, 0x2000, 0x3000, None, 0x6000, 0x5000, need, None) == -1
    assert acc.acc_rsvd_workspace_bytes(acc.make_desc(**ok, r=72), False) > need
    assert acc.acc_rsvd_workspace_bytes(acc.make_desc(n=2048, d_in=2048, d_out=512, r=520), False) == 0


def test_flag_constants_match_the_header():
    text = open(HEADER).read()
    declared = [(m.group(1), int(m.group(2)) << int(m.group(3) or 0))
                for m in re.finditer(r"\b(ACC_FLAG_[A-Z_0-9]+)\s*=\s*(\d+)u(?:\s*<<\s*(\d+))?", text)]
    assert len(declared) >= 7
    for name, value in declared:
        if hasattr(acc, name):
            assert getattr(acc, name) == value, name
    assert acc.ACC_FLAG_SKIP_SKETCH == 1 and acc.ACC_FLAG_ONE_LAUNCH == 2 and acc.ACC_FLAG_W_OUT_IN == 4
    assert acc.ACC_FLAG_DW_ACCUMULATE == 8
    shift = int(re.search(r"#define ACC_FLAG_RSVD_POWER_SHIFT (\d+)", text).group(1))
    assert acc.ACC_FLAG_RSVD_POWER_SHIFT == shift == 8
    assert re.search(r"ACC_F32 = 0, ACC_BF16 = 1", text) and (acc.ACC_F32, acc.ACC_BF16) == (0, 1)


def test_lowrank_optimizer_entry_points_validate_their_arguments():
    d = acc.make_desc(n=256, d_in=256, d_out=512, r=64)
    h = acc.make_hyper(1, 1e-3)
    step, proj = acc._lib.acc_lowrank_adamw_step, acc._lib.acc_lowrank_projector
    big = 1 << 40
    ptrs = (0x1000, 0x2000, 0x3000, 0x4000, 0x6000)   # left, Gr, M, V, W

    def call_step(desc=d, hyper=h, P=0x7000, k=16, ws=0x5000, ws_bytes=big, ptrs=ptrs):
        return step(ctypes.byref(desc) if desc is not None else None, ctypes.byref(hyper) if hyper is not None else None,
                    P, k, *ptrs, ws, ws_bytes, None)

    assert call_step() in (0, -6)
    assert call_step(P=None, k=0) in (0, -6)
    assert call_step(desc=None) == -1 and call_step(hyper=None) == -1
    for i in range(5):
        bad = list(ptrs); bad[i] = None
        assert call_step(ptrs=tuple(bad)) == -1, i
    assert call_step(P=0x7004) == -3 and call_step(ws=0x5008) == -3
    for k in (12, 264, -8):
        assert call_step(k=k) == -2, k
    assert call_step(P=None, k=12) in (0, -6)           # k is ignored without a projector
    need = acc.acc_lowrank_workspace_bytes(d, 16)
    assert need > 0 and acc.acc_lowrank_workspace_bytes(d, 0) == 512 * 64 * 2
    assert call_step(ws=None) == -5
    assert call_step(P=None, k=0, ws_bytes=512 * 64 * 2 - 1) == -5
    for kw in (dict(step=0), dict(beta1=1.0), dict(beta2=1.5), dict(eps=-1e-8), dict(lr=float("inf")),
               dict(weight_decay=float("nan")), dict(scale=float("inf"))):
        assert call_step(hyper=acc.make_hyper(**{**dict(step=1, lr=1e-3), **kw})) == -1, kw
    for flag in (acc.ACC_FLAG_SKIP_SKETCH, acc.ACC_FLAG_ONE_LAUNCH, acc.ACC_FLAG_DW_ACCUMULATE):
        assert call_step(desc=acc.make_desc(n=256, d_in=256, d_out=512, r=64, flags=flag)) == -1
    assert call_step(desc=acc.make_desc(n=256, d_in=256, d_out=512, r=64, flags=acc.ACC_FLAG_W_OUT_IN)) in (0, -6)

    def call_proj(k=16, left=0x1000, Gr=0x2000, P=0x7000, ws=0x5000, ws_bytes=big):
        return proj(ctypes.byref(d), k, left, Gr, P, ws, ws_bytes, None)

    assert call_proj() in (0, -6)
    assert call_proj(left=None) == -1 and call_proj(Gr=None) == -1 and call_proj(P=None) == -1
    for k in (0, 4, 72, 128):      # below 8, not a multiple of 8, above r = 64
        assert call_proj(k=k) == -2, k
    d512 = acc.make_desc(n=256, d_in=1024, d_out=1024, r=640)
    assert proj(ctypes.byref(d512), 128, 0x1000, 0x2000, 0x7000, 0x5000, big, None) in (0, -6)   # blocked factorisation
    assert proj(ctypes.byref(d512), 520, 0x1000, 0x2000, 0x7000, 0x5000, big, None) == -2        # above the limit of 512
    assert call_proj(ws_bytes=need - 1) == -5 and call_proj(P=0x7002) == -3
    assert ctypes.sizeof(acc.AccAdamwHyper) == 32


def test_hyperparameter_struct_matches_header():
    text = open(HEADER).read()
    body = re.search(r"typedef struct acc_adamw_hyper \{(.*?)\} acc_adamw_hyper;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for typ, names in re.findall(r"\b(float|int32_t)\s+([\w\s,]+);", body):
        fields += [(n.strip(), ctypes.c_float if typ == "float" else ctypes.c_int32) for n in names.split(",")]
    assert fields == list(acc.AccAdamwHyper._fields_)


def test_static_scratch_forward_validates_before_it_touches_a_device():
    f = acc._lib.acc_linear_fwd_static
    args = (0x1000, 0x2000, 0x3000, 0x4000, None)
    assert f(None, *args) == -1
    d = acc.make_desc(256, 256, 512, 16, io_dtype=acc.ACC_F32)
    assert f(ctypes.byref(d), 0, 0x2000, 0x3000, 0x4000, None) == -1
    assert f(ctypes.byref(d), 0x1004, 0x2000, 0x3000, 0x4000, None) == -3
    assert f(ctypes.byref(acc.make_desc(256, 256, 512, 20)), *args) == -2
    # partial tiles beyond the static array: refused, nothing launched
    big = acc.make_desc(65536, 4096, 4096, 512)
    assert acc.acc_linear_workspace_bytes(big, False) > acc.ACC_STATIC_SCRATCH_BYTES
    assert f(ctypes.byref(big), *args) == -5
    # with the sketch skipped no scratch is needed at all
    skip = acc.make_desc(65536, 4096, 4096, 512, flags=acc.ACC_FLAG_SKIP_SKETCH)
    assert f(ctypes.byref(skip), 0x1000, 0x2000, 0x3000, None, None) in (0, -6)
    header = open(HEADER).read()
    assert re.search(r"#define ACC_STATIC_SCRATCH_BYTES \(\(size_t\)32 << 20\)", header)
    assert acc.ACC_STATIC_SCRATCH_BYTES == 32 << 20


def test_factor_stride_and_the_dense_gradient_call_are_validated():
    ok = dict(n=256, d_in=256, d_out=512, r=16)
    for bad in (8, 20, 12, (1 << 24) + 8):          # smaller than r, not a multiple of 8, above the limit
        assert _fwd(acc.make_desc(**ok, ldf=bad)) == -2, bad
    assert _fwd(acc.make_desc(**ok, ldf=48)) in (0, -6)
    f = acc._lib.acc_linear_dw
    d = acc.make_desc(**ok, ldf=48)
    assert f(None, 0x1000, 0x2000, 0x3000, None) == -1
    assert f(ctypes.byref(d), 0, 0x2000, 0x3000, None) == -1
    assert f(ctypes.byref(d), 0x1000, 0x2000, 0, None) == -1
    assert f(ctypes.byref(d), 0x1000, 0x2008, 0x3000, None) == -3
    assert f(ctypes.byref(acc.make_desc(**ok, flags=acc.ACC_FLAG_SKIP_SKETCH)), 0x1000, 0x2000, 0x3000, None) == -1
    assert f(ctypes.byref(acc.make_desc(**ok, flags=acc.ACC_FLAG_DW_ACCUMULATE)), 0x1000, 0x2000, 0x3000, None) in (0, -6)
    # the RSVD and optimizer calls read dense factors only
    r = acc.make_desc(n=256, d_in=256, d_out=512, r=32, ldf=64)
    assert acc.acc_rsvd_workspace_bytes(r, False) == 0
    assert acc.acc_lowrank_workspace_bytes(r, 16) == 0


def test_mfma_probe_hook_validates_arguments():
    f = acc._lib.acc_probe_mfma
    fl = ctypes.c_double(0.0)
    big = 256 * 512 * 4
    assert f(0, 1, 0, 100, None, big, ctypes.byref(fl), None) == -1
    assert f(0, 1, 0, 100, 0x1000, big, None, None) == -1
    assert f(3, 1, 0, 100, 0x1000, big, ctypes.byref(fl), None) == -2
    assert f(0, 3, 0, 100, 0x1000, big, ctypes.byref(fl), None) == -2
    assert f(0, 1, 0, 0, 0x1000, big, ctypes.byref(fl), None) == -2
    assert f(0, 1, 0, 100, 0x1004, big, ctypes.byref(fl), None) == -3
    assert f(1, 2, 1, 100, 0x1000, 256 * 512 * 4 - 1, ctypes.byref(fl), None) == -5


def test_fp8_entry_points_validate_before_they_touch_a_device():
    fwd, bwd = acc._lib.acc_linear_fwd_fp8, acc._lib.acc_linear_bwd_fp8
    ws = 1 << 26
    ok = acc.make_desc(1000, 512, 640, 64)

    def f(d, X=0x1000, X8=0x2000, W8=0x3000, scale=1.0, Y=0x4000, Xs=0x5000, w=0x6000):
        return fwd(ctypes.byref(d), X, X8, W8, ctypes.c_float(scale), Y, Xs, w, ws, None)

    def b(d, dY=0x1000, dY8=0x2000, fmt=acc.ACC_FP8_E5M2, W8=0x3000, scale=1.0, Xs=0x4000, dX=0x5000, Gr=0x6000,
          dW=0x7000, w=0x8000):
        return bwd(ctypes.byref(d), dY, dY8, fmt, W8, ctypes.c_float(scale), Xs, dX, Gr, dW, w, ws, None)

    assert f(ok) in (0, -6) and b(ok) in (0, -6)
    assert fwd(None, 0x1000, 0x2000, 0x3000, ctypes.c_float(1.0), 0x4000, 0x5000, 0x6000, ws, None) == -1
    assert f(ok, X8=0) == -1 and f(ok, W8=0) == -1 and f(ok, Y=0) == -1 and f(ok, X=0) == -1 and f(ok, Xs=0) == -1
    assert f(ok, scale=float("nan")) == -1 and b(ok, scale=float("nan")) == -1
    assert f(ok, X8=0x2004) == -3 and b(ok, dY8=0x2008) == -3
    assert b(ok, dY8=0) == -1 and b(ok, fmt=2) == -4 and b(ok, Xs=0) == -1 and b(ok, Xs=0, dW=0) in (0, -6)
    # fp32 tensors beside the 8-bit operands are not supported
    assert f(acc.make_desc(1000, 512, 640, 64, io_dtype=acc.ACC_F32)) == -4
    # with the sketch skipped neither X nor Xs nor a workspace is needed
    skip = acc.make_desc(1000, 512, 640, 64, flags=acc.ACC_FLAG_SKIP_SKETCH)
    assert fwd(ctypes.byref(skip), None, 0x2000, 0x3000, ctypes.c_float(1.0), 0x4000, None, None, 0, None) in (0, -6)
    assert b(skip) == -1
    # contraction length: a multiple of 128, at least 384 (d_in forward, d_out backward); no slower fall-back
    assert f(acc.make_desc(1000, 448, 640, 64)) == -2 and f(acc.make_desc(1000, 256, 640, 64)) == -2
    assert b(acc.make_desc(1000, 512, 576, 64)) == -2 and b(acc.make_desc(1000, 512, 256, 64)) == -2
    assert f(acc.make_desc(1000, 512, 576, 64)) in (0, -6)     # forward only needs d_out % 16 (a 16-byte row of W8)
    assert f(acc.make_desc(1000, 512, 648, 64)) == -2
    # row strides of the 8-bit operands: multiples of 16 bytes
    assert f(acc.make_desc(1000, 512, 640, 64, ldx=520)) == -2 and f(acc.make_desc(1000, 512, 640, 64, ldx=528)) in (0, -6)
    # too small a workspace
    assert fwd(ctypes.byref(ok), 0x1000, 0x2000, 0x3000, ctypes.c_float(1.0), 0x4000, 0x5000, 0x6000, 16, None) == -5
