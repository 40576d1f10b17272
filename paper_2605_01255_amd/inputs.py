"""Seeded synthetic workloads for the compressed linear layer.

This module only *generates data* (random matrices with the shapes and value
structure of LLaMA-style linear layers) and converts between float32 and
bfloat16 bit patterns.  It holds none of the method's arithmetic (no sketch, no
Philox counter map, no matrix products of the layer itself) and is the only
code shared by the CPU oracle's tests and the GPU path's tests/benchmark, so
both sides always see the same bits.

The paper trains LLaMA3-3B / Qwen3-4B on public corpora (Experimental Setup);
those activations are not available here, so the recipes below stand in for
them: Gaussian token rows with a few large "outlier" feature channels (a known
property of LLM activations), small Gaussian weights and small Gaussian
incoming gradients.  Nothing from any dataset is reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

DATA_SEED = 12345


# ----------------------------------------------------------------------------
# bfloat16 bit helpers (data formatting only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = a.view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# 8-bit floating-point bit helpers (OCP fp8 e4m3 and e5m2; data formatting only)
# ----------------------------------------------------------------------------
def _fp8_table(fmt: str) -> np.ndarray:
    """float32 value of every bit pattern 0x00 .. 0x7F of the format (NaN / inf patterns as nan / inf)."""
    ebits, mbits, bias = (4, 3, 7) if fmt == "e4m3" else (5, 2, 15)
    out = np.empty(128, dtype=np.float64)
    for b in range(128):
        e, m = b >> mbits, b & ((1 << mbits) - 1)
        if e == 0:
            out[b] = m * 2.0 ** (1 - bias - mbits)
        else:
            out[b] = (1 + m * 2.0 ** -mbits) * 2.0 ** (e - bias)
    if fmt == "e4m3":
        out[0x7F] = np.nan                      # the only NaN; no infinities, largest finite value 448
    else:
        out[0x7C] = np.inf
        out[0x7D:] = np.nan                     # largest finite value 57344
    return out


def fp8_max(fmt: str) -> float:
    return 448.0 if fmt == "e4m3" else 57344.0


def f32_to_fp8_bits(a: np.ndarray, fmt: str = "e4m3") -> np.ndarray:
    """float32 -> 8-bit float bit patterns (uint8): round to nearest, ties to the even pattern, saturating at the
    largest finite value (the cast an fp8 training recipe applies after scaling)."""
    tab = _fp8_table(fmt)
    last = 0x7E if fmt == "e4m3" else 0x7B      # largest finite pattern
    pos = tab[:last + 1]
    a = np.ascontiguousarray(a, dtype=np.float32)
    flat = a.reshape(-1)
    out = np.empty(flat.shape, dtype=np.uint8)
    step = 1 << 22                              # bounded temporaries for operands of a gigabyte
    for s0 in range(0, flat.size, step):
        v = flat[s0:s0 + step]
        mag = np.minimum(np.abs(v).astype(np.float64), pos[-1])
        hi = np.clip(np.searchsorted(pos, mag, side="left"), 0, last)
        lo = np.maximum(hi - 1, 0)
        d_hi, d_lo = pos[hi] - mag, mag - pos[lo]
        pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ((hi & 1) == 0))
        bits = np.where(pick_hi, hi, lo).astype(np.uint8)
        out[s0:s0 + step] = bits | (np.signbit(v).astype(np.uint8) << np.uint8(7))
    return out.reshape(a.shape)


def fp8_bits_to_f64(bits: np.ndarray, fmt: str = "e4m3") -> np.ndarray:
    """8-bit float bit patterns (uint8) -> float64 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    val = _fp8_table(fmt)[bits & np.uint8(0x7F)]
    return np.where(bits >> np.uint8(7), -val, val)


def as_f64(a: np.ndarray) -> np.ndarray:
    """Widen a stored array (float32 values or uint16 bf16 bits) to float64, exactly."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Format a float32 array the way the device receives it: 'f32' -> float32, 'bf16' -> uint16 bits."""
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# workload description
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Linear:
    """One compressed linear layer instance."""
    name: str
    n: int
    d_in: int
    d_out: int
    r: int
    dtype: str = "bf16"            # storage type of X, W, dY, Y, dX
    x_kind: str = "outlier"        # "plain" | "outlier" | "swiglu" | "lowrank"
    n_outliers: int = 8
    seed: int = 0                  # sketch seed handed to the layer
    data_seed: int = DATA_SEED

    def flops(self, with_dw: bool = False) -> int:
        """Algorithmic flops of forward + backward (S generation counts zero)."""
        f = 2 * self.n * self.d_in * self.d_out + 2 * self.n * self.d_in * self.r
        b = 2 * self.n * self.d_in * self.d_out + 2 * self.n * self.r * self.d_out
        d = 2 * self.d_in * self.r * self.d_out if with_dw else 0
        return f + b + d

    def activation_bytes(self, factor_bytes: int = 2):
        """(bytes of X kept by a dense layer, bytes kept here: Xs + 8-byte seed)."""
        esize = 2 if self.dtype == "bf16" else 4
        return self.n * self.d_in * esize, self.d_in * self.r * factor_bytes + 8


def outlier_channels(d_in: int, k: int):
    """Channel indices that carry the x20 outliers: c_j = j * (d_in // k) + 5 (wrapped for tiny d_in)."""
    return sorted({(j * (d_in // k) + 5) % d_in for j in range(k)})


def _rng(data_seed: int, tag: int) -> np.random.Generator:
    return np.random.default_rng([data_seed, tag])


def _normal(rng, shape, scale=1.0, chunk_rows=8192):
    out = np.empty(shape, dtype=np.float32)
    rows = shape[0]
    for s in range(0, rows, chunk_rows):
        e = min(rows, s + chunk_rows)
        out[s:e] = rng.standard_normal((e - s,) + tuple(shape[1:]), dtype=np.float32)
    if scale != 1.0:
        out *= np.float32(scale)
    return out


def make_x(lin: Linear) -> np.ndarray:
    """Input activation X [n, d_in] as float32 (before storage rounding)."""
    rng = _rng(lin.data_seed, 1)
    if lin.x_kind == "plain":
        return _normal(rng, (lin.n, lin.d_in))
    if lin.x_kind == "outlier":
        x = _normal(rng, (lin.n, lin.d_in))
        x[:, outlier_channels(lin.d_in, lin.n_outliers)] *= np.float32(20.0)
        return x
    if lin.x_kind == "swiglu":
        # Input of an MLP down-projection: SiLU(gate) * up of generated gate/up values.
        # gate/up stand for outputs of 3072->8192 projections of the "outlier" X with
        # W ~ N(0, 0.02^2): their per-entry standard deviation is about 1.6.
        x = np.empty((lin.n, lin.d_in), dtype=np.float32)
        for s in range(0, lin.n, 4096):
            e = min(lin.n, s + 4096)
            gate = rng.standard_normal((e - s, lin.d_in), dtype=np.float32) * np.float32(1.6)
            up = rng.standard_normal((e - s, lin.d_in), dtype=np.float32) * np.float32(1.6)
            x[s:e] = gate / (1.0 + np.exp(-gate)) * up
        return x
    if lin.x_kind == "lowrank":
        # rank-64 component + N(0, 0.1^2) noise, then outlier channels.
        k = 64
        b = rng.standard_normal((k, lin.d_in), dtype=np.float32) * np.float32(1.0 / np.sqrt(k))
        x = np.empty((lin.n, lin.d_in), dtype=np.float32)
        for s in range(0, lin.n, 8192):
            e = min(lin.n, s + 8192)
            a = rng.standard_normal((e - s, k), dtype=np.float32)
            x[s:e] = a @ b + np.float32(0.1) * rng.standard_normal((e - s, lin.d_in), dtype=np.float32)
        x[:, outlier_channels(lin.d_in, lin.n_outliers)] *= np.float32(20.0)
        return x
    raise ValueError(lin.x_kind)


def make_w(lin: Linear) -> np.ndarray:
    """Weight W [d_in, d_out] ~ N(0, 0.02^2) as float32."""
    return _normal(_rng(lin.data_seed, 2), (lin.d_in, lin.d_out), 0.02)


def make_dy(lin: Linear) -> np.ndarray:
    """Incoming gradient dY [n, d_out] ~ N(0, 0.01^2) as float32."""
    return _normal(_rng(lin.data_seed, 3), (lin.n, lin.d_out), 0.01)


def make_gradient_factors(lin: Linear, steps: int, factor_dtype: str = None):
    """Inputs of the optimizer step on the factored gradient, at the magnitudes the layer's own factors have:
    one left factor [d_in, r] ~ N(0, n / r) (a sketch of unit-variance activations) and, per step t, a small
    factor [r, d_out] ~ N(0, (0.01 * 0.7^t)^2 * n / r) (gradients that shrink as training goes on).  Stored
    format of `factor_dtype` (default: the layer's dtype).  Returns (left, [Gr_1, ..., Gr_steps])."""
    dt = factor_dtype or lin.dtype
    s = float(np.sqrt(lin.n / lin.r))
    left = store(_normal(_rng(lin.data_seed, 4), (lin.d_in, lin.r), s), dt)
    grs = [store(_normal(_rng(lin.data_seed, 100 + t), (lin.r, lin.d_out), 0.01 * 0.7 ** t * s), dt)
           for t in range(1, steps + 1)]
    return left, grs


def make(lin: Linear):
    """Stored-format inputs: dict with X, W, dY (float32 arrays or uint16 bf16 bit arrays)."""
    return {"X": store(make_x(lin), lin.dtype),
            "W": store(make_w(lin), lin.dtype),
            "dY": store(make_dy(lin), lin.dtype)}


# ----------------------------------------------------------------------------
# the benchmark configurations
# ----------------------------------------------------------------------------
def config(name: str):
    """List of Linear instances of a named configuration.

    c1        tiny fp32 layer (n=256, 256->512, r=16)
    c2        LLaMA-3B-shaped attention projection (n=16384, 3072->3072, r=256), bf16
    c3_r{R}   LLaMA-3B-shaped MLP: gate, up 3072->8192 and down 8192->3072, rank R
    c4        LLaMA-3B-shaped decoder layer: q,o,k,v,gate,up,down, r=256, one seed
    c5        LLaMA-8B-shaped layer, n=65536, r=512, low-rank-plus-noise X
    """
    if name == "c1":
        return [Linear("c1", 256, 256, 512, 16, dtype="f32", x_kind="plain")]
    if name == "c2":
        return [Linear("c2.attn_proj", 16384, 3072, 3072, 256)]
    if name.startswith("c3"):
        r = int(name.split("_r")[1]) if "_r" in name else 256
        return [Linear("c3.gate", 16384, 3072, 8192, r),
                Linear("c3.up", 16384, 3072, 8192, r, data_seed=DATA_SEED + 1),
                Linear("c3.down", 16384, 8192, 3072, r, x_kind="swiglu")]
    if name == "c4":
        n, h, kv, inter, r = 16384, 3072, 1024, 8192, 256
        return [Linear("c4.q", n, h, h, r), Linear("c4.k", n, h, kv, r),
                Linear("c4.v", n, h, kv, r), Linear("c4.o", n, h, h, r, data_seed=DATA_SEED + 2),
                Linear("c4.gate", n, h, inter, r, data_seed=DATA_SEED + 3),
                Linear("c4.up", n, h, inter, r, data_seed=DATA_SEED + 3),
                Linear("c4.down", n, inter, h, r, x_kind="swiglu")]
    if name == "c5":
        n, h, kv, inter, r = 65536, 4096, 1024, 14336, 512
        kw = dict(x_kind="lowrank", n_outliers=16)
        return [Linear("c5.q", n, h, h, r, **kw), Linear("c5.k", n, h, kv, r, **kw),
                Linear("c5.v", n, h, kv, r, **kw), Linear("c5.o", n, h, h, r, data_seed=DATA_SEED + 2, **kw),
                Linear("c5.gate", n, h, inter, r, data_seed=DATA_SEED + 3, **kw),
                Linear("c5.up", n, h, inter, r, data_seed=DATA_SEED + 3, **kw),
                Linear("c5.down", n, inter, h, r, x_kind="swiglu")]
    raise ValueError(name)
