"""Seeded synthetic inputs for the butterfly + quantisation hot path.

This module only draws random numbers and casts them to storage dtypes.  It holds none of the
method's arithmetic (no rotations, no quantiser), so both the CPU oracle's tests and the HIP path's
tests/bench may import it without sharing any of the computation under test.

The five workloads mirror the shapes the paper calibrates on (hidden size 4096, 128 sequences of
2048 tokens; Experiments, "Hardware") and the outlier statistics it reports for un-rotated
activations (Appendix "Activation Kurtosis and Outlier Analysis": heavy tails, a few channels far
above 3 sigma).  They stand in for LLaMA-2 activations on WikiText-2, which are not available here.

Storage dtypes are named "f32", "f16", "bf16".  bf16 arrays are carried as numpy uint16 bit
patterns (numpy has no bfloat16); `to_f64` turns any storage array into exact float64 values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

ROOT_SEED = 9679

# ---------------------------------------------------------------------------------------------
# dtype plumbing (casts only)
# ---------------------------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even on the upper 16 bits); returns uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def cast_storage(a64: np.ndarray, dtype: str) -> np.ndarray:
    """Cast float64 draws to the storage dtype (fp16 saturates at +-65504 instead of inf)."""
    if dtype == "f32":
        return a64.astype(np.float32)
    if dtype == "f16":
        return np.clip(a64, -65504.0, 65504.0).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(a64.astype(np.float32))
    raise ValueError(dtype)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of every stored element."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a).astype(np.float64)


def to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(a)
    return np.asarray(a).astype(np.float32)


def storage_itemsize(dtype: str) -> int:
    return {"f32": 4, "f16": 2, "bf16": 2}[dtype]


def log2_exact(n: int) -> int:
    k = int(n).bit_length() - 1
    if n < 2 or (1 << k) != n:
        raise ValueError(f"n={n} is not a power of two >= 2")
    return k


# ---------------------------------------------------------------------------------------------
# draws
# ---------------------------------------------------------------------------------------------


def _streams(cfg: int, salt: int = 0):
    ss = np.random.SeedSequence([ROOT_SEED, int(cfg), int(salt)])
    return [np.random.default_rng(s) for s in ss.spawn(4)]  # x, theta, outlier channels, dy


def theta_uniform(rng: np.random.Generator, n: int, heads: int = 1) -> np.ndarray:
    """Angles U[-pi, pi) drawn in float64, stored float32, layout [heads][log2 n][n/2]."""
    k = log2_exact(n)
    t = rng.uniform(-math.pi, math.pi, size=(heads, k, n // 2))
    return t.astype(np.float32)


def student_t3(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_t(3.0, size=shape)


@dataclass
class Workload:
    """One synthetic workload: storage arrays plus the shape/quantiser parameters."""

    cfg: int
    name: str
    n: int
    heads: int
    rows: int
    dtype: str
    x: np.ndarray
    theta: np.ndarray
    bits: int = 4
    group: int = 0  # 0 => not quantised
    scale_dtype: str = "f32"
    dy: Optional[np.ndarray] = None
    outlier_channels: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    full_rows: int = 0  # the row count the workload has at full size

    @property
    def width(self) -> int:
        return self.n * self.heads


FULL_ROWS = {1: 1024, 2: 64, 3: 262144, 4: 8192, 5: 65536}


def make_workload(cfg: int, rows: Optional[int] = None, salt: int = 0) -> Workload:
    """Build workload `cfg` (1..5) on the host with `rows` rows (default: its full size, except
    3 and 5 whose default is a 2048-row sample of the same distribution)."""
    rx, rt, ro, rdy = _streams(cfg, salt)
    if cfg == 1:
        n, heads, dtype = 128, 1, "f32"
        T = FULL_ROWS[1] if rows is None else rows
        x = rx.standard_normal((T, n))
        ch = np.array([3, 77])
        x[:, ch] *= 50.0
        return Workload(1, "c1_n128_f32_int4_token", n, heads, T, dtype, cast_storage(x, dtype),
                        theta_uniform(rt, n), bits=4, group=n, scale_dtype="f32",
                        outlier_channels=ch, full_rows=FULL_ROWS[1])
    if cfg in (2, 3):
        n, heads, dtype = 4096, 1, "f16"
        if rows is None:
            T = FULL_ROWS[2] if cfg == 2 else 2048
        else:
            T = rows
        ch = np.sort(ro.choice(n, size=41, replace=False))
        x = student_t3(rx, (T, n))
        x[:, ch] *= 100.0
        bits = 4 if cfg == 2 else 2
        name = "c2_decode_n4096_f16_int4_g128" if cfg == 2 else "c3_prefill_n4096_f16_int2_g128"
        return Workload(cfg, name, n, heads, T, dtype, cast_storage(x, dtype), theta_uniform(rt, n),
                        bits=bits, group=128, scale_dtype="f16", outlier_channels=ch,
                        full_rows=FULL_ROWS[cfg])
    if cfg == 4:
        n, heads, dtype = 128, 32, "bf16"
        T = FULL_ROWS[4] if rows is None else rows
        x = rx.standard_normal((T, heads * n))
        ch = np.concatenate([h * n + np.sort(ro.choice(n, size=2, replace=False)) for h in range(heads)])
        x[:, ch] *= 30.0
        return Workload(4, "c4_heads32_n128_bf16_int4_head", n, heads, T, dtype, cast_storage(x, dtype),
                        theta_uniform(rt, n, heads), bits=4, group=n, scale_dtype="f32",
                        outlier_channels=ch, full_rows=FULL_ROWS[4])
    if cfg == 5:
        n, heads, dtype = 8192, 1, "bf16"
        T = 2048 if rows is None else rows
        x = student_t3(rx, (T, n))
        dy = rdy.standard_normal((T, n))
        return Workload(5, "c5_bwd_n8192_bf16", n, heads, T, dtype, cast_storage(x, dtype),
                        theta_uniform(rt, n), group=0, dy=cast_storage(dy, dtype),
                        full_rows=FULL_ROWS[5])
    raise ValueError(f"unknown workload {cfg}")


def small_case(n: int, rows: int, dtype: str, heads: int = 1, seed: int = 0, outliers: int = 2,
               with_dy: bool = False, dist: str = "t3"):
    """Generic seeded case for parity sweeps over shapes: returns (x, theta, dy-or-None)."""
    ss = np.random.SeedSequence([ROOT_SEED, 1000, n, rows, heads, seed])
    rx, rt, ro, rdy = [np.random.default_rng(s) for s in ss.spawn(4)]
    w = n * heads
    x = student_t3(rx, (rows, w)) if dist == "t3" else rx.standard_normal((rows, w))
    if outliers and w > outliers:
        ch = ro.choice(w, size=outliers, replace=False)
        x[:, ch] *= 40.0
    theta = theta_uniform(rt, n, heads)
    dy = cast_storage(rdy.standard_normal((rows, w)), dtype) if with_dy else None
    return cast_storage(x, dtype), theta, dy


# ---------------------------------------------------------------------------------------------
# full-size device-side generation (same recipe, torch's seeded device generator; plumbing only)
# ---------------------------------------------------------------------------------------------


def torch_dtype(dtype: str):
    import torch

    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]


def device_rows(cfg: int, rows: int, device="cuda:0", salt: int = 0, want_dy: bool = False):
    """Draw `rows` rows of workload `cfg` directly in device memory, in chunks, with the same
    distribution recipe as `make_workload`.  Returns (x, theta_host_f32, dy-or-None); x/dy are torch
    tensors in the storage dtype.  The outlier channels and theta come from the host streams so
    they equal those of `make_workload(cfg)`."""
    import torch

    ref = make_workload(cfg, rows=1, salt=salt)
    n, heads, dtype = ref.n, ref.heads, ref.dtype
    w = n * heads
    tdt = torch_dtype(dtype)
    g = torch.Generator(device=device)
    g.manual_seed(ROOT_SEED * 1000 + cfg * 10 + salt)
    x = torch.empty((rows, w), dtype=tdt, device=device)
    dy = torch.empty((rows, w), dtype=tdt, device=device) if want_dy else None
    scale = torch.ones(w, dtype=torch.float32, device=device)
    mult = {1: 50.0, 2: 100.0, 3: 100.0, 4: 30.0, 5: 1.0}[cfg]
    if ref.outlier_channels.size:
        scale[torch.as_tensor(ref.outlier_channels, device=device)] = mult
    heavy = cfg in (2, 3, 5)
    chunk = max(1, min(rows, (1 << 26) // w))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        z = torch.randn((r1 - r0, w), generator=g, device=device, dtype=torch.float32)
        if heavy:
            # Student-t(3) = N(0,1) / sqrt(chi2_3 / 3)
            c = torch.randn((3, r1 - r0, w), generator=g, device=device, dtype=torch.float32)
            z = z / torch.sqrt((c * c).sum(0) / 3.0)
            del c
        z = z * scale
        if dtype == "f16":
            z = z.clamp_(-65504.0, 65504.0)
        x[r0:r1] = z.to(tdt)
        if want_dy:
            dy[r0:r1] = torch.randn((r1 - r0, w), generator=g, device=device, dtype=torch.float32).to(tdt)
    return x, ref.theta, dy


def torch_to_storage(t, dtype: str) -> np.ndarray:
    """Copy a torch tensor in storage dtype to the numpy storage representation."""
    import torch

    t = t.detach().cpu().contiguous()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def storage_to_torch(a: np.ndarray, dtype: str, device="cpu"):
    import torch

    if dtype == "bf16":
        t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16).copy()).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(a).copy())
    return t.to(device)
