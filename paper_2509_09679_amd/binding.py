"""ctypes binding of libbq.so: the same entry points as include/bq.h, taking torch tensors.

Argument marshalling only — every step of the path runs in the library's HIP kernels.  torch is used
for device memory and the current stream, nothing else.  There is no CPU or eager fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbq.so")

BQ_OK = 0
BQ_F32, BQ_F16, BQ_BF16 = 0, 1, 2
STATUS_NAMES = {0: "BQ_OK", 1: "BQ_ERR_NULL", 2: "BQ_ERR_SHAPE", 3: "BQ_ERR_DTYPE", 4: "BQ_ERR_ALIGN",
                5: "BQ_ERR_WORKSPACE", 6: "BQ_ERR_UNSUPPORTED", 7: "BQ_ERR_HIP"}
DTYPE_CODES = {"f32": BQ_F32, "f16": BQ_F16, "bf16": BQ_BF16}

EXPORTS = ["bq_plan_bytes", "bq_plan_build", "bq_butterfly_fwd", "bq_butterfly_inv", "bq_butterfly_fwd_quant",
           "bq_butterfly_fwd_fakequant", "bq_hadamard_fwd", "bq_cayley_build", "bq_kron_fwd", "bq_kron_inv",
           "bq_butterfly_bwd_workspace_bytes", "bq_butterfly_bwd", "bq_butterfly_bwd_static",
           "bq_butterfly_bwd_static_max_bytes", "bq_probe_copy", "bq_probe_read", "bq_probe_read_sink_bytes",
           "bq_probe_fma", "bq_probe_fma_out_floats",
           "bq_status_string", "bq_last_error",
           "bq_version"]


class bq_rows(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("n", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("ld_x", ctypes.c_int64), ("ld_y", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class bq_quant(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int32), ("group", ctypes.c_int32), ("scale_dtype", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class BqError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


_LIB = None


def lib() -> ctypes.CDLL:
    """Load libbq.so (built in-tree by paper_2509_09679_amd.build); fails loudly if it is absent."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2509_09679_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.bq_plan_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
        L.bq_plan_bytes.restype = sz
        L.bq_plan_build.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, sz, vp]
        L.bq_plan_build.restype = ctypes.c_int
        for name in ("bq_butterfly_fwd", "bq_butterfly_inv"):
            f = getattr(L, name)
            f.argtypes = [vp, vp, vp, ctypes.POINTER(bq_rows), vp]
            f.restype = ctypes.c_int
        L.bq_hadamard_fwd.argtypes = [vp, vp, ctypes.POINTER(bq_rows), vp]
        L.bq_hadamard_fwd.restype = ctypes.c_int
        L.bq_butterfly_fwd_quant.argtypes = [vp, vp, vp, vp, ctypes.POINTER(bq_quant), ctypes.POINTER(bq_rows), vp]
        L.bq_butterfly_fwd_fakequant.argtypes = [vp, vp, vp, vp, ctypes.POINTER(bq_quant), ctypes.POINTER(bq_rows), vp]
        L.bq_butterfly_fwd_fakequant.restype = ctypes.c_int
        L.bq_cayley_build.argtypes = [vp, ctypes.c_int32, vp, vp]
        L.bq_cayley_build.restype = ctypes.c_int
        for f in (L.bq_kron_fwd, L.bq_kron_inv):
            f.argtypes = [vp, vp, vp, ctypes.c_int32, vp, ctypes.POINTER(bq_rows), vp]
            f.restype = ctypes.c_int
        L.bq_butterfly_fwd_quant.restype = ctypes.c_int
        L.bq_butterfly_bwd_workspace_bytes.argtypes = [ctypes.POINTER(bq_rows)]
        L.bq_butterfly_bwd_workspace_bytes.restype = sz
        L.bq_butterfly_bwd.argtypes = [vp, vp, vp, vp, vp, vp, sz, ctypes.POINTER(bq_rows), vp]
        L.bq_butterfly_bwd.restype = ctypes.c_int
        L.bq_butterfly_bwd_static.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(bq_rows), vp]
        L.bq_butterfly_bwd_static.restype = ctypes.c_int
        L.bq_butterfly_bwd_static_max_bytes.argtypes = []
        L.bq_butterfly_bwd_static_max_bytes.restype = sz
        L.bq_probe_copy.argtypes = [vp, vp, sz, vp]
        L.bq_probe_copy.restype = ctypes.c_int
        L.bq_probe_read.argtypes = [vp, sz, vp, vp]
        L.bq_probe_read.restype = ctypes.c_int
        L.bq_probe_read_sink_bytes.argtypes = []
        L.bq_probe_read_sink_bytes.restype = sz
        L.bq_probe_fma.argtypes = [vp, ctypes.c_int32, vp]
        L.bq_probe_fma.restype = ctypes.c_int64
        L.bq_probe_fma_out_floats.argtypes = []
        L.bq_probe_fma_out_floats.restype = sz
        L.bq_status_string.argtypes = [ctypes.c_int]
        L.bq_status_string.restype = ctypes.c_char_p
        L.bq_last_error.restype = ctypes.c_char_p
        L.bq_version.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _check(status: int):
    if status != BQ_OK:
        raise BqError(status, lib().bq_last_error().decode())


def _dtype_code(t) -> int:
    import torch

    return {torch.float32: BQ_F32, torch.float16: BQ_F16, torch.bfloat16: BQ_BF16}[t.dtype]


def _stream_ptr(stream=None) -> int:
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def make_rows(x, n: int, heads: int, out=None) -> bq_rows:
    """Descriptor for 2-D row tensors (last dimension contiguous)."""
    assert x.dim() == 2 and (x.shape[0] == 0 or x.stride(1) == 1)
    r = bq_rows()
    r.rows, r.n, r.heads = x.shape[0], n, heads
    r.ld_x = x.stride(0) if x.shape[0] > 1 else n * heads
    o = x if out is None else out
    r.ld_y = o.stride(0) if o.shape[0] > 1 else n * heads
    r.dtype = _dtype_code(x)
    return r


def make_kron_rows(x, d2: int) -> bq_rows:
    """Descriptor for bq_kron_fwd / bq_kron_inv: dense rows of d1 * d2 elements, butterfly size d2."""
    assert x.dim() == 2 and x.is_contiguous() and x.shape[1] % d2 == 0
    r = bq_rows()
    r.rows, r.n, r.heads = x.shape[0], d2, 1
    r.ld_x = r.ld_y = x.shape[1]
    r.dtype = _dtype_code(x)
    return r


# --- entry points, same names as the C ABI -----------------------------------------------------

def bq_plan_bytes(n: int, heads: int = 1) -> int:
    return int(lib().bq_plan_bytes(n, heads))


def bq_plan_build(theta, n: int, heads: int, plan, stream=None) -> None:
    """theta: float32 device tensor [heads, log2 n, n/2]; plan: uint8 device tensor of bq_plan_bytes."""
    _check(lib().bq_plan_build(_ptr(theta), n, heads, _ptr(plan), plan.numel() * plan.element_size(),
                               _stream_ptr(stream)))


def bq_butterfly_fwd(x, y, plan, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_butterfly_fwd(_ptr(x), _ptr(y), _ptr(plan), ctypes.byref(rows), _stream_ptr(stream)))


def bq_butterfly_inv(y, x, plan, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_butterfly_inv(_ptr(y), _ptr(x), _ptr(plan), ctypes.byref(rows), _stream_ptr(stream)))


def bq_hadamard_fwd(x, y, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_hadamard_fwd(_ptr(x), _ptr(y), ctypes.byref(rows), _stream_ptr(stream)))


def bq_butterfly_fwd_quant(x, plan, codes, scales, quant: bq_quant, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_butterfly_fwd_quant(_ptr(x), _ptr(plan), _ptr(codes), _ptr(scales), ctypes.byref(quant),
                                        ctypes.byref(rows), _stream_ptr(stream)))


def bq_butterfly_fwd_fakequant(x, plan, yq, hist, quant: bq_quant, rows: bq_rows, stream=None) -> None:
    """yq (rows' dtype, or None) and hist (uint64/int64 tensor of 2^bits counters, or None)."""
    _check(lib().bq_butterfly_fwd_fakequant(_ptr(x), _ptr(plan), _ptr(yq), _ptr(hist), ctypes.byref(quant),
                                            ctypes.byref(rows), _stream_ptr(stream)))


def bq_cayley_build(params, d1: int, q1, stream=None) -> None:
    _check(lib().bq_cayley_build(_ptr(params), d1, _ptr(q1), _stream_ptr(stream)))


def bq_kron_fwd(x, y, q1, d1: int, plan, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_kron_fwd(_ptr(x), _ptr(y), _ptr(q1), d1, _ptr(plan), ctypes.byref(rows), _stream_ptr(stream)))


def bq_kron_inv(y, x, q1, d1: int, plan, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_kron_inv(_ptr(y), _ptr(x), _ptr(q1), d1, _ptr(plan), ctypes.byref(rows), _stream_ptr(stream)))


def bq_butterfly_bwd_workspace_bytes(rows: bq_rows) -> int:
    return int(lib().bq_butterfly_bwd_workspace_bytes(ctypes.byref(rows)))


def bq_butterfly_bwd(x, dy, plan, dx, dtheta, workspace, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_butterfly_bwd(_ptr(x), _ptr(dy), _ptr(plan), _ptr(dx), _ptr(dtheta), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), ctypes.byref(rows),
                                  _stream_ptr(stream)))


def bq_butterfly_bwd_static(x, dy, plan, dx, dtheta, rows: bq_rows, stream=None) -> None:
    _check(lib().bq_butterfly_bwd_static(_ptr(x), _ptr(dy), _ptr(plan), _ptr(dx), _ptr(dtheta), ctypes.byref(rows),
                                         _stream_ptr(stream)))


def bq_butterfly_bwd_static_max_bytes() -> int:
    return int(lib().bq_butterfly_bwd_static_max_bytes())


def bq_probe_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(lib().bq_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream_ptr(stream)))


def bq_probe_read_sink_bytes() -> int:
    return int(lib().bq_probe_read_sink_bytes())


def bq_probe_read(src, nbytes: int, sink, stream=None) -> None:
    _check(lib().bq_probe_read(_ptr(src), nbytes, _ptr(sink), _stream_ptr(stream)))


def bq_probe_fma_out_floats() -> int:
    return int(lib().bq_probe_fma_out_floats())


def bq_probe_fma(out, iters: int, stream=None) -> int:
    """Launches the FMA loop; returns the number of lane-FMAs of the launch."""
    n = int(lib().bq_probe_fma(_ptr(out), iters, _stream_ptr(stream)))
    if n < 0:
        raise BqError(7, "bq_probe_fma failed")
    return n


def bq_version() -> int:
    return int(lib().bq_version())


# --- small conveniences that only allocate (no arithmetic) -------------------------------------

def alloc_plan(theta, n: int, heads: int = 1, stream=None):
    """Allocate a plan buffer with torch and fill it from `theta` (float32 device tensor)."""
    import torch

    nbytes = bq_plan_bytes(n, heads)
    if nbytes == 0:
        raise BqError(2, f"invalid plan shape n={n} heads={heads}")
    plan = torch.empty(nbytes, dtype=torch.uint8, device=theta.device)
    bq_plan_build(theta, n, heads, plan, stream)
    return plan


def alloc_quant_outputs(rows: int, n: int, heads: int, bits: int, group: int, scale_dtype: str, device):
    import torch

    codes = torch.empty((rows, n * heads * bits // 8), dtype=torch.uint8, device=device)
    sd = torch.float16 if scale_dtype == "f16" else torch.float32
    scales = torch.empty((rows, n * heads // group), dtype=sd, device=device)
    return codes, scales


def make_quant(bits: int, group: int, scale_dtype: str) -> bq_quant:
    q = bq_quant()
    q.bits, q.group, q.scale_dtype = bits, group, DTYPE_CODES[scale_dtype]
    return q
