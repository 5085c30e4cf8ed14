"""The C-ABI library loads, exports every symbol include/bq.h declares, and rejects bad arguments
with the documented status before anything is launched (no GPU needed: validation precedes any
HIP call, and pointers are never dereferenced on the host)."""
import ctypes
import os
import re

import pytest

from paper_2509_09679_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # never dereferenced: every case below fails validation or has rows == 0


def _header_functions():
    text = open(os.path.join(ROOT, "include", "bq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bq_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _header_functions()
    assert {"bq_butterfly_fwd", "bq_butterfly_inv", "bq_butterfly_fwd_quant", "bq_butterfly_bwd",
            "bq_plan_build", "bq_plan_bytes", "bq_butterfly_bwd_workspace_bytes"} <= set(names)
    L = B.lib()
    for name in names:
        assert hasattr(L, name), name
    assert sorted(B.EXPORTS) == names


def test_binding_has_same_names_as_header():
    for name in _header_functions():
        if name in ("bq_status_string", "bq_last_error"):
            continue
        assert callable(getattr(B, name)), name


def _rows(rows=4, n=128, heads=1, dtype=B.BQ_F32, ld=None):
    r = B.bq_rows()
    r.rows, r.n, r.heads, r.dtype = rows, n, heads, dtype
    r.ld_x = r.ld_y = n * heads if ld is None else ld
    return r


def _fwd(r, x=FAKE, y=FAKE, plan=FAKE):
    return B.lib().bq_butterfly_fwd(x, y, plan, ctypes.byref(r), None)


def test_struct_sizes_match_header():
    assert ctypes.sizeof(B.bq_rows) == 40
    assert ctypes.sizeof(B.bq_quant) == 16


def test_plan_bytes():
    assert B.bq_plan_bytes(4096, 1) > 24576 * 8
    assert B.bq_plan_bytes(4096, 1) % 256 == 0
    for bad in [(3, 1), (0, 1), (1, 1), (32768, 1), (128, 0), (-4, 1)]:
        assert B.bq_plan_bytes(*bad) == 0


@pytest.mark.parametrize("n", [0, 1, 3, 6, 100, 32768, -8])
def test_rejects_bad_n(n):
    assert _fwd(_rows(n=n)) == 2
    assert b"power of two" in B.lib().bq_last_error()


def test_rejects_other_bad_shapes_and_types():
    assert _fwd(_rows(heads=0)) == 2
    assert _fwd(_rows(rows=-1)) == 2
    assert _fwd(_rows(ld=64)) == 2
    assert _fwd(_rows(dtype=7)) == 3
    assert _fwd(_rows(), x=None) == 1
    assert _fwd(_rows(), plan=None) == 1
    assert B.lib().bq_butterfly_fwd(FAKE, FAKE, FAKE, None, None) == 1
    assert _fwd(_rows(), plan=FAKE + 16) == 4
    assert _fwd(_rows(dtype=B.BQ_F32), x=FAKE + 2) == 4
    assert B.lib().bq_butterfly_inv(FAKE, FAKE, FAKE, ctypes.byref(_rows(n=12)), None) == 2


def test_rejects_batches_beyond_the_documented_limits():
    assert _fwd(_rows(rows=(1 << 33) + 1, n=128)) == 2             # rows * H * n > 2^40
    assert _fwd(_rows(n=16384, heads=2048)) == 2                   # H * n > 2^24
    assert _fwd(_rows(rows=1 << 20, n=128, ld=(1 << 24) + 128)) == 2  # rows * ld > 2^44
    assert b"leading dimension" in B.lib().bq_last_error()


def test_zero_rows_is_ok_without_launch():
    assert _fwd(_rows(rows=0)) == 0
    assert B.lib().bq_last_error() == b""


def test_quant_validation():
    L = B.lib()

    def call(q, r=None, codes=FAKE, scales=FAKE):
        r = _rows(rows=0) if r is None else r
        return L.bq_butterfly_fwd_quant(FAKE, FAKE, codes, scales, ctypes.byref(q) if q is not None else None,
                                        ctypes.byref(r), None)

    assert call(B.make_quant(4, 128, "f16")) == 0
    assert call(B.make_quant(2, 8, "f32")) == 0
    assert call(None) == 1
    assert call(B.make_quant(3, 128, "f16")) == 6
    assert call(B.make_quant(8, 128, "f16")) == 6
    assert call(B.make_quant(4, 96, "f16")) == 2
    assert call(B.make_quant(4, 4, "f16")) == 2
    assert call(B.make_quant(4, 256, "f16")) == 2  # group > n
    q = B.make_quant(4, 128, "f16")
    q.scale_dtype = B.BQ_BF16
    assert call(q) == 3
    assert call(B.make_quant(4, 128, "f16"), r=_rows(rows=3), codes=None) == 1
    assert call(B.make_quant(4, 128, "f32"), scales=FAKE + 2) == 4


def test_bwd_validation_and_workspace_query():
    L = B.lib()
    r = _rows(rows=64, n=1024, dtype=B.BQ_BF16)
    need = B.bq_butterfly_bwd_workspace_bytes(r)
    assert need > 0 and need % 256 == 0
    assert B.bq_butterfly_bwd_workspace_bytes(_rows(n=24)) == 0

    def call(ws=FAKE, ws_bytes=need, dx=FAKE, dth=FAKE, rr=r):
        return L.bq_butterfly_bwd(FAKE, FAKE, FAKE, dx, dth, ws, ws_bytes, ctypes.byref(rr), None)

    assert call(ws_bytes=need - 1) == 5
    assert b"needed" in L.bq_last_error()
    assert call(ws=None) == 1
    assert call(ws=FAKE + 64) == 4
    assert call(dx=None, dth=None) == 1
    assert call(rr=_rows(n=7)) == 2


def test_workspace_query_over_many_shapes():
    # host arithmetic only: every valid shape gets a size (a positive multiple of 256), whichever kernel family
    # the shape belongs to
    for n in (2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384):
        for heads in (1, 2, 3, 5, 7, 12, 24, 40, 64, 86, 513):
            for rows in (0, 1, 7, 1000, 300000):
                for dtype in (B.BQ_F32, B.BQ_F16):
                    need = B.bq_butterfly_bwd_workspace_bytes(_rows(rows=rows, n=n, heads=heads, dtype=dtype))
                    assert need % 256 == 0, (n, heads, rows)
                    valid = n * heads <= 1 << 24 and rows * n * heads <= 1 << 40  # the documented limits
                    assert (need > 0) == valid, (n, heads, rows)


def test_plan_build_validation():
    L = B.lib()
    need = B.bq_plan_bytes(256, 2)
    assert L.bq_plan_build(FAKE, 256, 2, FAKE, need - 1, None) == 5
    assert L.bq_plan_build(None, 256, 2, FAKE, need, None) == 1
    assert L.bq_plan_build(FAKE, 255, 2, FAKE, need, None) == 2
    assert L.bq_plan_build(FAKE, 256, 2, FAKE + 8, need, None) == 4


def test_status_strings():
    L = B.lib()
    for code, name in B.STATUS_NAMES.items():
        assert L.bq_status_string(code).decode() == name
    assert B.bq_version() >= 100


def test_fakequant_validation():
    L = B.lib()

    def call(q, r=None, yq=FAKE, hist=FAKE, x=FAKE, plan=FAKE):
        r = _rows(rows=5) if r is None else r
        return L.bq_butterfly_fwd_fakequant(x, plan, yq, hist, ctypes.byref(q) if q is not None else None,
                                            ctypes.byref(r), None)

    q = B.make_quant(4, 128, "f16")
    assert call(None) == 1
    assert call(q, yq=None, hist=None) == 1
    assert b"both NULL" in L.bq_last_error()
    assert call(q, x=None) == 1
    assert call(q, plan=None) == 1
    assert call(B.make_quant(3, 128, "f16")) == 6
    assert call(B.make_quant(4, 48, "f16")) == 2
    assert call(B.make_quant(4, 256, "f16")) == 2            # group > n
    assert call(q, hist=FAKE + 4) == 4                        # counters are 64-bit
    assert call(q, r=_rows(rows=5, dtype=B.BQ_F32), yq=FAKE + 2) == 4
    assert call(q, r=_rows(rows=-2)) == 2
    assert call(q, r=_rows(rows=0), hist=None) == 0           # empty batch, nothing to clear: no launch


def test_cayley_and_kron_validation():
    L = B.lib()
    assert L.bq_cayley_build(FAKE, 1, FAKE, None) == 2
    assert L.bq_cayley_build(FAKE, 65, FAKE, None) == 2
    assert L.bq_cayley_build(None, 40, FAKE, None) == 1
    assert L.bq_cayley_build(FAKE, 40, None, None) == 1
    assert L.bq_cayley_build(FAKE + 2, 40, FAKE, None) == 4

    def call(fn, d1=40, r=None, x=FAKE, y=FAKE, q1=FAKE, plan=FAKE):
        r = _rows(rows=3, n=128, ld=40 * 128) if r is None else r
        return fn(x, y, q1, d1, plan, ctypes.byref(r), None)

    for fn in (L.bq_kron_fwd, L.bq_kron_inv):
        assert call(fn, d1=1) == 2
        assert call(fn, d1=65) == 2
        assert call(fn, r=_rows(rows=3, n=128, heads=2, ld=40 * 128)) == 2      # the butterfly factor is shared
        assert call(fn, r=_rows(rows=3, n=128, ld=40 * 128 + 8)) == 6            # rows must be dense
        assert b"dense" in L.bq_last_error()
        assert call(fn, r=_rows(rows=3, n=100, ld=4000)) == 2
        assert call(fn, x=None) == 1
        assert call(fn, q1=None) == 1
        assert call(fn, plan=None) == 1
        assert call(fn, plan=FAKE + 32) == 4
        assert call(fn, r=_rows(rows=3, n=128, ld=40 * 128, dtype=B.BQ_F16), x=FAKE + 2) == 4  # two elements at a time
        assert call(fn, r=_rows(rows=0, n=128, ld=40 * 128), x=None, y=None) == 0


def test_bwd_empty_batch_needs_no_plan_or_workspace():
    # dx alone on an empty batch: nothing to launch, nothing to clear
    L = B.lib()
    r = _rows(rows=0, n=1024, dtype=B.BQ_F16)
    assert L.bq_butterfly_bwd(None, None, None, FAKE, None, None, 0, ctypes.byref(r), None) == 0
    assert L.bq_butterfly_bwd_static(None, None, None, FAKE, None, ctypes.byref(r), None) == 0
    assert L.bq_butterfly_bwd(None, None, None, None, None, None, 0, ctypes.byref(r), None) == 1  # no output at all


def test_bwd_static_validation():
    L = B.lib()
    cap = B.bq_butterfly_bwd_static_max_bytes()
    assert cap == 32 << 20

    def call(r, x=FAKE, dy=FAKE, plan=FAKE, dx=FAKE, dth=FAKE):
        return L.bq_butterfly_bwd_static(x, dy, plan, dx, dth, ctypes.byref(r), None)

    r = _rows(rows=64, n=1024, dtype=B.BQ_BF16)
    assert call(r, x=None) == 1
    assert call(r, plan=None) == 1
    assert call(r, dx=None, dth=None) == 1
    assert call(r, plan=FAKE + 16) == 4
    assert call(_rows(rows=64, n=48)) == 2
    # a batch whose scratch need exceeds the fixed array is refused before anything touches the GPU
    big = _rows(rows=4096, n=128, heads=4096, dtype=B.BQ_F16)
    assert B.bq_butterfly_bwd_workspace_bytes(big) > cap
    assert call(big) == 5
    assert b"fixed scratch" in L.bq_last_error()


def test_hadamard_validation():
    L = B.lib()

    def call(r, x=FAKE, y=FAKE):
        return L.bq_hadamard_fwd(x, y, ctypes.byref(r), None)

    assert call(_rows(rows=0, n=4096, dtype=B.BQ_F16)) == 0
    assert call(_rows(rows=3, n=4096, dtype=B.BQ_F16), x=None) == 1
    assert call(_rows(rows=3, n=1024, dtype=B.BQ_F16)) == 6       # only n = 4096 and 8192
    assert call(_rows(rows=3, n=4096, dtype=B.BQ_F16, ld=4100)) == 6  # rows not 16-byte aligned
    assert call(_rows(rows=3, n=4096, dtype=B.BQ_F32), y=FAKE + 2) == 4
    assert call(_rows(rows=3, n=48)) == 2
