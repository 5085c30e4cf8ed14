"""GPU parity at the full workload sizes, in the launch configuration bench.py times: inputs are
drawn on the device, the library runs on the whole batch, and the oracle checks sampled rows (rows are
independent) or, where it is cheap enough, the whole result (dtheta summed over all rows, in chunks)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_09679_amd import binding as B
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu
gu = pytest.importorskip("gpu_util")

DEV = "cuda:0"


def _sample_rows(T, count, seed):
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, 1, T // 2, T - 2, T - 1], rng.integers(0, T, size=count)]))
    return rows


def test_workload3_full_size_fused_forward_inverse():
    cfg, T = 3, 262144
    x, th, _ = synth.device_rows(cfg, T, DEV)
    wl = synth.make_workload(cfg, rows=1)
    n = wl.n
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, 1)
    rows = B.make_rows(x, n, 1)
    pick = _sample_rows(T, 96, 1)
    xs = synth.torch_to_storage(x[torch.as_tensor(pick, device=DEV)], wl.dtype)
    y_ref = oracle.forward(synth.to_f64(xs, wl.dtype), th, n)
    for bits in (2, 4):
        codes, scales = B.alloc_quant_outputs(T, n, 1, bits, 128, "f16", DEV)
        codes.fill_(0x5A)
        B.bq_butterfly_fwd_quant(x, plan, codes, scales, B.make_quant(bits, 128, "f16"), rows)
        torch.cuda.synchronize()
        c = codes[torch.as_tensor(pick, device=DEV)].cpu().numpy()
        s = scales[torch.as_tensor(pick, device=DEV)].float().cpu().numpy()
        gu.check_fused_codes(c, s, y_ref, bits, 128, "f16", wl.dtype, f"c3 full int{bits}")
        # properties that hold for every row: codes in range, every non-zero group reaches +-qmax
        qmax = 2 ** (bits - 1) - 1
        blk = codes[:4096].cpu().numpy()
        q = oracle.unpack_codes(blk, bits).reshape(4096, -1, 128)
        assert np.abs(q).max() <= qmax
        nz = scales[:4096].float().cpu().numpy() > 0
        assert (np.abs(q).max(axis=2)[nz] == qmax).all()
        del codes, scales
    y = torch.empty_like(x)
    B.bq_butterfly_fwd(x, y, plan, rows)
    torch.cuda.synchronize()
    ys = synth.torch_to_storage(y[torch.as_tensor(pick, device=DEV)], wl.dtype)
    gu.check_rotated(ys, y_ref, wl.dtype, "c3 full fwd")
    xi = torch.empty_like(x)
    B.bq_butterfly_inv(y, xi, plan, rows)
    torch.cuda.synchronize()
    xis = synth.torch_to_storage(xi[torch.as_tensor(pick, device=DEV)], wl.dtype)
    gu.check_rotated(xis, oracle.inverse(synth.to_f64(ys, wl.dtype), th, n), wl.dtype, "c3 full inv")
    # norm preservation on a large block of rows (any row): |Bx| = |x| up to output rounding
    nx = torch.linalg.vector_norm(x[:65536].float(), dim=1)
    ny = torch.linalg.vector_norm(y[:65536].float(), dim=1)
    assert torch.all((nx - ny).abs() <= 2e-3 * nx)


def test_workload3_every_row_against_the_oracle():
    """The whole calibration batch, every element: forward, inverse, INT2 and INT4 codes and scales.  The oracle runs
    on the CPU chunk by chunk; the comparisons (the criteria of gpu_util.check_rotated / check_fused_codes) run in
    torch on the device."""
    cfg, T, chunk = 3, 262144, 16384
    x, th, _ = synth.device_rows(cfg, T, DEV)
    wl = synth.make_workload(cfg, rows=1)
    n, dtype = wl.n, wl.dtype
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, 1)
    rows = B.make_rows(x, n, 1)
    y, xi = torch.empty_like(x), torch.empty_like(x)
    B.bq_butterfly_fwd(x, y, plan, rows)
    B.bq_butterfly_inv(y, xi, plan, rows)
    out = {}
    for bits in (2, 4):
        out[bits] = B.alloc_quant_outputs(T, n, 1, bits, 128, "f16", DEV)
        B.bq_butterfly_fwd_quant(x, plan, out[bits][0], out[bits][1], B.make_quant(bits, 128, "f16"), rows)
    torch.cuda.synchronize()
    worst = 0.0
    for r0 in range(0, T, chunk):
        sl = slice(r0, r0 + chunk)
        x64 = synth.to_f64(synth.torch_to_storage(x[sl], dtype), dtype)
        y_ref = oracle.forward(x64, th, n)
        worst = max(worst, gu.check_rotated_dev(y[sl], y_ref, dtype, f"c3 rows {r0}.. fwd"))
        for bits in (2, 4):
            gu.check_fused_codes_dev(out[bits][0][sl], out[bits][1][sl], y_ref, bits, 128, "f16", dtype, f"c3 rows {r0}.. int{bits}")
        # the inverse is checked on what the forward kernel actually stored
        y64 = synth.to_f64(synth.torch_to_storage(y[sl], dtype), dtype)
        gu.check_rotated_dev(xi[sl], oracle.inverse(y64, th, n), dtype, f"c3 rows {r0}.. inv")
    assert worst > 0.0


def test_workload4_full_size_per_head_quant():
    cfg, T = 4, 8192
    x, th, _ = synth.device_rows(cfg, T, DEV)
    wl = synth.make_workload(cfg, rows=1)
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, wl.n, wl.heads)
    codes, scales = B.alloc_quant_outputs(T, wl.n, wl.heads, 4, wl.n, "f32", DEV)
    B.bq_butterfly_fwd_quant(x, plan, codes, scales, B.make_quant(4, wl.n, "f32"), B.make_rows(x, wl.n, wl.heads))
    torch.cuda.synchronize()
    xs = synth.torch_to_storage(x, wl.dtype)
    y_ref = oracle.forward(synth.to_f64(xs, wl.dtype), th, wl.n, wl.heads)  # the whole batch
    gu.check_fused_codes(codes.cpu().numpy(), scales.cpu().numpy(), y_ref, 4, wl.n, "f32", wl.dtype, "c4 full")


def _oracle_dtheta_in_chunks(x, dy, th, n, dtype, chunk=8192):
    T = x.shape[0]
    acc = None
    ab = None
    for r0 in range(0, T, chunk):
        xs = synth.to_f64(synth.torch_to_storage(x[r0:r0 + chunk], dtype), dtype)
        gs = synth.to_f64(synth.torch_to_storage(dy[r0:r0 + chunk], dtype), dtype)
        _, d, a = oracle.backward(xs, gs, th, n)
        acc = d if acc is None else acc + d
        ab = a if ab is None else ab + a
    return acc, ab


@pytest.mark.parametrize("cfg,T", [(5, 65536), (5, 131072 + 2500), (3, 262144), (3, 262144 + 4500)])
def test_backward_full_size(cfg, T):
    # cfg 5: n=8192 bf16; cfg 3 shape: n=4096 f16.  Each at its benchmark size (one chunk of the backward
    # pipeline) and just above the chunk size (two chunks, the second short and ragged)
    x, th, dy = synth.device_rows(cfg, T, DEV, want_dy=True)
    wl = synth.make_workload(cfg, rows=1)
    n, dtype = wl.n, wl.dtype
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, 1)
    rows = B.make_rows(x, n, 1)
    dx = torch.empty_like(x)
    dth = torch.empty_like(theta)
    ws = torch.empty(B.bq_butterfly_bwd_workspace_bytes(rows), dtype=torch.uint8, device=DEV)
    B.bq_butterfly_bwd(x, dy, plan, dx, dth, ws, rows)
    torch.cuda.synchronize()
    del ws
    for r0 in range(0, T, 16384):  # dx of every row (the comparison itself runs on the device)
        g64 = synth.to_f64(synth.torch_to_storage(dy[r0:r0 + 16384], dtype), dtype)
        gu.check_rotated_dev(dx[r0:r0 + 16384], oracle.inverse(g64, th, n), dtype, f"cfg {cfg} full dx rows {r0}..")
    ref, ab = _oracle_dtheta_in_chunks(x, dy, th, n, dtype)
    gu.check_dtheta(dth.cpu().numpy(), ref, ab, what=f"cfg {cfg} full dtheta")


@pytest.mark.parametrize("m", [4096, 11008])
def test_weight_side_rotation_quant_and_gradient(m):
    # W' = W B^T is the forward transform over the rows of W ([m, n], n = 4096, fp16, no outlier channels);
    # group-wise INT2 quantisation of W' (the weight side of W2A16) and the weight side's dtheta, which is
    # the same backward call with the rows of W in place of activations.  Checked on the whole matrix.
    n, dtype = 4096, "f16"
    W, theta, dW = synth.small_case(n, m, dtype, seed=90 + m % 7, outliers=0, dist="normal", with_dy=True)
    th = torch.from_numpy(theta).to(DEV)
    plan = B.alloc_plan(th, n, 1)
    Wd = synth.storage_to_torch(W, dtype, DEV)
    dWd = synth.storage_to_torch(dW, dtype, DEV)
    rows = B.make_rows(Wd, n, 1)
    codes, scales = B.alloc_quant_outputs(m, n, 1, 2, 128, "f16", DEV)
    B.bq_butterfly_fwd_quant(Wd, plan, codes, scales, B.make_quant(2, 128, "f16"), rows)
    dth = torch.empty_like(th)
    ws = torch.empty(B.bq_butterfly_bwd_workspace_bytes(rows), dtype=torch.uint8, device=DEV)
    B.bq_butterfly_bwd(Wd, dWd, plan, None, dth, ws, rows)
    torch.cuda.synchronize()
    W64 = synth.to_f64(W, dtype)
    gu.check_fused_codes(codes.cpu().numpy(), scales.float().cpu().numpy(), oracle.forward(W64, theta, n), 2, 128, "f16",
                         dtype, f"weight side m={m}")
    _, ref, ab = oracle.backward(W64, synth.to_f64(dW, dtype), theta, n)
    gu.check_dtheta(dth.cpu().numpy(), ref, ab, what=f"weight side m={m} dtheta")


def test_n8192_full_size_forward_inverse_quant():
    # the rows of the n = 8192 workload (T = 65536, bf16) through forward, inverse and the fused quantiser
    cfg, T = 5, 65536
    x, th, _ = synth.device_rows(cfg, T, DEV)
    wl = synth.make_workload(cfg, rows=1)
    n, dtype = wl.n, wl.dtype
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, 1)
    rows = B.make_rows(x, n, 1)
    pick = torch.as_tensor(_sample_rows(T, 48, 3), device=DEV)
    xs = synth.torch_to_storage(x[pick], dtype)
    y_ref = oracle.forward(synth.to_f64(xs, dtype), th, n)
    y = torch.empty_like(x)
    B.bq_butterfly_fwd(x, y, plan, rows)
    torch.cuda.synchronize()
    ys = synth.torch_to_storage(y[pick], dtype)
    gu.check_rotated(ys, y_ref, dtype, "n8192 full fwd")
    xi = torch.empty_like(x)
    B.bq_butterfly_inv(y, xi, plan, rows)
    torch.cuda.synchronize()
    gu.check_rotated(synth.torch_to_storage(xi[pick], dtype), oracle.inverse(synth.to_f64(ys, dtype), th, n), dtype,
                     "n8192 full inv")
    nx = torch.linalg.vector_norm(x.float(), dim=1)
    ny = torch.linalg.vector_norm(y.float(), dim=1)
    assert torch.all((nx - ny).abs() <= 4e-3 * nx)  # bf16 output rounding
    del xi, y
    codes, scales = B.alloc_quant_outputs(T, n, 1, 2, 128, "f16", DEV)
    B.bq_butterfly_fwd_quant(x, plan, codes, scales, B.make_quant(2, 128, "f16"), rows)
    torch.cuda.synchronize()
    gu.check_fused_codes(codes[pick].cpu().numpy(), scales[pick].float().cpu().numpy(), y_ref, 2, 128, "f16", dtype,
                         "n8192 full int2")


def test_workload4_full_size_per_head_backward():
    # 32 heads x n = 128, T = 8192, bf16: dx and dtheta on the whole batch
    cfg, T = 4, 8192
    x, th, dy = synth.device_rows(cfg, T, DEV, want_dy=True)
    wl = synth.make_workload(cfg, rows=1)
    n, H, dtype = wl.n, wl.heads, wl.dtype
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, H)
    rows = B.make_rows(x, n, H)
    dx = torch.empty_like(x)
    dth = torch.empty_like(theta)
    ws = torch.empty(B.bq_butterfly_bwd_workspace_bytes(rows), dtype=torch.uint8, device=DEV)
    B.bq_butterfly_bwd(x, dy, plan, dx, dth, ws, rows)
    torch.cuda.synchronize()
    xs = synth.to_f64(synth.torch_to_storage(x, dtype), dtype)
    gs = synth.to_f64(synth.torch_to_storage(dy, dtype), dtype)
    rdx, rdth, ab = oracle.backward(xs, gs, th, n, H)
    gu.check_rotated(synth.torch_to_storage(dx, dtype), rdx, dtype, "c4 full dx")
    gu.check_dtheta(dth.cpu().numpy(), rdth, ab, what="c4 full dtheta")


@pytest.mark.parametrize("n,heads", [(256, 1), (512, 2)])
def test_backward_blocks_of_small_transforms_across_two_chunks(n, heads):
    # n < 4096: the kernels work on 4096-element blocks, 2^18 of them per launch.  A batch just above that runs a
    # second launch whose last block is short: dx on sampled rows, dtheta on the whole batch (oracle in chunks).
    dtype = "f16"
    width = n * heads
    block_rows = 4096 // width
    T = (1 << 18) * block_rows + 2 * block_rows + max(1, block_rows // 3)
    g = torch.Generator(device=DEV)
    g.manual_seed(9679 + n)
    x = torch.randn((T, width), generator=g, device=DEV, dtype=torch.float32).to(torch.float16)
    dy = torch.randn((T, width), generator=g, device=DEV, dtype=torch.float32).to(torch.float16)
    th = synth.small_case(n, 1, dtype, heads=heads, seed=7)[1]
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, heads)
    rows = B.make_rows(x, n, heads)
    dx = torch.empty_like(x)
    dth = torch.empty_like(theta)
    ws = torch.empty(B.bq_butterfly_bwd_workspace_bytes(rows), dtype=torch.uint8, device=DEV)
    B.bq_butterfly_bwd(x, dy, plan, dx, dth, ws, rows)
    torch.cuda.synchronize()
    del ws
    pick = np.unique(np.concatenate([_sample_rows(T, 64, 4), np.arange(T - 3 * block_rows, T),
                                     np.arange((1 << 18) * block_rows - 4, (1 << 18) * block_rows + 4)]))
    pt = torch.as_tensor(pick, device=DEV)
    gs = synth.torch_to_storage(dy[pt], dtype)
    gu.check_rotated(synth.torch_to_storage(dx[pt], dtype), oracle.inverse(synth.to_f64(gs, dtype), th, n, heads), dtype,
                     f"two chunks dx n={n}")
    acc = ab = None
    step = 1 << 16
    for r0 in range(0, T, step):
        xs = synth.to_f64(synth.torch_to_storage(x[r0:r0 + step], dtype), dtype)
        g64 = synth.to_f64(synth.torch_to_storage(dy[r0:r0 + step], dtype), dtype)
        _, d, a = oracle.backward(xs, g64, th, n, heads)
        acc = d if acc is None else acc + d
        ab = a if ab is None else ab + a
    gu.check_dtheta(dth.cpu().numpy(), acc, ab, what=f"two chunks dtheta n={n} H={heads}")


def test_backward_small_transforms_many_rows():
    # n = 128, one head: 16 rows per workgroup pass, 4096 slots of partial sums, about 500 row groups per workgroup
    n, heads, dtype = 128, 1, "bf16"
    T = (1 << 21) + 5
    g = torch.Generator(device=DEV)
    g.manual_seed(9679)
    x = torch.randn((T, n), generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    dy = torch.randn((T, n), generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    th = synth.small_case(n, 1, dtype, seed=11)[1]
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, heads)
    rows = B.make_rows(x, n, heads)
    dx = torch.empty_like(x)
    dth = torch.empty_like(theta)
    ws = torch.empty(B.bq_butterfly_bwd_workspace_bytes(rows), dtype=torch.uint8, device=DEV)
    B.bq_butterfly_bwd(x, dy, plan, dx, dth, ws, rows)
    torch.cuda.synchronize()
    pt = torch.as_tensor(_sample_rows(T, 256, 5), device=DEV)
    gs = synth.torch_to_storage(dy[pt], dtype)
    gu.check_rotated(synth.torch_to_storage(dx[pt], dtype), oracle.inverse(synth.to_f64(gs, dtype), th, n), dtype, "many rows dx")
    acc = ab = None
    step = 1 << 18
    for r0 in range(0, T, step):
        xs = synth.to_f64(synth.torch_to_storage(x[r0:r0 + step], dtype), dtype)
        g64 = synth.to_f64(synth.torch_to_storage(dy[r0:r0 + step], dtype), dtype)
        _, d, a = oracle.backward(xs, g64, th, n)
        acc = d if acc is None else acc + d
        ab = a if ab is None else ab + a
    gu.check_dtheta(dth.cpu().numpy(), acc, ab, what="many rows dtheta n=128")


@pytest.mark.parametrize("cfg,T", [(3, 131072), (5, 32768)])
def test_float32_rows_at_the_sizes_bench_times(cfg, T):
    # the rows of the n = 4096 / n = 8192 workloads as float32 (the 1e-5 tolerance class): forward, inverse,
    # fused quantiser and fake quantisation with histogram on the whole batch, sampled rows against the oracle
    xh, th, _ = synth.device_rows(cfg, T, DEV)
    x = xh.float()
    del xh
    n, dtype = synth.make_workload(cfg, rows=1).n, "f32"
    plan = B.alloc_plan(torch.from_numpy(th).to(DEV), n, 1)
    rows = B.make_rows(x, n, 1)
    pick = torch.as_tensor(_sample_rows(T, 48, 5), device=DEV)
    xs = synth.torch_to_storage(x[pick], dtype)
    y_ref = oracle.forward(synth.to_f64(xs, dtype), th, n)
    y = torch.empty_like(x)
    B.bq_butterfly_fwd(x, y, plan, rows)
    torch.cuda.synchronize()
    ys = synth.torch_to_storage(y[pick], dtype)
    gu.check_rotated(ys, y_ref, dtype, f"f32 n={n} full fwd")
    nx, ny = torch.linalg.vector_norm(x.double(), dim=1), torch.linalg.vector_norm(y.double(), dim=1)
    assert torch.all((nx - ny).abs() <= 1e-5 * nx)  # every row: the transform preserves the norm
    B.bq_butterfly_inv(y, y, plan, rows)  # in place
    torch.cuda.synchronize()
    gu.check_rotated(synth.torch_to_storage(y[pick], dtype), oracle.inverse(synth.to_f64(ys, dtype), th, n), dtype,
                     f"f32 n={n} full inv")
    assert torch.all(torch.linalg.vector_norm((y - x).double(), dim=1) <= 2e-5 * nx)  # every row: inverse o forward
    q = B.make_quant(4, 128, "f16")
    codes, scales = B.alloc_quant_outputs(T, n, 1, 4, 128, "f16", DEV)
    B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, rows)
    hist = torch.zeros(16, dtype=torch.int64, device=DEV)
    B.bq_butterfly_fwd_fakequant(x, plan, y, hist, q, rows)
    torch.cuda.synchronize()
    gu.check_fused_codes(codes[pick].cpu().numpy(), scales[pick].float().cpu().numpy(), y_ref, 4, 128, "f16", dtype,
                         f"f32 n={n} full int4")
    # the fake-quantised rows and the histogram agree with the fused kernel's codes and scales on the whole batch
    shift = torch.arange(0, 8, 4, device=DEV, dtype=torch.uint8)
    c = ((codes.unsqueeze(-1) >> shift) & 15).reshape(T, n).to(torch.int64)
    c = torch.where(c >= 8, c - 16, c)
    assert torch.equal(torch.bincount((c + 8).reshape(-1), minlength=16), hist)
    want = c.reshape(T, n // 128, 128).float() * scales.float().unsqueeze(-1)
    assert torch.equal(want.reshape(T, n), y)


@pytest.mark.parametrize("n,heads,T,dtype,group", [(4096, 1, (1 << 20) + 5, "f16", 128), (128, 32, (1 << 20) + 3, "bf16", 128),
                                                   (16384, 1, (1 << 18) + 3, "f16", 256), (8192, 1, (1 << 19) + 2, "bf16", 128)])
def test_row_offsets_beyond_four_gibibytes(n, heads, T, dtype, group):
    """8 GiB per array, so row offsets pass 2^31 and 2^32 bytes (and 2^31 elements), on each kernel family: n = 4096,
    per-head transforms of 128, the general kernel (n = 16384) and n = 8192.  The rows around those boundaries and the
    last ones are checked against the oracle: forward, inverse, fused quantiser, and a backward pass whose dy is
    non-zero only in the last rows (dtheta then comes from there alone)."""
    w = n * heads
    tdt = synth.torch_dtype(dtype)
    g = torch.Generator(device=DEV).manual_seed(20 + n)
    x = torch.empty((T, w), dtype=tdt, device=DEV)
    piece = (1 << 30) // w
    for r0 in range(0, T, piece):  # in pieces: the float32 draw of the whole batch would take 16 GiB more
        r1 = min(T, r0 + piece)
        x[r0:r1] = (torch.randn((r1 - r0, w), generator=g, device=DEV) * 1.5).to(tdt)
    rng = np.random.default_rng(21 + n)
    k = n.bit_length() - 1
    th = (rng.standard_normal((heads, k, n // 2)) * 0.7).astype(np.float32)
    theta = torch.from_numpy(th).to(DEV)
    plan = B.alloc_plan(theta, n, heads)
    rows = B.make_rows(x, n, heads)
    b31 = (1 << 31) // (w * 2)  # the row whose first byte is at 2^31
    pick = np.array([0, b31 - 1, b31, b31 + 1, 2 * b31 - 1, 2 * b31, 2 * b31 + 1, 3 * b31, T - 3, T - 2, T - 1])
    sel = torch.as_tensor(pick, device=DEV)
    xs = synth.torch_to_storage(x[sel], dtype)
    y_ref = oracle.forward(synth.to_f64(xs, dtype), th, n, heads)
    y = torch.full_like(x, 7.0)
    B.bq_butterfly_fwd(x, y, plan, rows)
    torch.cuda.synchronize()
    ys = synth.torch_to_storage(y[sel], dtype)
    gu.check_rotated(ys, y_ref, dtype, "8 GiB fwd")
    assert not (y[T - 1024:] == 7.0).all(dim=1).any() and not (y[2 * b31 - 512:2 * b31 + 512] == 7.0).all(dim=1).any()
    for bits in (2, 4):
        codes, scales = B.alloc_quant_outputs(T, n, heads, bits, group, "f16", DEV)
        B.bq_butterfly_fwd_quant(x, plan, codes, scales, B.make_quant(bits, group, "f16"), rows)
        torch.cuda.synchronize()
        gu.check_fused_codes(codes[sel].cpu().numpy(), scales[sel].float().cpu().numpy(), y_ref, bits, group, "f16", dtype,
                             f"8 GiB int{bits}")
        del codes, scales
    B.bq_butterfly_inv(y, y, plan, rows)  # in place
    torch.cuda.synchronize()
    gu.check_rotated(synth.torch_to_storage(y[sel], dtype), oracle.inverse(synth.to_f64(ys, dtype), th, n, heads), dtype, "8 GiB inv")
    # backward: dy is zero except in the last 37 rows
    R = 37
    dy = y
    dy.zero_()
    dy[T - R:] = (torch.randn((R, w), generator=g, device=DEV)).to(tdt)
    dx = torch.full_like(x, 7.0)
    dth = torch.empty_like(theta)
    ws = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(rows)), dtype=torch.uint8, device=DEV)
    B.bq_butterfly_bwd(x, dy, plan, dx, dth, ws, rows)
    torch.cuda.synchronize()
    xt = synth.torch_to_storage(x[T - R:], dtype)
    dyt = synth.torch_to_storage(dy[T - R:], dtype)
    dx_ref, dth_ref, absacc = oracle.backward(synth.to_f64(xt, dtype), synth.to_f64(dyt, dtype), th, n, heads, want_abs=True)
    gu.check_rotated(synth.torch_to_storage(dx[T - R:], dtype), dx_ref, dtype, "8 GiB dx tail")
    gu.check_dtheta(dth.cpu().numpy(), dth_ref, absacc, what="8 GiB dtheta")
    assert (dx[sel[:8]] == 0).all()  # dy = 0 there
