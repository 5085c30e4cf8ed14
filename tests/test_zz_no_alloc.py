"""bq_butterfly_bwd_static (fixed scratch array inside the library, no allocation) against bq_butterfly_bwd
(caller's workspace): same kernels, same summation order, so dx and dtheta must be identical bit for bit.
Two calls in a row share the array; the second has a smaller batch and a different shape."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _both(n, heads, rows, dtype, seed):
    import torch

    from paper_2509_09679_amd import binding as B
    from paper_2509_09679_amd import synth

    x_s, theta, dy_s = synth.small_case(n, rows, dtype, seed=seed, heads=heads, with_dy=True)
    dev = "cuda:0"
    x = synth.storage_to_torch(x_s, dtype, dev)
    dy = synth.storage_to_torch(dy_s, dtype, dev)
    th = torch.from_numpy(np.ascontiguousarray(theta)).to(dev)
    plan = B.alloc_plan(th, n, heads)
    r = B.make_rows(x, n, heads)
    need = B.bq_butterfly_bwd_workspace_bytes(r)
    assert need <= B.bq_butterfly_bwd_static_max_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    dx_a, dx_b = torch.zeros_like(x), torch.zeros_like(x)
    dth_a, dth_b = torch.full_like(th, 3.0), torch.full_like(th, -3.0)
    B.bq_butterfly_bwd(x, dy, plan, dx_a, dth_a, ws, r)
    torch.cuda.synchronize()
    # everything the second call needs exists now: it must not allocate
    before = torch.cuda.memory_allocated()
    B.bq_butterfly_bwd_static(x, dy, plan, dx_b, dth_b, r)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return (dx_a.view(torch.uint8).cpu().numpy(), dx_b.view(torch.uint8).cpu().numpy(),
            dth_a.cpu().numpy(), dth_b.cpu().numpy(), x_s, dy_s, theta)


def test_static_scratch_backward_matches_workspace_backward_twice():
    import oracle
    from paper_2509_09679_amd import synth
    import gpu_util as gu

    # first call: the n = 4096 kernels on several hundred rows; second: fewer rows of another shape
    for n, heads, rows, dtype, seed in ((4096, 1, 300, "f16", 11), (1024, 1, 77, "bf16", 12), (128, 4, 33, "f32", 13)):
        dx_a, dx_b, dth_a, dth_b, x_s, dy_s, theta = _both(n, heads, rows, dtype, seed)
        assert np.array_equal(dx_a, dx_b), (n, rows)
        assert np.array_equal(dth_a.view(np.uint32), dth_b.view(np.uint32)), (n, rows)
        # and both agree with the oracle
        rdx, rdth, ab = oracle.backward(synth.to_f64(x_s, dtype), synth.to_f64(dy_s, dtype), theta, n, heads)
        gu.check_dtheta(dth_b, rdth, ab, what=f"static n={n}")


def test_static_scratch_refuses_oversized_batches():
    import torch

    from paper_2509_09679_amd import binding as B

    r = B.bq_rows()
    r.rows, r.n, r.heads, r.dtype = 4096, 128, 4096, B.BQ_F16
    r.ld_x = r.ld_y = 128 * 4096
    assert B.bq_butterfly_bwd_workspace_bytes(r) > B.bq_butterfly_bwd_static_max_bytes()
    t = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.BqError) as e:
        B.bq_butterfly_bwd_static(t, t, t, t, t, r)
    assert e.value.status == 5
