"""A plan buffer that bq_plan_build did not fill for the call's (n, heads) is recognised on the device: the
kernels return before their first table access and the outputs keep their contents.  The buffers here are
always as large as the call's own plan would be, so that no access could leave them even if the check failed."""
import numpy as np
import pytest

from paper_2509_09679_amd import binding as B

pytestmark = pytest.mark.gpu

SHAPES = [(64, 4, 300), (512, 1, 257), (1024, 4, 64), (4096, 1, 70), (4096, 2, 33), (8192, 1, 40), (16384, 1, 9)]


def _wrong_plan(n, heads, kind):
    import torch

    size = B.bq_plan_bytes(n, heads)
    plan = torch.zeros(size, dtype=torch.uint8, device="cuda:0")
    if kind == "other_shape":  # a valid plan of a smaller shape at the front of the buffer
        m = n // 2
        theta = torch.full((1, m.bit_length() - 1, m // 2), 0.3, dtype=torch.float32, device="cuda:0")
        B.bq_plan_build(theta, m, 1, plan)
    return plan


@pytest.mark.parametrize("kind", ["never_built", "other_shape"])
@pytest.mark.parametrize("n,heads,rows", SHAPES)
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_outputs_keep_their_contents(n, heads, rows, dtype, kind):
    import torch

    tdt = torch.float16 if dtype == "f16" else torch.float32
    g = torch.Generator(device="cuda:0").manual_seed(n + rows)
    x = torch.randn((rows, n * heads), generator=g, device="cuda:0", dtype=torch.float32).to(tdt)
    plan = _wrong_plan(n, heads, kind)
    r = B.make_rows(x, n, heads)
    k = n.bit_length() - 1

    y = torch.full_like(x, 7.0)
    B.bq_butterfly_fwd(x, y, plan, r)
    B.bq_butterfly_inv(x, y, plan, r)
    assert (y == 7.0).all()

    for bits, group in ((2, 128), (4, 64)):
        if group > n:
            continue
        codes, scales = B.alloc_quant_outputs(rows, n, heads, bits, group, "f16", x.device)
        codes.fill_(0x5A)
        scales.fill_(3.0)
        B.bq_butterfly_fwd_quant(x, plan, codes, scales, B.make_quant(bits, group, "f16"), r)
        assert (codes == 0x5A).all() and (scales == 3.0).all()

    dx = torch.full_like(x, 7.0)
    dth = torch.full((heads, k, n // 2), 5.0, dtype=torch.float32, device="cuda:0")
    ws = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(r)), dtype=torch.uint8, device="cuda:0")
    B.bq_butterfly_bwd(x, x, plan, dx, dth, ws, r)
    B.bq_butterfly_bwd(x, x, plan, None, dth, ws, r)
    torch.cuda.synchronize()
    assert (dx == 7.0).all() and (dth == 5.0).all()


def test_a_rebuilt_plan_is_accepted_again():
    import torch

    n, rows = 4096, 50
    x = torch.randn((rows, n), device="cuda:0", dtype=torch.float32)
    plan = _wrong_plan(n, 1, "other_shape")
    y = torch.full_like(x, 7.0)
    r = B.make_rows(x, n, 1)
    B.bq_butterfly_fwd(x, y, plan, r)
    assert (y == 7.0).all()
    theta = torch.zeros((1, 12, n // 2), dtype=torch.float32, device="cuda:0")
    B.bq_plan_build(theta, n, 1, plan)
    B.bq_butterfly_fwd(x, y, plan, r)
    assert np.array_equal(y.cpu().numpy(), x.cpu().numpy())  # theta = 0: the identity
