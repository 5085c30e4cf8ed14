"""The library's calls only enqueue kernels (no allocation, no synchronisation, no memset), so a sequence of
them can be captured into a HIP graph.  Every replay must reproduce the eager results bit for bit, also with
other work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2509_09679_amd import binding as B
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _bits(t):
    return t.contiguous().view(torch.uint8).cpu().numpy()


@pytest.mark.parametrize("n,heads,rows,dtype", [(4096, 1, 8, "f16"), (128, 32, 64, "bf16"), (8192, 1, 5, "bf16"),
                                                 (512, 1, 19, "f16")])
def test_captured_sequence_replays_bit_exact(n, heads, rows, dtype):
    k = n.bit_length() - 1
    xs, th, dys = synth.small_case(n, rows, dtype, heads=heads, seed=31 + n, with_dy=True)
    x = synth.storage_to_torch(xs, dtype, DEV)
    dy = synth.storage_to_torch(dys, dtype, DEV)
    theta = torch.from_numpy(th).to(DEV)
    plan = torch.empty(B.bq_plan_bytes(n, heads), dtype=torch.uint8, device=DEV)
    r = B.make_rows(x, n, heads)
    group = min(n, 128)
    q = B.make_quant(4, group, "f16")
    codes, scales = B.alloc_quant_outputs(rows, n, heads, 4, group, "f16", DEV)
    y, xi, yq, dx = (torch.empty_like(x) for _ in range(4))
    hist = torch.zeros(16, dtype=torch.int64, device=DEV)
    dth = torch.empty_like(theta)
    ws = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(r)), dtype=torch.uint8, device=DEV)
    outs = [codes, scales, y, xi, yq, hist, dx, dth]

    def sequence():
        B.bq_plan_build(theta, n, heads, plan)
        B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, r)
        B.bq_butterfly_fwd(x, y, plan, r)
        B.bq_butterfly_inv(y, xi, plan, r)
        B.bq_butterfly_fwd_fakequant(x, plan, yq, hist, q, r)
        B.bq_butterfly_bwd(x, dy, plan, dx, dth, ws, r)

    sequence()
    torch.cuda.synchronize()
    want = [_bits(o) for o in outs]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sequence()  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            sequence()
    torch.cuda.synchronize()

    for replay in range(3):
        for o in outs:
            o.fill_(3)  # every output must be rewritten by the replay
        ws.fill_(0xA5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, o, w in zip(("codes", "scales", "y", "xi", "yq", "hist", "dx", "dtheta"), outs, want):
            assert np.array_equal(_bits(o), w), f"replay {replay}: {name} differs from the eager result"
        # the program's own eager work between replays
        sequence()
        torch.cuda.synchronize()
