"""The measurement helpers: the copy copies, the read probe sees every byte once, the FMA loop reports its count."""
import numpy as np
import pytest

from paper_2509_09679_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes", [16, 4096 * 16 + 16, 50_000_000 - 50_000_000 % 16, 0])
def test_copy_and_read_probe(nbytes):
    import torch

    g = torch.Generator(device="cuda:0").manual_seed(nbytes + 1)
    src = torch.randint(0, 256, (max(nbytes, 16),), generator=g, device="cuda:0", dtype=torch.uint8)
    dst = torch.full_like(src, 7)
    B.bq_probe_copy(src, dst, nbytes)
    assert torch.equal(dst[:nbytes], src[:nbytes]) and (dst[nbytes:] == 7).all()
    sink = torch.empty(B.bq_probe_read_sink_bytes(), dtype=torch.uint8, device="cuda:0")
    B.bq_probe_read(src, nbytes, sink)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32).reshape(-1, 4), axis=0)
    want = np.bitwise_xor.reduce(src[:nbytes].cpu().numpy().view(np.uint32).reshape(-1, 4), axis=0) if nbytes else np.zeros(4, np.uint32)
    assert np.array_equal(got, want)


def test_fma_probe_counts_its_work():
    import torch

    out = torch.zeros(B.bq_probe_fma_out_floats(), dtype=torch.float32, device="cuda:0")
    n = B.bq_probe_fma(out, 8)
    assert n == out.numel() * 16 * 8
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out != 0).any()
