"""bq_hadamard_fwd (additions and subtractions only, no plan) against the Hadamard oracle."""
import numpy as np
import pytest

import gpu_util as gu
import oracle
from paper_2509_09679_amd import binding as B
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu


def _run(x_store, n, heads, dtype, pad=0, inplace=False):
    import torch

    rows, w = x_store.shape
    xfull = torch.zeros((rows, w + pad), dtype=synth.torch_dtype(dtype), device="cuda:0")
    xfull[:, :w] = synth.storage_to_torch(x_store, dtype, "cuda:0")
    x = xfull[:, :w]
    if inplace:
        y = x
    else:
        yfull = torch.full((rows, w + pad), 7.0, dtype=x.dtype, device="cuda:0")
        y = yfull[:, :w]
    B.bq_hadamard_fwd(x, y, B.make_rows(x, n, heads, y))
    torch.cuda.synchronize()
    if pad and not inplace:
        assert (yfull[:, w:] == 7.0).all(), "kernel wrote into the row padding"
    return synth.torch_to_storage(y, dtype)


@pytest.mark.parametrize("n,heads,rows,dtype,pad", [(4096, 1, 700, "f16", 0), (4096, 1, 1, "f16", 0), (4096, 2, 333, "bf16", 16),
                                                    (4096, 1, 300, "f32", 8), (8192, 1, 517, "bf16", 0), (8192, 1, 130, "f16", 24),
                                                    (8192, 2, 65, "f32", 0), (4096, 3, 2000, "f16", 0)])
def test_hadamard_matches_oracle(n, heads, rows, dtype, pad):
    x, _, _ = synth.small_case(n, rows, dtype, heads=heads, seed=rows)
    ref = oracle.hadamard(synth.to_f64(x, dtype), n, heads)
    y = _run(x, n, heads, dtype, pad=pad)
    gu.check_rotated(y, ref, dtype, f"hadamard n={n}")
    if pad == 0:
        y2 = _run(x, n, heads, dtype, inplace=True)
        assert np.array_equal(y2, y)


def test_hadamard_equals_the_butterfly_kernel_at_a_quarter_pi_up_to_signs():
    # the learned transform with every angle at pi/4 is H_n diag((-1)^popcount) / sqrt(n)
    n, rows, dtype = 4096, 256, "f32"
    x, _, _ = synth.small_case(n, rows, dtype, seed=5)
    sign = np.array([(-1.0) ** bin(c).count("1") for c in range(n)], dtype=np.float32)
    theta = np.full((1, 12, n // 2), np.pi / 4, dtype=np.float32)
    yb = gu.run_transform(x * sign, theta, n, 1, dtype)
    yh = _run(x, n, 1, dtype)  # x * sign * sign = x
    ref = oracle.hadamard(synth.to_f64(x, dtype), n)
    gu.check_rotated(yh, ref, dtype, "hadamard")
    # float32(pi/4) is not exactly pi/4: the butterfly deviates by about 12 layers x 4e-8
    assert np.abs(yb.astype(np.float64) - ref).max() <= 2e-6 * np.abs(ref).max()


def test_hadamard_rejects_other_sizes():
    import torch

    x = torch.zeros((4, 1024), dtype=torch.float16, device="cuda:0")
    with pytest.raises(B.BqError) as e:
        B.bq_hadamard_fwd(x, x, B.make_rows(x, 1024, 1))
    assert e.value.status == 6
