"""Pins for the oracle's transform (forward / inverse): the paper's printed matrices, the dense
definition, closed forms and invariants.  CPU only."""
import math
import os

import numpy as np
import pytest
from scipy.linalg import hadamard

import oracle
from oracle.dense import dense_butterfly, dense_layer, pair_indices


def _theta(rng, n, heads=1):
    k = n.bit_length() - 1
    return rng.uniform(-math.pi, math.pi, size=(heads, k, n // 2)).astype(np.float32)


def _read_constants(golden_dir):
    out = {}
    for line in open(os.path.join(golden_dir, "paper_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


# --- P1: index <-> angle map and sign convention, against the printed 8x8 layers -------------

def test_printed_n8_layers_match_dense_layer_and_stage_loop(golden_dir):
    rng = np.random.default_rng(1)
    theta = rng.uniform(-3, 3, size=(3, 4))
    printed = [np.zeros((8, 8)) for _ in range(3)]
    for line in open(os.path.join(golden_dir, "paper_n8_layers.txt")):
        if line.startswith("#") or not line.strip():
            continue
        layer, r, c, sign, fn, j = line.split()
        layer, r, c, j = int(layer), int(r), int(c), int(j)
        v = math.cos(theta[layer - 1, j - 1]) if fn == "cos" else math.sin(theta[layer - 1, j - 1])
        printed[layer - 1][r, c] = v if sign == "+" else -v
    for i in (1, 2, 3):
        assert np.array_equal(dense_layer(theta[i - 1], 8, i), printed[i - 1])
    # the C stage loop applies exactly these layers, layer 1 first
    th32 = theta.astype(np.float32)
    printed32 = [dense_layer(th32[i].astype(np.float64), 8, i + 1) for i in range(3)]
    x = rng.standard_normal((5, 8))
    want = (printed32[2] @ printed32[1] @ printed32[0] @ x.T).T
    got = oracle.forward(x, th32, 8)
    assert np.allclose(got, want, rtol=0, atol=1e-14)


def test_one_angle_at_a_time_n8():
    # a single non-zero angle must touch exactly the pair the paper prints for it
    expected_pairs = {1: [(0, 1), (2, 3), (4, 5), (6, 7)],
                      2: [(0, 2), (1, 3), (4, 6), (5, 7)],
                      3: [(0, 4), (1, 5), (2, 6), (3, 7)]}
    for i in (1, 2, 3):
        assert pair_indices(8, i) == expected_pairs[i]
        for j in range(4):
            th = np.zeros((1, 3, 4), np.float32)
            th[0, i - 1, j] = 0.3
            B = oracle.forward(np.eye(8), th, 8).T  # rows of result are B e_c => transpose
            a, b = expected_pairs[i][j]
            c, s = math.cos(np.float32(0.3)), math.sin(np.float32(0.3))
            want = np.eye(8)
            want[a, a], want[a, b], want[b, a], want[b, b] = c, -s, s, c
            assert np.allclose(B, want, atol=1e-15)


# --- P2: stage loop == dense definitional product -------------------------------------------

@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_stage_loop_equals_dense_product(n):
    rng = np.random.default_rng(n)
    th = _theta(rng, n)
    x = rng.standard_normal((7, n))
    B = dense_butterfly(th[0], n)
    assert np.allclose(oracle.forward(x, th, n), x @ B.T, rtol=0, atol=1e-13)
    assert np.allclose(oracle.inverse(x, th, n), x @ B, rtol=0, atol=1e-13)


def test_layer_order_matters_and_is_layer1_first():
    # B_k...B_1 differs from B_1...B_k for generic angles; the oracle must equal the former
    rng = np.random.default_rng(5)
    n = 8
    th = _theta(rng, n)
    L = [dense_layer(th[0, i].astype(np.float64), n, i + 1) for i in range(3)]
    first = L[2] @ L[1] @ L[0]
    other = L[0] @ L[1] @ L[2]
    assert np.abs(first - other).max() > 1e-2
    x = rng.standard_normal((3, n))
    assert np.allclose(oracle.forward(x, th, n), x @ first.T, atol=1e-14)
    # the other reading is the inverse with negated angles
    assert np.allclose(oracle.inverse(x, -th, n), x @ other.T, atol=1e-14)


# --- P3: theta = pi/4 everywhere is a signed Hadamard transform ------------------------------

@pytest.mark.parametrize("n", [2, 4, 16, 64, 256])
def test_hadamard_special_case(n, golden_dir):
    k = n.bit_length() - 1
    th = np.full((1, k, n // 2), math.pi / 4, dtype=np.float32)
    B = oracle.forward(np.eye(n), th, n).T
    H = hadamard(n).astype(np.float64) / math.sqrt(n)  # Sylvester construction, as in the paper
    pop = np.array([bin(c).count("1") for c in range(n)])
    want = H * ((-1.0) ** pop)[None, :]  # H_2 = G(pi/4) diag(1,-1) => B = H_n diag((-1)^popcount)
    assert np.allclose(B, want, atol=5e-7)  # float32(pi/4) is not exactly pi/4
    mu = np.abs(B).max()
    assert abs(mu - 1 / math.sqrt(n)) < 1e-6
    if n == 64:
        consts = _read_constants(golden_dir)
        assert consts["welch_n4096"] == 1 / math.sqrt(4096)


# --- P4: one angle per layer => Kronecker product of 2x2 rotations ---------------------------

@pytest.mark.parametrize("n", [4, 8, 32])
def test_layerwise_uniform_angles_give_kronecker_product(n):
    rng = np.random.default_rng(100 + n)
    k = n.bit_length() - 1
    phi = rng.uniform(-3, 3, size=k).astype(np.float32)
    th = np.repeat(phi[None, :, None], n // 2, axis=2).astype(np.float32)

    def G(t):
        t = float(t)
        return np.array([[math.cos(t), -math.sin(t)], [math.sin(t), math.cos(t)]])

    K = np.eye(1)
    for i in range(k):  # layer i+1 acts on bit i; the highest bit is the leftmost Kronecker factor
        K = np.kron(G(phi[i]), K)
    B = oracle.forward(np.eye(n), th, n).T
    assert np.allclose(B, K, atol=1e-14)


# --- P5: invariants --------------------------------------------------------------------------

@pytest.mark.parametrize("n,heads", [(8, 1), (64, 1), (128, 3), (1024, 1)])
def test_orthogonality_norm_and_roundtrip(n, heads):
    rng = np.random.default_rng(n + heads)
    th = _theta(rng, n, heads)
    x = rng.standard_normal((9, n * heads))
    y = oracle.forward(x, th, n, heads)
    xb = x.reshape(9, heads, n)
    yb = y.reshape(9, heads, n)
    assert np.allclose(np.linalg.norm(yb, axis=2), np.linalg.norm(xb, axis=2), rtol=1e-13)
    assert np.allclose(oracle.inverse(y, th, n, heads), x, atol=1e-13)
    if n <= 128:
        for h in range(heads):
            B = oracle.forward(np.eye(n * heads)[h * n:(h + 1) * n], th, n, heads)[:, h * n:(h + 1) * n].T
            assert np.allclose(B.T @ B, np.eye(n), atol=1e-13)
            # each layer has exactly 2n non-zeros
            for i in range(1, n.bit_length()):
                assert np.count_nonzero(dense_layer(th[h, i - 1], n, i)) == 2 * n


def test_zero_angles_are_identity_bit_exact():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 256))
    th = np.zeros((1, 8, 128), np.float32)
    assert np.array_equal(oracle.forward(x, th, 256), x)
    assert np.array_equal(oracle.inverse(x, th, 256), x)


def test_heads_are_block_diagonal():
    rng = np.random.default_rng(8)
    n, heads = 16, 4
    th = _theta(rng, n, heads)
    x = rng.standard_normal((3, n * heads))
    y = oracle.forward(x, th, n, heads)
    for h in range(heads):
        assert np.array_equal(y[:, h * n:(h + 1) * n], oracle.forward(x[:, h * n:(h + 1) * n], th[h:h + 1], n))


# --- P6: parameter / flop counts -------------------------------------------------------------

def test_parameter_counts(golden_dir):
    consts = _read_constants(golden_dir)

    def angles(n):
        return n * (n.bit_length() - 1) // 2

    assert angles(128) == consts["angles_n128"]
    assert angles(4096) == consts["angles_n4096"]
    assert 3 * 4096 * 12 == consts["flops_butterfly_n4096"]
    assert consts["adds_n4096"] + consts["mults_n4096"] == consts["flops_butterfly_n4096"]
    assert 40 * 39 // 2 + angles(128) == consts["composite_params_5120"]
    for n in (2, 8, 128):
        k = n.bit_length() - 1
        assert sum(len(pair_indices(n, i)) for i in range(1, k + 1)) == angles(n)
