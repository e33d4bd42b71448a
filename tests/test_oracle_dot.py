"""Pins for Part D of the CPU oracle (dual-PoT inner product, Eq. 4): dense fp64 matmul of
an independently dequantised matrix, exact integer partials, textbook reductions.  No GPU."""
import os

import numpy as np
import pytest

import goq_inputs
from tests import bruteforce as bf


def _quantized(oracle, bw, out, inn, cid):
    W = goq_inputs.weights(out, inn, config_id=cid, tensor_id=bw)
    return oracle.quantize_geo(bw, W, threads=2)


@pytest.mark.parametrize("bw", [3, 4])
def test_dequant_matches_independent_reconstruction(oracle, bw):
    q = _quantized(oracle, bw, 5, 256, 11)
    d = oracle.dequant(q)
    b1, b2 = bf.bases(q)
    assert np.array_equal(d["b1"], b1) and np.array_equal(d["b2"], b2)
    assert np.array_equal(d["what"], bf.dequant(q))


@pytest.mark.parametrize("bw", [3, 4])
def test_a16_equals_dense_matmul_of_dequantised_matrix(oracle, bw):
    q = _quantized(oracle, bw, 17, 384, 12)
    x = goq_inputs.activations_a16(3, 384, config_id=12, tensor_id=100, outlier_frac=0.01)
    y = oracle.gemm_a16(q, x)
    ref = x.astype(np.float64) @ bf.dequant(q).T
    scale = np.abs(x.astype(np.float64)) @ np.abs(bf.dequant(q)).T
    assert np.max(np.abs(y - ref) / scale) < 1e-14
    # threads do not change the result (rows are independent)
    assert np.array_equal(y, oracle.gemm_a16(q, x, threads=4))


def test_a16_pairwise_form_of_the_residual_dot(oracle):
    # x.b2 = sum over pairs eta * (x_j b1_i - x_i b1_j): b2 never needs to be stored
    q = _quantized(oracle, 3, 4, 128, 13)
    x = goq_inputs.activations_a16(1, 128, config_id=13)[0].astype(np.float64)
    b1, b2 = bf.bases(q)
    for o in range(4):
        tot = 0.0
        for m in range(16):
            s = int(q["pattern"][o, m]) + 1
            for p, (i, j) in enumerate(bf.PAIRS[s]):
                eta = -1.0 if (q["signs"][o, m] >> p) & 1 else 1.0
                tot += eta * (x[8 * m + j] * b1[o, 8 * m + i] - x[8 * m + i] * b1[o, 8 * m + j])
        assert np.isclose(tot, x @ b2[o], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("bw", [3, 4])
def test_a8_partials_are_exact_integers_and_output_matches(oracle, bw):
    q = _quantized(oracle, bw, 9, 256, 14)
    xq, sx = goq_inputs.activations_a8(5, 256, config_id=14)
    y, parts = oracle.gemm_a8(q, xq, sx, want_partials=True)
    b1, b2 = bf.bases(q)
    scale = 2 ** ((1 << (bw - 1)) - 1)
    i1 = (b1 * scale).astype(np.int64)
    i2 = (b2 * scale).astype(np.int64)
    assert np.array_equal(i1 / scale, b1) and np.array_equal(i2 / scale, b2)
    X = xq.astype(np.int64)
    for g in range(2):
        sl = slice(128 * g, 128 * g + 128)
        assert np.array_equal(parts[:, :, g, 0], X[:, sl] @ i1[:, sl].T)
        assert np.array_equal(parts[:, :, g, 1], X[:, sl] @ i2[:, sl].T)
    ref = (xq.astype(np.float64) * sx[:, None].astype(np.float64)) @ bf.dequant(q).T
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_a8_saturating_inputs_fit_int32(oracle):
    # every lane at +-127 against the largest magnitudes: |P| <= 127 * 2^(E-1) * 128
    for bw, bound in ((3, 127 * 8 * 128), (4, 127 * 128 * 128)):
        q = goq_inputs.canonical_random(bw, 2, 128, config_id=15)
        q["codes"][0, :] = 0                                  # all +1
        q["codes"][1, :] = 1 << (bw - 1)                      # all -1
        x = np.full((1, 128), 127, np.int8)
        y, parts = oracle.gemm_a8(q, x, np.ones(1, np.float32), want_partials=True)
        assert parts[0, 0, 0, 0] == bound and parts[0, 1, 0, 0] == -bound
        assert abs(int(parts[0, 0, 0, 1])) <= bound


def test_single_basis_and_rowsum_reductions(oracle):
    q = goq_inputs.canonical_random(3, 6, 256, config_id=16)
    x = goq_inputs.activations_a16(2, 256, config_id=16)
    # c2 = 0 -> plain K=1 PoT layer
    q1 = dict(q)
    q1["c2"] = np.zeros_like(q["c2"])
    L = bf.LATTICE_W3
    c1 = q["c1"].view(np.float16).astype(np.float64)
    ref = x.astype(np.float64) @ (np.repeat(c1, 128, axis=1) * L[q["codes"]]).T
    assert np.allclose(oracle.gemm_a16(q1, x), ref, rtol=1e-13, atol=1e-13)
    # all codes +1, c1 = 1, c2 = 0 -> row sum of x
    q2 = dict(q1)
    q2["codes"] = np.zeros_like(q["codes"])
    q2["c1"] = np.full_like(q["c1"], np.float16(1.0).view(np.uint16))
    y = oracle.gemm_a16(q2, x)
    assert np.allclose(y, np.repeat(x.astype(np.float64).sum(1)[:, None], 6, 1), rtol=1e-13)


def test_worked_example_dot(oracle):
    g = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "worked_example_w3.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            g[k] = np.array([float(t) for t in v])
    codes = np.full((1, 128), 3, np.uint8)
    codes[0, :8] = g["codes"]
    pat = np.zeros((1, 16), np.uint8)
    pat[0, 0] = int(g["s_star"][0]) - 1
    one = np.float16(1.0).view(np.uint16)
    x = np.zeros((1, 128))
    x[0, :8] = g["x"]
    for c1, c2, want in ((one, 0, g["x_b1"][0]), (0, one, g["x_b2"][0])):
        q = {"bw": 3, "codes": codes, "pattern": pat, "signs": np.zeros((1, 16), np.uint8),
             "c1": np.full((1, 1), c1, np.uint16), "c2": np.full((1, 1), c2, np.uint16)}
        assert oracle.gemm_a16(q, x.astype(np.float16))[0, 0] == want
    q["c1"][:] = one
    _, parts = oracle.gemm_a8(q, x.astype(np.int8), np.ones(1, np.float32), want_partials=True)
    assert parts[0, 0, 0].tolist() == [int(g["P1_int"][0]), int(g["P2_int"][0])]


def test_planted_mistakes_are_caught(oracle):
    """The pins above must fail for plausible mistakes: check on a perturbed copy that the
    independent reconstruction really disagrees (guards against vacuous comparisons)."""
    q = _quantized(oracle, 3, 3, 128, 17)
    base = bf.dequant(q)
    q_bad = dict(q)
    q_bad["signs"] = q["signs"] ^ 1
    assert not np.array_equal(bf.dequant(q_bad), base)
    q_bad = dict(q)
    q_bad["pattern"] = (q["pattern"] + 1) % 4
    assert not np.array_equal(bf.dequant(q_bad), base)
    x = goq_inputs.activations_a16(1, 128, config_id=17)
    assert not np.allclose(oracle.gemm_a16(q_bad, x), oracle.gemm_a16(q, x))
