"""Pins for Part R of the CPU oracle (REF mode, Sec. 3.4, Eq. 3: ridge regression of the two block
coefficients on calibration inputs).  Each pin is something other than the oracle's own formula:
a generic least-squares routine on the ridge-augmented system, the closed form the method has for
identity inputs (which ties REF to the GEO coefficients of Eq. 2), exact recovery of weights in
the span of the bases, the limit of a large ridge.  No GPU."""
import numpy as np
import pytest

import goq_inputs
from tests import bruteforce as bf


def _setup(oracle, bw, out, inn, tokens, cid):
    W = goq_inputs.weights(out, inn, config_id=cid, tensor_id=bw)
    q = oracle.quantize_geo(bw, W, threads=2)
    X = goq_inputs.activations_a16(tokens, inn, config_id=cid, tensor_id=100, outlier_frac=0.01)
    return W, q, X


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("lam", [1e-4, 0.5])
def test_ref_equals_generic_least_squares_on_the_augmented_system(oracle, bw, lam):
    """min ||A c - Y||^2 + lam ||c||^2 is the ordinary least-squares problem [A; sqrt(lam) I] c = [Y; 0]:
    numpy's SVD-based lstsq solves it without forming the normal equations."""
    out, inn, tokens = 6, 256, 50
    W, q, X = _setup(oracle, bw, out, inn, tokens, 21)
    _, c = oracle.ref_coefficients(q, W, X, lam=lam)
    b1, b2 = bf.bases(q)
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    for o in range(out):
        for g in range(inn // 128):
            sl = slice(128 * g, 128 * g + 128)
            A = np.stack([Xd[:, sl] @ b1[o, sl], Xd[:, sl] @ b2[o, sl]], axis=1)
            Y = Xd[:, sl] @ Wd[o, sl]
            Aa = np.vstack([A, np.sqrt(lam) * np.eye(2)])
            Ya = np.concatenate([Y, np.zeros(2)])
            ref = np.linalg.lstsq(Aa, Ya, rcond=None)[0]
            assert np.allclose(c[o, g], ref, rtol=1e-9, atol=1e-12), (o, g, c[o, g], ref)


@pytest.mark.parametrize("bw", [3, 4])
def test_identity_inputs_give_the_geo_coefficients(oracle, bw):
    """With X_q = I the responses are the bases themselves and Y = w; b1 and b2 are orthogonal
    (Theorem 1), so c_m = <w, b_m> / (||b_m||^2 + lam): Eq. 2 with the ridge in the denominator, and
    with lam = 0 the very coefficients the GEO quantizer stores."""
    out, inn = 9, 128
    W = goq_inputs.weights(out, inn, config_id=22, tensor_id=bw)
    q = oracle.quantize_geo(bw, W)
    X = np.eye(128, dtype=np.float16)
    b1, b2 = bf.bases(q)
    Wd = W.astype(np.float64)
    for lam in (0.0, 1e-4, 3.0):
        r, c = oracle.ref_coefficients(q, W, X, lam=lam)
        ref1 = np.sum(Wd * b1, axis=1) / (np.sum(b1 * b1, axis=1) + lam)
        ref2 = np.sum(Wd * b2, axis=1) / (np.sum(b2 * b2, axis=1) + lam)
        assert np.allclose(c[:, 0, 0], ref1, rtol=1e-12, atol=0) and np.allclose(c[:, 0, 1], ref2, rtol=1e-12, atol=1e-300)
        if lam == 0.0:
            assert np.array_equal(r["c1"], q["c1"]) and np.array_equal(r["c2"], q["c2"])


def test_weights_in_the_span_are_recovered_exactly(oracle):
    """If w = a b1 + b b2 then Y = A [a, b]^T for any inputs, and without a ridge the solution is
    (a, b) whatever the calibration inputs are.  A swapped right-hand side, a transposed Gram
    matrix or a wrong sign in the 2 x 2 inverse all break this."""
    bw, out, inn, tokens = 3, 7, 256, 40
    _, q, X = _setup(oracle, bw, out, inn, tokens, 23)
    b1, b2 = bf.bases(q)
    a, b = 0.5, -0.25                                        # powers of two: w stays fp16-representable
    W = (a * b1 + b * b2).astype(np.float16)
    assert np.array_equal(W.astype(np.float64), a * b1 + b * b2)
    r, c = oracle.ref_coefficients(q, W, X, lam=0.0)
    assert np.allclose(c[..., 0], a, rtol=1e-10) and np.allclose(c[..., 1], b, rtol=1e-10)
    assert np.all(r["c1"] == np.float16(a).view(np.uint16)) and np.all(r["c2"] == np.float16(b).view(np.uint16))


def test_ridge_shrinks_and_threads_do_not_matter(oracle):
    bw, out, inn, tokens = 4, 5, 128, 30
    W, q, X = _setup(oracle, bw, out, inn, tokens, 24)
    norms = []
    for lam in (0.0, 1e-4, 1.0, 1e3, 1e9):
        _, c = oracle.ref_coefficients(q, W, X, lam=lam)
        norms.append(np.linalg.norm(c, axis=2))
    for lo, hi in zip(norms[1:], norms[:-1]):
        assert np.all(lo <= hi * (1 + 1e-12))
    assert np.all(norms[-1] < 1e-6)
    _, c1 = oracle.ref_coefficients(q, W, X, lam=1e-4, threads=1)
    _, c4 = oracle.ref_coefficients(q, W, X, lam=1e-4, threads=4)
    assert np.array_equal(c1, c4)


def test_ref_does_not_increase_the_calibration_error(oracle):
    """On its own calibration inputs the refined pair cannot fit the slab outputs worse than the GEO
    pair (it minimises that error, up to the tiny ridge)."""
    bw, out, inn, tokens = 3, 8, 256, 64
    W, q, X = _setup(oracle, bw, out, inn, tokens, 25)
    _, c = oracle.ref_coefficients(q, W, X, lam=1e-4)
    b1, b2 = bf.bases(q)
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    cg = np.stack([goq_inputs_half(q["c1"]), goq_inputs_half(q["c2"])], axis=2)
    for o in range(out):
        for g in range(inn // 128):
            sl = slice(128 * g, 128 * g + 128)
            A = np.stack([Xd[:, sl] @ b1[o, sl], Xd[:, sl] @ b2[o, sl]], axis=1)
            Y = Xd[:, sl] @ Wd[o, sl]
            e_ref = np.sum((A @ c[o, g] - Y) ** 2) + 1e-4 * np.sum(c[o, g] ** 2)
            e_geo = np.sum((A @ cg[o, g] - Y) ** 2) + 1e-4 * np.sum(cg[o, g] ** 2)
            assert e_ref <= e_geo * (1 + 1e-9)


def goq_inputs_half(bits):
    return bits.view(np.float16).astype(np.float64)
