"""Pins for Part Q of the CPU oracle (GEO quantizer): printed constants, Theorem 1,
brute force over the lattice and over the 64 exchange candidates, generic least squares,
the worked example.  No GPU."""
import itertools
import os

import numpy as np
import pytest

import goq_inputs
from tests import bruteforce as bf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example_w3.txt")


def _golden():
    d = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        d[k] = np.array([float(t) for t in v])
    return d


def test_lattice_w3_is_the_printed_set(oracle):
    # Sec. 3.2 prints L_3bit = {-1,-0.5,-0.25,-0.125,0,+0.25,+0.5,+1}
    L = oracle.lattice(3)
    assert sorted(L.tolist()) == [-1.0, -0.5, -0.25, -0.125, 0.0, 0.25, 0.5, 1.0]
    assert np.array_equal(L, bf.LATTICE_W3)


def test_lattice_w4_reading(oracle):
    L = oracle.lattice(4)
    assert np.array_equal(L, bf.LATTICE_W4)
    assert len(set(L.tolist())) == 16 and 0.0 in L and 2.0 ** -7 not in L and -(2.0 ** -7) in L


def test_lattice_values_are_exact_pot(oracle):
    for bw in (3, 4):
        L = oracle.lattice(bw)
        scale = 2.0 ** ((1 << (bw - 1)) - 1)
        for v in L:
            assert v * scale == int(v * scale)
            if v != 0:
                m, e = np.frexp(abs(v))
                assert m == 0.5
            assert np.float16(v) == v


def test_exchange_matches_printed_pair_sets_and_theorem1(oracle):
    rng = np.random.default_rng(1)
    for bw in (3, 4):
        L = oracle.lattice(bw)
        for _ in range(50):
            x = rng.choice(L, size=8)
            for s, sg in itertools.product((1, 2, 3, 4), range(16)):
                y = oracle.exchange(x, s, sg)
                assert np.array_equal(y, bf.exchange(x, s, sg))
                assert float(x @ y) == 0.0                      # Theorem 1, exact
                assert float(y @ y) == float(x @ x)             # signed permutation
                # every coordinate is in exactly one pair: |y| is a permutation of |x| by i^s
                assert np.array_equal(np.abs(y), np.abs(x[np.arange(8) ^ s]))


def test_exchange_is_a_rotation_of_each_pair(oracle):
    # y_i = -eta x_j, y_j = +eta x_i with the pair order of the printed sets
    x = np.arange(1.0, 9.0)
    y = oracle.exchange(x, 2, 0b0101)      # pairs (0,2) eta=-1, (1,3) +1, (4,6) -1, (5,7) +1
    assert y.tolist() == [3.0, -4.0, -1.0, 2.0, 7.0, -8.0, -5.0, 6.0]


@pytest.mark.parametrize("bw", [3, 4])
def test_q_is_nearest_state_with_ties_toward_zero(oracle, bw):
    rng = np.random.default_rng(2)
    L = oracle.lattice(bw)
    w = rng.normal(0, 0.02, size=128).astype(np.float16).astype(np.float64)
    # plant exact ties: midpoints between neighbouring states, relative to s_norm = 1
    mids = np.sort(L)
    mids = (mids[1:] + mids[:-1]) / 2
    w[:len(mids)] = mids
    w[len(mids)] = 1.0                     # s_norm = 1 exactly
    w[len(mids) + 1] = -1.0
    codes, _, _, _, _ = oracle.quantize_block(bw, w)
    snorm = np.abs(w).max()
    for k in range(128):
        assert codes[k] == bf.nearest_code(bw, w[k] / snorm), k
    # zero always wins its ties; a tie never picks the larger magnitude
    for k in range(len(mids)):
        lo, hi = np.sort(L)[k], np.sort(L)[k + 1]
        assert abs(L[codes[k]]) == min(abs(lo), abs(hi))


@pytest.mark.parametrize("bw", [3, 4])
def test_block_against_bruteforce_and_invariants(oracle, bw):
    W = goq_inputs.weights(24, 256, config_id=7, tensor_id=bw).astype(np.float64)
    L = oracle.lattice(bw)
    for w in W.reshape(-1, 128):
        codes, pat, sg, c1, c2 = oracle.quantize_block(bw, w)
        b1 = L[codes]
        n1 = b1 @ b1
        assert n1 >= 1.0                                   # the max element maps to +-1
        assert np.all(w * b1 >= 0)                         # never an opposite-sign state
        r = w - (w @ b1) / n1 * b1
        assert abs(r @ b1) < 1e-15
        b2 = np.zeros(128)
        total_align = 0.0
        for m in range(16):
            x, rr = b1[8 * m:8 * m + 8], r[8 * m:8 * m + 8]
            a_best, s_best, sg_best = bf.best_exchange(x, rr)
            y = oracle.exchange(x, int(pat[m]) + 1, int(sg[m]))
            b2[8 * m:8 * m + 8] = y
            # the analytical choice reaches the exhaustive optimum of the candidate family
            assert abs(float(y @ rr) - a_best) <= 1e-15 * max(1.0, abs(a_best))
            total_align += a_best
        assert b1 @ b2 == 0.0 and b2 @ b2 == n1
        # GEO coefficients = generic least squares on [b1 b2]
        sol, *_ = np.linalg.lstsq(np.stack([b1, b2], 1), w, rcond=None)
        assert np.allclose([c1, c2], sol, rtol=1e-10, atol=1e-15)
        assert c1 > 0 and c2 >= 0
        assert np.isclose(w @ b2, total_align, rtol=1e-9, atol=1e-15)
        # Pythagoras: the second basis can only reduce the error
        e2 = np.sum((w - c1 * b1 - c2 * b2) ** 2)
        assert np.isclose(e2, w @ w - c1 * c1 * n1 - c2 * c2 * n1, rtol=1e-8, atol=1e-14)
        assert e2 <= np.sum((w - c1 * b1) ** 2) + 1e-18


def test_pattern_tie_goes_to_smallest_s_and_zero_cross_term_to_plus(oracle):
    # a block whose residual is zero everywhere: all scores tie at 0, all cross terms are 0
    w = np.zeros(128)
    w[:8] = [1, 0.5, 0.25, -0.125, -1, -0.5, -0.25, 0.25]      # exactly representable
    codes, pat, sg, c1, c2 = oracle.quantize_block(3, w)
    assert np.all(pat == 0) and np.all(sg == 0)
    assert c1 == 1.0 and c2 == 0.0


def test_all_zero_block(oracle):
    for bw in (3, 4):
        codes, pat, sg, c1, c2 = oracle.quantize_block(bw, np.zeros(128))
        assert np.all(oracle.lattice(bw)[codes] == 0.0)
        assert np.all(pat == 0) and np.all(sg == 0) and c1 == 0.0 and c2 == 0.0


def test_worked_example(oracle):
    g = _golden()
    w = np.zeros(128)
    w[:8] = g["w"]
    codes, pat, sg, c1, c2 = oracle.quantize_block(3, w)
    assert codes[:8].tolist() == g["codes"].astype(int).tolist()
    L = oracle.lattice(3)
    b1 = L[codes]
    assert b1[:8].tolist() == g["b1"].tolist() and np.all(b1[8:] == 0)
    assert pat[0] + 1 == int(g["s_star"][0]) and sg[0] == int(g["signs"][0])
    assert np.all(pat[1:] == 0) and np.all(sg[1:] == 0)
    assert np.isclose(c1, g["w_b1"][0] / g["b1_sq"][0], rtol=1e-14)
    assert np.isclose(c2, g["w_b2"][0] / g["b1_sq"][0], rtol=1e-12)
    y = oracle.exchange(b1[:8], pat[0] + 1, sg[0])
    assert y.tolist() == g["b2"].tolist()
    # the four scores, recomputed from the printed pair sets
    r = w[:8] - c1 * b1[:8]
    for s in (1, 2, 3, 4):
        A = sum(abs(b1[i] * r[j] - b1[j] * r[i]) for i, j in bf.PAIRS[s])
        assert np.isclose(A, g["A"][s - 1], rtol=1e-12)
    assert np.isclose(np.sum((w[:8] - c1 * b1[:8]) ** 2), g["err_k1"][0], rtol=1e-5)
    assert np.isclose(np.sum((w[:8] - c1 * b1[:8] - c2 * y) ** 2), g["err_k2"][0], rtol=1e-5)


def test_coefficients_are_rounded_to_fp16_nearest_even(oracle):
    rng = np.random.default_rng(3)
    xs = np.concatenate([rng.normal(0, 1, 2000), rng.normal(0, 1e-5, 2000), rng.normal(0, 3e4, 500),
                         [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25,
                          1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 6.1e-5, 6.09e-5]])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(x) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, ref)
    back = np.array([oracle.half_to_double(int(b)) for b in range(0, 0x7c00, 7)])
    assert np.array_equal(back, np.arange(0, 0x7c00, 7, dtype=np.uint16).view(np.float16).astype(np.float64))


def test_layer_quantizer_equals_blockwise_and_threads_agree(oracle):
    W = goq_inputs.weights(16, 384, config_id=9, tensor_id=0)
    q1 = oracle.quantize_geo(3, W, threads=1)
    q4 = oracle.quantize_geo(3, W, threads=4)
    for k in ("codes", "pattern", "signs", "c1", "c2"):
        assert np.array_equal(q1[k], q4[k])
    Wd = W.astype(np.float64)
    for o in (0, 7, 15):
        for g in range(3):
            codes, pat, sg, c1, c2 = oracle.quantize_block(3, Wd[o, 128 * g:128 * g + 128])
            assert np.array_equal(q1["codes"][o, 128 * g:128 * g + 128], codes)
            assert np.array_equal(q1["pattern"][o, 16 * g:16 * g + 16], pat)
            assert np.array_equal(q1["signs"][o, 16 * g:16 * g + 16], sg)
            assert q1["c1"][o, g] == np.float16(c1).view(np.uint16)
            assert q1["c2"][o, g] == np.float16(c2).view(np.uint16)


def test_statistics_on_the_workload_distribution(oracle):
    # smoke values for the synthetic weight distribution (not parity targets): two bases
    # beat one, and the four patterns are all used
    W = goq_inputs.weights(64, 4096, config_id=0, tensor_id=0)
    Wd = W.astype(np.float64)
    for bw, lo, hi in ((3, 0.15, 0.19), (4, 0.14, 0.17)):
        q = oracle.quantize_geo(bw, W, threads=4)
        d = oracle.dequant(q)
        c1 = q["c1"].view(np.float16).astype(np.float64)
        k1 = np.repeat(c1, 128, axis=1) * d["b1"]
        e1 = np.linalg.norm(Wd - k1) / np.linalg.norm(Wd)
        e2 = np.linalg.norm(Wd - d["what"]) / np.linalg.norm(Wd)
        assert e2 < e1 and lo < e2 < hi
        frac = np.bincount(q["pattern"].ravel(), minlength=4) / q["pattern"].size
        assert np.all(frac > 0.2) and np.all(frac < 0.3)
