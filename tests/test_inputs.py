"""The seeded input generators: determinism, shapes, dtypes, stated statistics.  No GPU."""
import numpy as np

import goq_inputs


def test_weights_are_seeded_fp16_with_heavy_tail():
    a = goq_inputs.weights(64, 1024, 0, 0)
    b = goq_inputs.weights(64, 1024, 0, 0)
    assert a.dtype == np.float16 and np.array_equal(a, b)
    assert not np.array_equal(a, goq_inputs.weights(64, 1024, 0, 1))
    assert 0.019 < a.astype(np.float64).std() < 0.022


def test_a16_outlier_channels():
    x = goq_inputs.activations_a16(256, 4096, 2, 100, outlier_frac=0.01).astype(np.float64)
    big = np.flatnonzero(x.std(axis=0) > 8)
    assert len(big) == 41


def test_a8_is_per_token_symmetric_int8():
    xq, sx = goq_inputs.activations_a8(16, 768, 4)
    assert xq.dtype == np.int8 and sx.dtype == np.float32 and sx.shape == (16,)
    assert np.all(np.abs(xq.astype(int)).max(axis=1) == 127) and xq.min() >= -127


def test_low_bit_activations_and_int4_packing():
    for bits in (3, 4, 6):
        xq, sx = goq_inputs.activations_int(8, 256, bits, 4)
        top = (1 << (bits - 1)) - 1
        assert xq.dtype == np.int8 and np.all(np.abs(xq.astype(int)).max(axis=1) == top)
    xq, _ = goq_inputs.activations_int(8, 256, 4, 4)
    xq[0, :4] = [-8, 7, -1, 0]
    p = goq_inputs.pack_int4(xq)
    assert p.shape == (8, 128) and p.dtype == np.uint8
    lo = (p & 0xF).astype(np.int8)
    hi = (p >> 4).astype(np.int8)
    lo[lo > 7] -= 16
    hi[hi > 7] -= 16
    assert np.array_equal(lo, xq[:, 0::2]) and np.array_equal(hi, xq[:, 1::2])
    assert p[0, 0] == 0x78 and p[0, 1] == 0x0F


def test_canonical_random_ranges():
    for bw in (3, 4):
        q = goq_inputs.canonical_random(bw, 8, 256, 5)
        assert q["codes"].max() < (1 << bw) and q["pattern"].max() <= 3 and q["signs"].max() <= 15
        assert q["codes"].shape == (8, 256) and q["pattern"].shape == (8, 32) and q["c1"].shape == (8, 2)
        assert q["c1"].dtype == np.uint16
