"""Pins for oracle/direct.py and oracle/winograd.py (unquantised paths)."""
from fractions import Fraction

import numpy as np
import pytest
from scipy.signal import correlate2d

import synth_inputs as si
from oracle import direct, matrices as mx, winograd as wg


def test_direct_vectorised_equals_loops_and_scipy():
    rng = np.random.default_rng(5)
    x = rng.integers(-127, 128, size=(2, 5, 6, 3))
    w = rng.integers(-127, 128, size=(4, 3, 3, 3))
    y = direct.direct_conv(x, w, dtype=np.int64)
    loops = np.array(direct.direct_conv_loops(x.tolist(), w.tolist()))
    assert np.array_equal(y, loops)
    # textbook library routine: 'same' cross-correlation with zero fill
    for b in range(2):
        for k in range(4):
            acc = np.zeros((5, 6), dtype=np.int64)
            for c in range(3):
                acc += correlate2d(x[b, :, :, c], w[k, c], mode="same", boundary="fill")
            assert np.array_equal(acc, y[b, :, :, k])


def test_direct_conv_fraction_tiny():
    rng = np.random.default_rng(6)
    x = rng.integers(-5, 6, size=(1, 3, 3, 2))
    w = rng.integers(-5, 6, size=(2, 2, 3, 3))
    yf = direct.direct_conv_loops(direct.to_fraction_nested(x), direct.to_fraction_nested(w),
                                  zero=Fraction(0))
    yi = direct.direct_conv(x, w, dtype=np.int64)
    assert np.array_equal(np.array([[[[int(v) for v in a] for a in b] for b in c] for c in yf]), yi)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_unquantised_winograd_equals_direct_fp64(m):
    """eq. 3 and eq. 4 against the definition, rel err <= 1e-10, cfg1-sized input."""
    x, w = si.make_real(1, 8, 8, 16, 16, seed=0)
    M = mx.Matrices(m, 3)
    yd = direct.direct_conv(x, w)
    scale = np.abs(yd).max()
    assert np.abs(wg.conv_eq3(x, w, M) - yd).max() <= 1e-10 * scale
    assert np.abs(wg.conv_eq4(x, w, M) - yd).max() <= 1e-10 * scale


@pytest.mark.parametrize("m,H,W", [(4, 7, 9), (6, 8, 8), (6, 4, 4), (2, 5, 3), (4, 1, 1)])
def test_ragged_sizes(m, H, W):
    """H, W not multiples of m: zero-extend bottom/right, compute full tiles, crop."""
    x, w = si.make_real(2, H, W, 3, 5, seed=11)
    M = mx.Matrices(m, 3)
    yd = direct.direct_conv(x, w)
    y3 = wg.conv_eq3(x, w, M)
    assert y3.shape == yd.shape
    assert np.abs(y3 - yd).max() <= 1e-10 * np.abs(yd).max()
    assert np.abs(wg.conv_eq4(x, w, M) - yd).max() <= 1e-9 * np.abs(yd).max()


def test_tile_order_and_padding():
    x = np.arange(1 * 8 * 8 * 1).reshape(1, 8, 8, 1) + 1
    d = wg.extract_tiles(x, 4, 3)
    assert d.shape == (4, 6, 6, 1)
    # tile 0: first row and column are the zero pad, then x[0:5, 0:5]
    assert np.all(d[0, 0, :, 0] == 0) and np.all(d[0, :, 0, 0] == 0)
    assert np.array_equal(d[0, 1:, 1:, 0], x[0, 0:5, 0:5, 0])
    # tile 1 is (ty=0, tx=1): columns 3..8 of the image, last one is the right pad
    assert np.array_equal(d[1, 1:, :5, 0], x[0, 0:5, 3:8, 0])
    assert np.all(d[1, :, 5, 0] == 0)
    # tile 2 is (ty=1, tx=0)
    assert np.array_equal(d[2, :5, 1:, 0], x[0, 3:8, 0:5, 0])
    Y = np.arange(4 * 4 * 4 * 1).reshape(4, 4, 4, 1)
    y = wg.scatter_tiles(Y, 1, 8, 8, 4)
    assert np.array_equal(y[0, 0:4, 4:8, 0], Y[1, :, :, 0])
    assert np.array_equal(y[0, 4:8, 0:4, 0], Y[2, :, :, 0])
