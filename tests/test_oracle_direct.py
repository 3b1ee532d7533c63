"""Pins for the direct-convolution oracle (the plain definition of the result).

It is checked against things other than itself: a brute-force Python loop, a
library convolution in float64 (exact at these magnitudes), impulse responses
that fix orientation and index order, and a closed form.
"""
import itertools

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import direct_conv2d, requant_shift_clamp, maxpool2x2


def brute(x, w, pad):
    N, C, H, W = x.shape
    K, _, r, _ = w.shape
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    y = np.zeros((N, K, Ho, Wo), dtype=object)
    for n, k, oy, ox in itertools.product(range(N), range(K), range(Ho), range(Wo)):
        acc = 0
        for c, i, j in itertools.product(range(C), range(r), range(r)):
            iy, ix = oy + i - pad, ox + j - pad
            if 0 <= iy < H and 0 <= ix < W:
                acc += int(x[n, c, iy, ix]) * int(w[k, c, i, j])
        y[n, k, oy, ox] = acc
    return y.astype(np.int64)


@pytest.mark.parametrize("shape", [(1, 2, 3, 5, 5, 3, 1), (2, 3, 2, 7, 6, 5, 2), (1, 1, 1, 4, 6, 3, 0),
                                   (1, 2, 2, 3, 3, 3, 1), (1, 1, 2, 5, 5, 5, 0)])
def test_matches_brute_force(shape):
    N, C, K, H, W, r, pad = shape
    x = si.int8_tensor(11, (N, C, H, W))
    w = si.int8_tensor(12, (K, C, r, r))
    assert np.array_equal(direct_conv2d(x, w, pad).astype(np.int64), brute(x, w, pad))


@pytest.mark.parametrize("shape", [(2, 5, 4, 13, 17, 3, 1), (1, 8, 6, 12, 12, 5, 2), (1, 3, 3, 9, 9, 3, 0)])
def test_matches_library_conv_float64(shape):
    N, C, K, H, W, r, pad = shape
    x = si.int8_tensor(21, (N, C, H, W))
    w = si.int8_tensor(22, (K, C, r, r))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), padding=pad)
    assert np.array_equal(direct_conv2d(x, w, pad).astype(np.float64), ref.numpy())


def test_impulse_filter_copies_a_shifted_channel():
    # w[k,c,i,j] one-hot => y[k] = x[c] shifted by (i-pad, j-pad): fixes correlation orientation
    x = si.int8_tensor(31, (1, 3, 6, 7))
    w = np.zeros((2, 3, 3, 3), dtype=np.int8)
    w[1, 2, 0, 2] = 1       # output channel 1 <- input channel 2, tap (row 0, col 2)
    y = direct_conv2d(x, w, pad=1)
    assert not y[0, 0].any()
    for oy in range(6):
        for ox in range(7):
            iy, ix = oy + 0 - 1, ox + 2 - 1
            expect = int(x[0, 2, iy, ix]) if 0 <= iy < 6 and 0 <= ix < 7 else 0
            assert y[0, 1, oy, ox] == expect


def test_impulse_input_prints_the_flipped_filter():
    x = np.zeros((1, 1, 5, 5), dtype=np.int8)
    x[0, 0, 2, 2] = 1
    w = si.int8_tensor(32, (1, 1, 3, 3))
    y = direct_conv2d(x, w, pad=1)
    # y[oy,ox] = w[2-oy+... ]: the tap that lands on the impulse is (i,j) = (2-oy+1-... ) written out:
    for oy in range(5):
        for ox in range(5):
            i, j = 2 - oy + 1, 2 - ox + 1
            expect = int(w[0, 0, i, j]) if 0 <= i < 3 and 0 <= j < 3 else 0
            assert y[0, 0, oy, ox] == expect


def test_all_minus_128_closed_form():
    C, r = 5, 3
    x = np.full((1, C, 6, 6), -128, dtype=np.int8)
    w = np.full((2, C, r, r), -128, dtype=np.int8)
    y = direct_conv2d(x, w, pad=1)
    assert (y[:, :, 1:-1, 1:-1] == (1 << 14) * r * r * C).all()
    assert y[0, 0, 0, 0] == (1 << 14) * 4 * C            # corner sees a 2x2 window
    assert y[0, 0, 0, 2] == (1 << 14) * 6 * C            # edge sees 2x3


def test_requant_is_floor_shift_and_clamp():
    y = np.array([0, 1, -1, 511, 512, -512, -513, 1 << 20, -(1 << 20), 127 * 512 + 511, -128 * 512], dtype=np.int32)
    a = requant_shift_clamp(y, 9)
    assert a.tolist() == [0, 0, -1, 0, 1, -1, -2, 127, -128, 127, -128]
    rnd = (si.int8_tensor(5, (1000,)).astype(np.int32)) * 777
    assert np.array_equal(requant_shift_clamp(rnd, 6), np.clip(np.floor(rnd / 64.0), -128, 127).astype(np.int8))
    # the ends of the shift range: shift 0 only clamps; shift 31 leaves the sign (floor(y / 2^31) is -1 or 0)
    edge = np.array([-2 ** 31, -2 ** 31 + 1, -129, -128, -1, 0, 1, 127, 128, 2 ** 31 - 1], dtype=np.int32)
    assert requant_shift_clamp(edge, 0).tolist() == [-128, -128, -128, -128, -1, 0, 1, 127, 127, 127]
    assert requant_shift_clamp(edge, 31).tolist() == [-1, -1, -1, -1, -1, 0, 0, 0, 0, 0]
    assert requant_shift_clamp(edge, 30).tolist() == [-2, -2, -1, -1, -1, 0, 0, 0, 0, 1]


def test_maxpool():
    a = si.int8_tensor(6, (2, 3, 4, 6))
    b = maxpool2x2(a)
    ref = a.reshape(2, 3, 2, 2, 3, 2).max(axis=(3, 5))
    assert np.array_equal(b, ref)
