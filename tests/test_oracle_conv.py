"""Pins for the oracle's convolution loops (CPU only).

Each test checks the C loops against something that is not the loops
themselves: hand-enumerated values, a library routine on a special case, a
closed form, or an algebraic identity that a dropped term, wrong sign, wrong
index or transposed operand would break.
"""
import os

import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import nature_cnn as orc


def _read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([float(v) for v in vals])
    return out


def test_hand_enumerated_5x5(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "conv_5x5_k3.txt"))
    x = (np.arange(25, dtype=np.float64) + 1).reshape(1, 1, 5, 5)
    W = (np.arange(9, dtype=np.float64) + 1).reshape(1, 1, 3, 3)
    np.testing.assert_array_equal(orc.conv2d(x, W, None, 1).reshape(-1), g["stride1"])
    np.testing.assert_array_equal(orc.conv2d(x, W, None, 2).reshape(-1), g["stride2"])


def test_output_size_rule_paper_geometry():
    # appendix "Atari Frame Processing": 104x80 frames, conv2/conv3 padded by 1,
    # feature map "always 12x9"
    assert orc.out_size(104, 8, 4, 0) == 25 and orc.out_size(80, 8, 4, 0) == 19
    assert orc.out_size(25, 4, 2, 1) == 12 and orc.out_size(19, 4, 2, 1) == 9
    assert orc.out_size(12, 3, 1, 1) == 12 and orc.out_size(9, 3, 1, 1) == 9
    assert orc.PAPER_104x80.feature_shape() == (64, 12, 9)
    # the 84x84 network of this build: 20 -> 9 -> 7, 64*7*7 = 3136
    assert orc.NATURE_84.feature_shape() == (64, 7, 7)


@pytest.mark.parametrize("k,s,pad", [(3, 1, 0), (4, 2, 0), (8, 4, 0), (3, 1, 1), (4, 2, 1)])
def test_against_scipy_correlate(k, s, pad):
    """Multi-channel conv = sum over channels of scipy's 2-D correlation, strided."""
    r = np.random.default_rng(7)
    N, Cin, H, Wd, Cout = 2, 3, 13, 11, 4
    x = r.standard_normal((N, Cin, H, Wd))
    W = r.standard_normal((Cout, Cin, k, k))
    b = r.standard_normal(Cout)
    got = orc.conv2d(x, W, b, s, pad)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    for n in range(N):
        for co in range(Cout):
            full = sum(correlate2d(xp[n, ci], W[co, ci], mode="valid") for ci in range(Cin)) + b[co]
            np.testing.assert_allclose(got[n, co], full[::s, ::s], rtol=0, atol=1e-12)


def test_identity_kernel_is_strided_crop():
    r = np.random.default_rng(3)
    C, k, s = 5, 3, 2
    x = r.standard_normal((2, C, 9, 12))
    W = np.zeros((C, C, k, k))
    for c in range(C):
        W[c, c, 1, 2] = 1.0                  # tap (ky=1, kx=2): distinguishes row from column
    got = orc.conv2d(x, W, None, s)
    OH, OW = got.shape[2:]
    want = x[:, :, 1:1 + s * OH:s, 2:2 + s * OW:s]
    np.testing.assert_array_equal(got, want)


def test_all_ones_kernel_is_box_sum():
    r = np.random.default_rng(4)
    x = r.integers(0, 256, size=(1, 2, 20, 17)).astype(np.float64)
    k, s = 4, 2
    W = np.ones((1, 2, k, k))
    got = orc.conv2d(x, W, None, s)[0, 0]
    sat = np.zeros((21, 18))
    sat[1:, 1:] = x[0].sum(axis=0).cumsum(axis=0).cumsum(axis=1)      # summed-area table
    for oy in range(got.shape[0]):
        for ox in range(got.shape[1]):
            y0, x0 = oy * s, ox * s
            box = sat[y0 + k, x0 + k] - sat[y0, x0 + k] - sat[y0 + k, x0] + sat[y0, x0]
            assert got[oy, ox] == box


def test_linearity_in_x_and_w():
    r = np.random.default_rng(5)
    x1, x2 = r.standard_normal((2, 2, 3, 10, 10))
    W1, W2 = r.standard_normal((2, 4, 3, 3, 3))
    a, b = 0.7, -1.3
    lhs = orc.conv2d(a * x1 + b * x2, W1, None, 1)
    np.testing.assert_allclose(lhs, a * orc.conv2d(x1, W1, None, 1) + b * orc.conv2d(x2, W1, None, 1), atol=1e-12)
    lhs = orc.conv2d(x1, a * W1 + b * W2, None, 1)
    np.testing.assert_allclose(lhs, a * orc.conv2d(x1, W1, None, 1) + b * orc.conv2d(x1, W2, None, 1), atol=1e-12)


@pytest.mark.parametrize("k,s,pad", [(8, 4, 0), (4, 2, 0), (3, 1, 0), (4, 2, 1), (3, 1, 1)])
def test_adjoint_identities(k, s, pad):
    """conv is bilinear, so <dy, conv(x,W)> = <dx(dy), x> = <dW(dy), W>; db = sum dy."""
    r = np.random.default_rng(11)
    N, Cin, Cout = 3, 3, 5
    H, Wd = 8 * s + k, 7 * s + k + 1
    x = r.standard_normal((N, Cin, H, Wd))
    W = r.standard_normal((Cout, Cin, k, k))
    y = orc.conv2d(x, W, None, s, pad)
    dy = r.standard_normal(y.shape)
    dx = orc.conv2d_input_grad(x.shape, W, dy, s, pad)
    dW, db = orc.conv2d_weight_grad(x, dy, k, s, pad)
    ref = float((dy * y).sum())
    assert abs(float((dx * x).sum()) - ref) < 1e-9 * max(1.0, abs(ref))
    assert abs(float((dW * W).sum()) - ref) < 1e-9 * max(1.0, abs(ref))
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), atol=1e-10)


def test_input_and_weight_grad_single_tap_brute_force():
    """One output element switched on: its gradients are the window and the kernel."""
    r = np.random.default_rng(12)
    x = r.standard_normal((1, 2, 9, 9))
    W = r.standard_normal((3, 2, 4, 4))
    s = 2
    dy = np.zeros((1, 3, 3, 3))
    dy[0, 1, 2, 1] = 1.0
    dx = orc.conv2d_input_grad(x.shape, W, dy, s)
    want = np.zeros_like(x)
    want[0, :, 4:8, 2:6] = W[1]
    np.testing.assert_array_equal(dx, want)
    dW, db = orc.conv2d_weight_grad(x, dy, 4, s)
    wantW = np.zeros_like(W)
    wantW[1] = x[0, :, 4:8, 2:6]
    np.testing.assert_array_equal(dW, wantW)
    np.testing.assert_array_equal(db, [0.0, 1.0, 0.0])


def test_weight_grad_independent_of_grouping():
    """Sum over samples is the sum of per-sample gradients (more samples than one group)."""
    r = np.random.default_rng(13)
    N = 70
    x = r.standard_normal((N, 2, 6, 6))
    dy = r.standard_normal((N, 3, 4, 4))
    dW, db = orc.conv2d_weight_grad(x, dy, 3, 1)
    acc = np.zeros_like(dW)
    for n in range(N):
        acc += orc.conv2d_weight_grad(x[n:n + 1], dy[n:n + 1], 3, 1)[0]
    np.testing.assert_allclose(dW, acc, atol=1e-11)
