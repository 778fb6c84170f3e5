"""Pins for the oracle's patch expansion, factor build and running average.

Each check compares the oracle with something it does not itself compute:
element-by-element Python sums, closed forms, statistical limits, or a special
case that collapses to a differently-shaped computation.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from synth import shapes


def brute_rows(layer, a):
    """Definition of the patch matrix by explicit index loops (independent of the oracle's slicing)."""
    rows = []
    for n in range(layer.n):
        for oy in range(layer.oh):
            for ox in range(layer.ow):
                row = []
                for c in range(layer.c_in):
                    for i in range(layer.kh):
                        for j in range(layer.kw):
                            y = oy * layer.stride - layer.ph + i
                            x = ox * layer.stride - layer.pw + j
                            inside = 0 <= y < layer.h and 0 <= x < layer.w
                            row.append(float(a[n, c, y, x]) if inside else 0.0)
                if layer.has_bias:
                    row.append(1.0)
                rows.append(row)
    return rows


def brute_factor(rows):
    d = len(rows[0])
    F = [[0.0] * d for _ in range(d)]
    for r in rows:                       # sum over samples of the outer product r r^T
        for i in range(d):
            for j in range(d):
                F[i][j] += r[i] * r[j]
    R = len(rows)
    return np.array(F) / R


CONV_CASES = [(k, s, p, b) for k, s, p, b in itertools.product((1, 3), (1, 2), (0, 1), (0, 1))] + [(7, 2, 3, 1), (2, 1, 0, 1)]


@pytest.mark.parametrize("k,s,p,bias", CONV_CASES)
def test_conv_factor_matches_bruteforce(k, s, p, bias):
    rng = np.random.default_rng(10 * k + 3 * s + p)
    h, w = (9, 8) if k == 7 else (5, 6)
    layer = shapes.conv(2, 3, h, w, 4, k, s, p, bias)
    a = rng.standard_normal(layer.act_shape).astype(np.float32)
    rows = brute_rows(layer, a)
    got_rows = oracle.im2col_rows(layer, a)
    assert got_rows.shape == (layer.R, layer.dA)
    np.testing.assert_array_equal(got_rows, np.array(rows))            # exact: pure data movement
    np.testing.assert_allclose(oracle.factor_from_rows(got_rows), brute_factor(rows), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("kh,kw,ph,pw,s", [(1, 7, 0, 3, 1), (7, 1, 3, 0, 1), (1, 3, 0, 1, 1), (3, 1, 1, 0, 1), (3, 5, 0, 2, 2)])
def test_rectangular_windows_with_different_pads_match_bruteforce(kh, kw, ph, pw, s):
    """Windows like 1x7 are padded along their long side only."""
    rng = np.random.default_rng(kh * 10 + kw)
    layer = shapes.Layer(kind=1, n=2, c_in=3, h=6, w=8, c_out=4, kh=kh, kw=kw, stride=s, pad=ph, pad_w=pw, has_bias=1)
    assert (layer.oh, layer.ow) == ((6 + 2 * ph - kh) // s + 1, (8 + 2 * pw - kw) // s + 1)
    a = rng.standard_normal(layer.act_shape).astype(np.float32)
    rows = brute_rows(layer, a)
    got_rows = oracle.im2col_rows(layer, a)
    np.testing.assert_array_equal(got_rows, np.array(rows))
    np.testing.assert_allclose(oracle.factor_from_rows(got_rows), brute_factor(rows), rtol=1e-13, atol=1e-15)


def test_gout_rows_bruteforce():
    layer = shapes.conv(2, 3, 5, 4, 6, 3, 1, 1)
    g = np.random.default_rng(1).standard_normal(layer.gout_shape).astype(np.float32)
    rows = oracle.gout_rows(layer, g)
    for n in range(2):
        for oy in range(layer.oh):
            for ox in range(layer.ow):
                r = (n * layer.oh + oy) * layer.ow + ox
                for c in range(6):
                    assert rows[r, c] == float(g[n, c, oy, ox])
    G = oracle.factor_from_rows(rows)
    np.testing.assert_allclose(G, brute_factor(rows.tolist()), rtol=1e-13)


def test_linear_rows_and_invariants():
    layer = shapes.linear(37, 11, 5)
    a = np.maximum(np.random.default_rng(2).standard_normal((37, 11)), 0).astype(np.float32)
    rows = oracle.im2col_rows(layer, a)
    np.testing.assert_array_equal(rows[:, :11], a.astype(np.float64))
    np.testing.assert_array_equal(rows[:, 11], np.ones(37))
    A = oracle.factor_from_rows(rows)
    assert A[-1, -1] == pytest.approx(1.0, abs=1e-15)                 # mean of 1*1
    np.testing.assert_allclose(A[-1, :11], a.astype(np.float64).mean(0), rtol=1e-13)   # bias row = column means
    np.testing.assert_array_equal(A, A.T)
    assert np.linalg.eigvalsh(A).min() > -1e-12
    assert np.trace(A) == pytest.approx((rows ** 2).sum() / 37, rel=1e-13)


def test_pointwise_conv_equals_linear_on_pixels():
    """A 1x1/stride-1 convolution is a linear layer applied to every pixel."""
    layer = shapes.conv(3, 5, 4, 6, 7, 1, 1, 0)
    a = np.random.default_rng(3).standard_normal(layer.act_shape).astype(np.float32)
    A = oracle.update_factor_A(layer, a, np.eye(layer.dA), xi=0.0)
    pix = a.astype(np.float64).transpose(0, 2, 3, 1).reshape(-1, 5)
    lin = shapes.linear(pix.shape[0], 5, 7)
    A_lin = oracle.update_factor_A(lin, pix, np.eye(6), xi=0.0)
    np.testing.assert_allclose(A, A_lin, rtol=1e-13)


def test_constant_image_closed_form():
    """a == c everywhere, 3x3/pad 1: entry ((ch,i,j),(ch',i',j')) = c^2 * fraction of output
    pixels whose two taps are both inside the image; the fraction factorises per axis."""
    c, H, W = 1.5, 6, 5
    layer = shapes.conv(2, 2, H, W, 3, 3, 1, 1, 1)
    a = np.full(layer.act_shape, c, dtype=np.float32)
    A = oracle.update_factor_A(layer, a, np.zeros((19, 19)), xi=0.0)

    def inside(i, size):      # output coordinates o for which tap i lands inside: 0 <= o - 1 + i < size
        return {o for o in range(size) if 0 <= o - 1 + i < size}

    for q, (ch, i, j) in enumerate(itertools.product(range(2), range(3), range(3))):
        for q2, (ch2, i2, j2) in enumerate(itertools.product(range(2), range(3), range(3))):
            fy = len(inside(i, H) & inside(i2, H)) / H
            fx = len(inside(j, W) & inside(j2, W)) / W
            assert A[q, q2] == pytest.approx(c * c * fy * fx, rel=1e-13)
        assert A[q, 18] == pytest.approx(c * len(inside(i, H)) / H * len(inside(j, W)) / W, rel=1e-13)
    assert A[18, 18] == pytest.approx(1.0)


def test_relu_gaussian_moments():
    """Independent ReLU(N(0,1)) entries: E[a^2] = 1/2, E[a]E[a'] = 1/(2 pi), E[a] = 1/sqrt(2 pi);
    g ~ N(0, sigma^2) gives G -> sigma^2 I."""
    R, d = 200_000, 6
    rng = np.random.default_rng(4)
    a = np.maximum(rng.standard_normal((R, d)), 0).astype(np.float32)
    A = oracle.update_factor_A(shapes.linear(R, d, 3), a, np.eye(d + 1), xi=0.0)
    tol = 5 / math.sqrt(R)
    assert np.all(np.abs(np.diag(A)[:d] - 0.5) < tol)
    off = A[:d, :d][~np.eye(d, dtype=bool)]
    assert np.all(np.abs(off - 1 / (2 * math.pi)) < tol)
    assert np.all(np.abs(A[d, :d] - 1 / math.sqrt(2 * math.pi)) < tol)
    sigma = 1e-3
    g = (sigma * rng.standard_normal((R, 3))).astype(np.float32)
    G = oracle.update_factor_G(shapes.linear(R, d, 3), g, np.eye(3), xi=0.0)
    assert np.all(np.abs(G / sigma ** 2 - np.eye(3)) < 2 * tol * 3)


def test_conv_pad_moments():
    """3x3/pad-1 patches of an i.i.d. ReLU image: the second moment of tap (i,j) is 1/2 times the
    exact fraction of output pixels for which the tap is inside the image."""
    H = W = 12
    layer = shapes.conv(64, 2, H, W, 2, 3, 1, 1, 0)
    a = np.maximum(np.random.default_rng(5).standard_normal(layer.act_shape), 0).astype(np.float32)
    A = oracle.update_factor_A(layer, a, np.zeros((18, 18)), xi=0.0)
    R = layer.R
    for q, (ch, i, j) in enumerate(itertools.product(range(2), range(3), range(3))):
        frac = ((H - 1) / H if i != 1 else 1.0) * ((W - 1) / W if j != 1 else 1.0)
        assert abs(A[q, q] - 0.5 * frac) < 5 / math.sqrt(R)


def test_custom_scale():
    rows = np.random.default_rng(6).standard_normal((10, 4))
    np.testing.assert_allclose(oracle.factor_from_rows(rows, scale=0.25), 2.5 * oracle.factor_from_rows(rows), rtol=1e-14)


def test_running_average_closed_form():
    rng = np.random.default_rng(7)
    rows = rng.standard_normal((50, 5))
    Fn = oracle.factor_from_rows(rows)
    xi = 0.95
    F = np.eye(5)
    for k in range(1, 8):
        F = oracle.running_average(F, Fn, xi)
        np.testing.assert_allclose(F, xi ** k * np.eye(5) + (1 - xi ** k) * Fn, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(oracle.running_average(np.eye(5), Fn, 0.0), Fn)
    np.testing.assert_array_equal(oracle.running_average(np.eye(5), Fn, 1.0), np.eye(5))
