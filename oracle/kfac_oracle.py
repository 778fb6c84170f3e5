"""Plain fp64 NumPy oracle of the per-worker K-FAC arithmetic (TEST INFRASTRUCTURE).

This module is the slow, obviously-correct definition that the HIP kernels are
checked against.  It is never used by the product path and imports nothing from
it.  All inputs are taken as given (fp32 arrays are upcast to float64 first) and
every result is float64.

What is computed, and where the paper defines it:

* Kronecker factors A = a a^T and G = g g^T of a layer (Sec. II-B, Eq. factorA /
  Eq. factorG), taken as the batch mean over the rows of the (patch-expanded)
  activation matrix and of the output-gradient matrix.  The paper prints only the
  outer product; the normalisation 1/R (R = number of rows), the ones column for
  the bias, the patch expansion for convolutions and the running average with
  decay xi are this build's stated readings (the paper defers to the K-FAC
  literature it cites for convolutions).
* Tikhonov-damped inverse (F + gamma I)^-1 of each factor (Sec. II-B, the damped
  update rule above Eq. kfacfinal; Sec. V-B says it is obtained through a Cholesky
  decomposition).
* Preconditioned gradient (A+gamma I)^-1 (x) (G+gamma I)^-1 applied to the layer's
  gradient (Eq. kfacfinal with P = 1), evaluated as G^-1 . V . A^-1 on the
  [dG, dA] weight-gradient matrix.

* Packed upper triangles of symmetric factors and inverses, the form in which the
  paper communicates them (Sec. IV-A: d(d+1)/2 elements per factor; Sec. V-B: upper
  triangle including the diagonal).

Parity pins live in tests/test_oracle_*.py: brute-force sums, closed forms
(Sherman-Morrison, diagonal, 2x2), statistical limits, and the brute-force
Kronecker solve.  Every function below has at least one such pin.
"""
from __future__ import annotations

import numpy as np

LINEAR, CONV2D = 0, 1


class NotPositiveDefinite(ArithmeticError):
    """Raised by damped_inverse; .info is the 1-based order of the first leading
    minor that is not positive (LAPACK convention)."""

    def __init__(self, info: int):
        super().__init__(f"leading minor of order {info} is not positive")
        self.info = info


# --------------------------------------------------------------------------- rows

def im2col_rows(layer, act) -> np.ndarray:
    """Activation matrix a-bar [R, dA] in float64 for one layer.

    Linear layer: a-bar = [a, 1] (ones column last when has_bias).
    Convolution (square or rectangular kernel, zero padding, dilation 1, groups 1):
    row r = (n*OH + oy)*OW + ox is the receptive field of output pixel (n, oy, ox);
    column q = (c*kh + i)*kw + j holds a[n, c, oy*stride - pad_h + i, ox*stride - pad_w + j]
    (0 outside the image), so columns are ordered like a weight tensor
    [C_out, C_in, kh, kw] flattened to [C_out, C_in*kh*kw]; ones column last.
    """
    a = np.asarray(act, dtype=np.float64)
    if layer.kind == LINEAR:
        assert a.shape == (layer.rows, layer.c_in)
        cols = a
    else:
        n, c, h, w = layer.n, layer.c_in, layer.h, layer.w
        assert a.shape == (n, c, h, w)
        kh, kw, s = layer.kh, layer.kw, layer.stride
        ph, pw = layer.ph, layer.pw                 # zero padding of the height / of the width
        oh, ow = layer.oh, layer.ow
        ap = np.zeros((n, c, h + 2 * ph, w + 2 * pw), dtype=np.float64)
        ap[:, :, ph:ph + h, pw:pw + w] = a
        patches = np.empty((n, oh, ow, c, kh, kw), dtype=np.float64)
        for i in range(kh):
            for j in range(kw):
                # rows oy*s + i, cols ox*s + j of the padded image
                win = ap[:, :, i:i + (oh - 1) * s + 1:s, j:j + (ow - 1) * s + 1:s]   # [n, c, oh, ow]
                patches[:, :, :, :, i, j] = win.transpose(0, 2, 3, 1)
        cols = patches.reshape(n * oh * ow, c * kh * kw)
    if layer.has_bias:
        cols = np.concatenate([cols, np.ones((cols.shape[0], 1), dtype=np.float64)], axis=1)
    return np.ascontiguousarray(cols)


def gout_rows(layer, gout) -> np.ndarray:
    """Output-gradient matrix g-bar [R, dG] in float64: one row per sample (linear) or
    per output pixel (n, oy, ox) (convolution), one column per output channel."""
    g = np.asarray(gout, dtype=np.float64)
    if layer.kind == LINEAR:
        assert g.shape == (layer.rows, layer.c_out)
        return np.ascontiguousarray(g)
    assert g.shape == (layer.n, layer.c_out, layer.oh, layer.ow)
    return np.ascontiguousarray(g.transpose(0, 2, 3, 1).reshape(-1, layer.c_out))


# ------------------------------------------------------------------------ factors

def factor_from_rows(rows: np.ndarray, scale: float | None = None) -> np.ndarray:
    """F_new = scale * rows^T rows  (Eq. factorA / Eq. factorG summed over the batch);
    scale defaults to 1/R with R the number of rows."""
    rows = np.asarray(rows, dtype=np.float64)
    if scale is None or scale <= 0:
        scale = 1.0 / rows.shape[0]
    return (rows.T @ rows) * scale


def running_average(F_old: np.ndarray, F_new: np.ndarray, xi: float) -> np.ndarray:
    """F <- xi * F_old + (1 - xi) * F_new (plain exponential average, no bias correction)."""
    return xi * np.asarray(F_old, dtype=np.float64) + (1.0 - xi) * np.asarray(F_new, dtype=np.float64)


def update_factor_A(layer, act, A_old, xi, scale=None) -> np.ndarray:
    return running_average(A_old, factor_from_rows(im2col_rows(layer, act), scale), xi)


def update_factor_G(layer, gout, G_old, xi, scale=None) -> np.ndarray:
    return running_average(G_old, factor_from_rows(gout_rows(layer, gout), scale), xi)


# ------------------------------------------------------------------------ inverse

def damped_inverse(F: np.ndarray, gamma: float) -> np.ndarray:
    """X = (F + gamma I)^-1 through a Cholesky factorisation (Sec. II-B damping; Sec. V-B).

    F + gamma I = L L^T,  Y = L^-1 (forward substitution against I),  X = Y^T Y.
    X is symmetric by construction.  Raises NotPositiveDefinite(info) when a
    leading minor is not positive.
    """
    F = np.asarray(F, dtype=np.float64)
    d = F.shape[0]
    assert F.shape == (d, d)
    M = F + gamma * np.eye(d)          # only the lower triangle is read below
    try:
        L = np.linalg.cholesky(M)
    except np.linalg.LinAlgError:
        raise NotPositiveDefinite(_first_bad_minor(M))
    if not np.all(np.isfinite(L)):
        raise NotPositiveDefinite(_first_bad_minor(M))
    from scipy.linalg import solve_triangular
    Y = solve_triangular(L, np.eye(d), lower=True)
    return Y.T @ Y


def _first_bad_minor(M: np.ndarray) -> int:
    """1-based order of the first non-positive pivot of an unblocked Cholesky."""
    d = M.shape[0]
    L = np.zeros_like(M)
    for j in range(d):
        s = M[j, j] - L[j, :j] @ L[j, :j]
        if not (s > 0.0) or not np.isfinite(s):
            return j + 1
        L[j, j] = np.sqrt(s)
        L[j + 1:, j] = (M[j + 1:, j] - L[j + 1:, :j] @ L[j, :j]) / L[j, j]
    return d


# ------------------------------------------------------------------- precondition

def precondition(XG: np.ndarray, XA: np.ndarray, V) -> np.ndarray:
    """P = X_G . V . X_A for the [dG, dA] gradient matrix V (Eq. kfacfinal, P = 1:
    the Kronecker-product inverse applied to the layer's gradient)."""
    V = np.asarray(V, dtype=np.float64)
    return np.asarray(XG, dtype=np.float64) @ V @ np.asarray(XA, dtype=np.float64)


# ------------------------------------------------------------- packed triangles

def packed_size(d: int) -> int:
    """Number of communicated elements of a symmetric d x d factor: d (d + 1) / 2 (Sec. IV-A)."""
    return d * (d + 1) // 2


def pack_upper(M: np.ndarray) -> np.ndarray:
    """Upper triangle of a symmetric matrix including the diagonal, row after row (Sec. V-B: only
    these elements of a factor or of an inverse are sent): [m00 m01 .. m0,d-1 | m11 .. | .. | m_d-1,d-1].
    Written as the explicit double loop; no symmetry is assumed (the lower triangle is ignored)."""
    M = np.asarray(M)
    d = M.shape[0]
    assert M.shape == (d, d)
    out = np.empty(packed_size(d), dtype=M.dtype)
    p = 0
    for i in range(d):
        for j in range(i, d):
            out[p] = M[i, j]
            p += 1
    return out


def unpack_upper(packed: np.ndarray, d: int) -> np.ndarray:
    """Inverse of pack_upper: the full symmetric matrix whose upper triangle is `packed`."""
    packed = np.asarray(packed)
    assert packed.shape == (packed_size(d),)
    M = np.empty((d, d), dtype=packed.dtype)
    p = 0
    for i in range(d):
        for j in range(i, d):
            M[i, j] = packed[p]
            M[j, i] = packed[p]
            p += 1
    return M


# --------------------------------------------------------------------- whole step

def kfac_step(layers, acts, gouts, gradWs, A_list, G_list, xi, gamma):
    """One iteration in the order the paper runs it (Fig. 1b): build every layer's
    factors, invert every damped factor, precondition every layer's gradient.
    Returns (A_list, G_list, XA_list, XG_list, P_list), all float64."""
    A_new = [update_factor_A(l, a, A, xi) for l, a, A in zip(layers, acts, A_list)]
    G_new = [update_factor_G(l, g, G, xi) for l, g, G in zip(layers, gouts, G_list)]
    XA = [damped_inverse(A, gamma) for A in A_new]
    XG = [damped_inverse(G, gamma) for G in G_new]
    P = [precondition(xg, xa, v) for xg, xa, v in zip(XG, XA, gradWs)]
    return A_new, G_new, XA, XG, P
