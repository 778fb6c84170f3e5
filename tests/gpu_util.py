"""Helpers shared by the GPU parity tests: device upload and the acceptance metrics."""
import numpy as np


def dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def host64(t):
    return t.detach().cpu().numpy().astype(np.float64)


def rel_fro(got, want):
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def inv_residual(F64, gamma, X64):
    d = F64.shape[0]
    return float(np.linalg.norm((F64 + gamma * np.eye(d)) @ X64 - np.eye(d)) / np.sqrt(d))


# acceptance bars of the build (fp32 path against the fp64 oracle)
TOL_FACTOR = 1e-5      # relative Frobenius error of a factor
TOL_INVERSE = 1e-4     # ||(F + gamma I) X - I||_F / sqrt(d), F = the oracle's factor
TOL_PRECOND = 1e-3     # relative Frobenius error of a preconditioned gradient


def max_abs_rel(got, want):
    """Largest element error relative to the largest element of the reference: a bound every single
    entry has to meet, beside the Frobenius norm that averages over them."""
    return float(np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-300))


TOL_FACTOR_ELEM = 1e-5   # max |got - want| / max |want| of a factor
