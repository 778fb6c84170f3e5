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
