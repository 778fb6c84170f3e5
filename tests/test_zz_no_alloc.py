"""kfac_precondition_noalloc (the entry point for callers that cannot allocate device memory) against
kfac_precondition: same inputs, two calls in a row on one GPU, the second with a smaller input that
leaves most of the static scratch array holding the first call's contents."""
import numpy as np
import pytest

import oracle
from gpu_util import dev, host64, rel_fro, TOL_PRECOND

pytestmark = pytest.mark.gpu


def make_case(shapes_, seed):
    rng = np.random.default_rng(seed)
    XG, XA, V = [], [], []
    for dG, dA in shapes_:
        B = rng.standard_normal((dG, dG)); XG.append((B @ B.T / dG + np.eye(dG)).astype(np.float32))
        B = rng.standard_normal((dA, dA)); XA.append((B @ B.T / dA + np.eye(dA)).astype(np.float32))
        V.append((1e-2 * rng.standard_normal((dG, dA))).astype(np.float32))
    return XG, XA, V


def test_noalloc_matches_precondition_two_calls_in_a_row(kfac_lib):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ctx = kfac_lib.Context(0)
    try:
        first = [(32, 65), (130, 300), (257, 64), (64, 577), (1, 1), (512, 1153)]    # ragged tiles, several tiles per layer
        second = [(10, 129), (33, 40)]                                                 # smaller: most of the scratch keeps stale data
        for shapes_, seed in ((first, 1), (second, 2)):
            XG, XA, V = make_case(shapes_, seed)
            dG, dA = [s[0] for s in shapes_], [s[1] for s in shapes_]
            XG_d, XA_d, V_d = [dev(x) for x in XG], [dev(x) for x in XA], [dev(x) for x in V]
            want_d = [torch.full((g, a), float("nan"), device="cuda") for g, a in shapes_]
            got_d = [torch.full((g, a), float("nan"), device="cuda") for g, a in shapes_]
            ctx.kfac_precondition(dG, dA, XG_d, XA_d, V_d, want_d)
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            ctx.kfac_precondition_noalloc(dG, dA, XG_d, XA_d, V_d, got_d)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            for l, (w, g) in enumerate(zip(want_d, got_d)):
                assert torch.equal(w, g), f"layer {l} {shapes_[l]}: differs from kfac_precondition"
                ref = oracle.precondition(XG[l].astype(np.float64), XA[l].astype(np.float64), V[l].astype(np.float64))
                assert rel_fro(host64(g), ref) <= TOL_PRECOND
        # in place, as kfac_precondition allows
        ctx.kfac_precondition_noalloc(dG, dA, XG_d, XA_d, V_d, V_d)
        torch.cuda.synchronize()
        for w, g in zip(want_d, V_d):
            assert torch.equal(w, g)
        # beyond the static limits: rejected on the host with the figures in the message, nothing launched
        big = [(4096, 4096)]
        t = [torch.empty(1, device="cuda")] * 1
        assert ctx.kfac_precondition_noalloc([4096], [4096], t, t, t, [torch.empty(1, device="cuda")], check=False) == kfac_lib.KFAC_ERR_INVALID_ARG
        assert "exceed" in ctx.last_error()
        n = 33
        assert ctx.kfac_precondition_noalloc([1] * n, [1] * n, t * n, t * n, t * n, [torch.empty(1, device="cuda")] * n, check=False) == kfac_lib.KFAC_ERR_INVALID_ARG
        assert "33 layers" in ctx.last_error()
        assert ctx.kfac_precondition_noalloc([], [], None, None, None, None) == 0
    finally:
        ctx.close()
