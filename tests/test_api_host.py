"""Host-side behaviour of the C ABI that needs no GPU: exported symbols, argument validation
(performed before any launch) and schedule construction on a host-only context."""
import ctypes
import os
import re

import pytest

import paper_2107_06533_amd as pk
from synth import shapes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hctx():
    if not pk.is_built():
        import __graft_entry__
        __graft_entry__.build()
    c = pk.Context(-1)
    yield c
    c.close()


def test_every_declared_symbol_is_exported(hctx):
    header = open(os.path.join(ROOT, "include", "kfac.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kfac_[a-z_A-Z0-9]+)\s*\(", header))
    assert declared == set(pk.EXPORTS)
    lib = ctypes.CDLL(pk.lib_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_layer_queries(hctx):
    lib = pk.load()
    for l in shapes.config_layers("r50")[:8] + shapes.config_layers("fc"):
        s = pk.make_layer(l)
        assert lib.kfac_layer_dA(ctypes.byref(s)) == l.dA
        assert lib.kfac_layer_dG(ctypes.byref(s)) == l.dG
        assert lib.kfac_layer_rows(ctypes.byref(s)) == l.R
    bad = pk.make_layer(shapes.Layer(kind=1, n=1, c_in=1, h=2, w=2, c_out=1, kh=3, kw=3))   # empty output
    assert lib.kfac_layer_dA(ctypes.byref(bad)) == 0


def test_update_factors_validation(hctx):
    L = shapes.linear(4, 3, 2)
    ok = dict(layers=[L], act=[1], gout=[1], A=[1], G=[1], xi=0.5)
    call = lambda **kw: hctx.kfac_update_factors(check=False, **{**ok, **kw})
    assert call() == pk.KFAC_ERR_DEVICE                       # valid, but host-only: nothing launched
    assert call(xi=1.5) == pk.KFAC_ERR_INVALID_ARG
    assert call(xi=-0.1) == pk.KFAC_ERR_INVALID_ARG
    assert call(xi=float("nan")) == pk.KFAC_ERR_INVALID_ARG
    assert call(A=[None]) == pk.KFAC_ERR_INVALID_ARG
    assert call(G=None) == pk.KFAC_ERR_INVALID_ARG
    assert call(scale_a=float("inf")) == pk.KFAC_ERR_INVALID_ARG
    assert call(act=None, A=None) == pk.KFAC_ERR_DEVICE       # skipping every A is fine
    for bad in (shapes.linear(0, 3, 2), shapes.linear(4, 0, 2), shapes.replace(L, kind=2), shapes.replace(L, has_bias=3),
                shapes.conv(1, 1, 2, 2, 1, 3), shapes.conv(1, 1, 8, 8, 1, 3, stride=0)):
        assert call(layers=[bad]) == pk.KFAC_ERR_INVALID_ARG, bad
        assert "layer 0" in hctx.last_error()
    assert hctx.kfac_update_factors([], None, None, None, None, 0.5) == pk.KFAC_OK   # empty: no-op
    lib = pk.load()
    assert lib.kfac_update_factors(None, 0, None, None, None, None, None, 0.5, 0, 0, None) == pk.KFAC_ERR_INVALID_ARG


def test_invert_validation(hctx):
    call = lambda dims=(3,), F=(1,), X=(2,), gamma=0.1: hctx.kfac_invert_batch(list(dims), list(F), list(X), gamma, check=False)
    assert call() == pk.KFAC_ERR_DEVICE
    assert call(dims=(0,)) == pk.KFAC_ERR_INVALID_ARG
    assert call(gamma=-1.0) == pk.KFAC_ERR_INVALID_ARG
    assert call(gamma=float("nan")) == pk.KFAC_ERR_INVALID_ARG
    assert call(X=(1,)) == pk.KFAC_ERR_INVALID_ARG            # aliasing
    assert call(F=(None,)) == pk.KFAC_ERR_INVALID_ARG
    assert hctx.kfac_invert_batch([], None, None, 0.1) == pk.KFAC_OK
    # the variant with a packed second output: same checks, and the buffer is required
    assert hctx.kfac_invert_batch_packed([3], [1], [2], 5, 0.1, check=False) == pk.KFAC_ERR_DEVICE
    assert hctx.kfac_invert_batch_packed([3], [1], [2], None, 0.1, check=False) == pk.KFAC_ERR_INVALID_ARG
    assert hctx.kfac_invert_batch_packed([0], [1], [2], 5, 0.1, check=False) == pk.KFAC_ERR_INVALID_ARG
    assert hctx.kfac_invert_batch_packed([], None, None, None, 0.1) == pk.KFAC_OK


def test_precondition_validation(hctx):
    call = lambda dG=(2,), dA=(3,), g=(1,), a=(2,), v=(3,), o=(4,): hctx.kfac_precondition(
        list(dG), list(dA), list(g), list(a), list(v), list(o), check=False)
    assert call() == pk.KFAC_ERR_DEVICE
    assert call(o=(3,)) == pk.KFAC_ERR_DEVICE                 # out may alias gradW
    assert call(o=(1,)) == pk.KFAC_ERR_INVALID_ARG            # ... but not an inverse
    assert call(dG=(0,)) == pk.KFAC_ERR_INVALID_ARG
    assert call(v=(None,)) == pk.KFAC_ERR_INVALID_ARG


def test_r50_schedule(hctx):
    ls = shapes.config_layers("r50")
    n = len(ls)
    assert hctx.kfac_update_factors(ls, [1] * n, [1] * n, [1] * n, [1] * n, 0.95, check=False) == pk.KFAC_ERR_DEVICE
    st = hctx.plan_stats(0)
    alg = shapes.flops(ls)
    # the 3x3 layers are built from lag products, which execute fewer flops than the patch-matrix
    # product the algorithmic count is defined on
    assert 0.6 * (alg["factor_a"] + alg["factor_g"]) <= st["mfma_flops"] <= 1.2 * (alg["factor_a"] + alg["factor_g"])
    assert st["ws_bytes"] == hctx.workspace_bytes_factors(ls)
    dims = [l.dA for l in ls] + [l.dG for l in ls]
    assert hctx.kfac_invert_batch(dims, [1] * 2 * n, [2] * 2 * n, 0.03, check=False) == pk.KFAC_ERR_DEVICE
    st = hctx.plan_stats(1)
    assert alg["inverse"] * 0.95 <= st["mfma_flops"] <= 1.15 * alg["inverse"]
    assert st["n_launches"] >= 1 + 2 + 3 * 37                 # small bucket + per group: init/finish + sweeps of (pivot, panel, update)
    assert st["ws_bytes"] == hctx.workspace_bytes_invert(dims)
    assert hctx.kfac_precondition([l.dG for l in ls], [l.dA for l in ls], [1] * n, [2] * n, [3] * n, [4] * n, check=False) == pk.KFAC_ERR_DEVICE
    st = hctx.plan_stats(2)
    assert alg["precondition"] <= st["mfma_flops"] <= 1.1 * alg["precondition"]


def test_packed_triangles_host_side(hctx):
    tot, off = hctx.packed_elems([64, 4608, 3])
    assert off == [0, 2080, 2080 + 10619136, 2080 + 10619136 + 6] and tot == off[-1]     # Sec. IV-A sizes
    assert hctx.packed_elems([])[0] == 0 and hctx.packed_elems([4, 0])[0] == 0
    ok = pk.KFAC_ERR_DEVICE            # validated and planned, then refused by the host-only context
    assert hctx.kfac_pack_triangles([5, 130], [1, 2], 3, check=False) == ok
    assert hctx.kfac_unpack_triangles([5, 130], 3, [1, 2], check=False) == ok
    bad = pk.KFAC_ERR_INVALID_ARG
    assert hctx.kfac_pack_triangles([5, 0], [1, 2], 3, check=False) == bad
    assert hctx.kfac_pack_triangles([5, 46341], [1, 2], 3, check=False) == bad
    assert hctx.kfac_pack_triangles([5, 6], [1, None], 3, check=False) == bad
    assert hctx.kfac_pack_triangles([5, 6], [1, 2], None, check=False) == bad
    assert hctx.kfac_unpack_triangles([5, 6], None, [1, 2], check=False) == bad
    assert hctx.kfac_pack_triangles([], None, None) == 0


def test_place_inversions_matches_the_oracle():
    """Host logic of the library against the oracle's Algorithm 1 on the ResNet-50 dimensions and on
    random instances, for the three bucket weights; plus argument validation."""
    import numpy as np
    from oracle import placement as pl
    ls = shapes.config_layers("r50")
    rng = np.random.default_rng(5)
    cases = [([l.dA for l in ls] + [l.dG for l in ls], 8), ([l.dA for l in ls] + [l.dG for l in ls], 64)]
    cases += [([int(d) for d in rng.integers(1, 6000, int(rng.integers(1, 60)))], int(rng.integers(1, 17))) for _ in range(20)]
    ai, bi, ab, bb = 2.0e-4, 9.0e-4, 1.5e-3, 2.0e-9            # seconds; orders of magnitude of the paper's fits
    for dims, P in cases:
        for wp in (1, 2, 3):
            st, owner, t = pk.place_inversions(dims, P, ai, bi, ab, bb, wp)
            want = pl.lbp(dims, P, lambda d: pl.t_comp(d, ai, bi), lambda d: pl.t_comm(d, ab, bb), wp)
            assert owner == want
            t_want = pl.overall_time(want, dims, P, lambda d: pl.t_comp(d, ai, bi), lambda d: pl.t_comm(d, ab, bb))
            assert abs(t - t_want) <= 1e-12 * max(1.0, t_want)
    bad = pk.KFAC_ERR_INVALID_ARG
    assert pk.place_inversions([4, 0], 2, ai, bi, ab, bb, check=False)[0] == bad
    assert pk.place_inversions([4, 5], 0, ai, bi, ab, bb, check=False)[0] == bad
    assert pk.place_inversions([4, 5], 2, -1.0, bi, ab, bb, check=False)[0] == bad
    assert pk.place_inversions([4, 5], 2, ai, bi, ab, bb, 4, check=False)[0] == bad
    assert pk.place_inversions([], 2, ai, bi, ab, bb)[0] == 0


def test_factor_dimension_limit(hctx):
    """A factor wider than 16384 would overflow the kernels' 32-bit byte offsets (d*d*4 >= 2^32 from
    d = 32768) and could not be inverted or used by kfac_precondition anyway: rejected up front."""
    call = lambda L: hctx.kfac_update_factors([L], [1], [1], [1], [1], 0.5, check=False)
    assert call(shapes.linear(32, 16383, 8, 1)) == pk.KFAC_ERR_DEVICE            # dA = 16384: accepted
    assert call(shapes.linear(32, 16384, 8, 1)) == pk.KFAC_ERR_INVALID_ARG       # dA = 16385
    assert "dA" in hctx.last_error()
    assert call(shapes.linear(32, 40000, 8, 1)) == pk.KFAC_ERR_INVALID_ARG       # the overflowing case itself
    assert call(shapes.linear(32, 8, 16385, 1)) == pk.KFAC_ERR_INVALID_ARG
    assert "dG" in hctx.last_error()
    assert call(shapes.conv(1, 4096, 4, 4, 8, 3, 1, 1)) == pk.KFAC_ERR_INVALID_ARG   # 9 * 4096 + 1 columns
    assert call(shapes.conv(1, 1820, 4, 4, 8, 3, 1, 1)) == pk.KFAC_ERR_DEVICE        # 16381 columns
    lib = pk.load()
    s = pk.make_layer(shapes.linear(32, 16384, 8, 1))
    assert lib.kfac_layer_dA(ctypes.byref(s)) == 0


def test_options(hctx):
    """Options are per context, validated, and read no environment variable."""
    c = pk.Context(-1)
    try:
        defaults = {"inv_groups": 2, "inv_agg": 4, "inv_agg_chain": 6, "inv_fuse": 1, "inv_side_pad": 56000,
                    "factor_lag": 1, "factor_vec11": 1, "factor_xcd": 0, "factor_kjob": 8192, "inv_chain_pad": 0, "inv_side": 1, "inv_split_long": 1, "inv_yield": 64, "inv_quarter": 1}
        assert set(defaults) == set(pk.OPTIONS)
        for k, v in defaults.items():
            assert c.get_option(k) == v, k
        for k, bad in (("inv_groups", 0), ("inv_groups", 5), ("inv_agg", 0), ("inv_agg_chain", 17), ("inv_fuse", 2),
                       ("inv_side_pad", -1), ("factor_lag", -1), ("factor_kjob", 16), ("factor_kjob", 8193)):
            assert c.set_option(k, bad, check=False) == pk.KFAC_ERR_INVALID_ARG, (k, bad)
            assert c.get_option(k) == defaults[k]
        lib = pk.load()
        assert lib.kfac_set_option(c.h, 99, 1) == pk.KFAC_ERR_INVALID_ARG
        assert lib.kfac_set_option(None, 0, 1) == pk.KFAC_ERR_INVALID_ARG
        c.set_option("inv_groups", 3)
        assert c.get_option("inv_groups") == 3 and hctx.get_option("inv_groups") == 2     # the other context is untouched
    finally:
        c.close()


def test_options_change_the_schedule_not_the_environment(hctx, monkeypatch):
    """The lag-product option changes the factor schedule of a context; environment variables do not."""
    L = [shapes.conv(2, 64, 8, 8, 16, 3, 1, 1)]
    monkeypatch.setenv("KFAC_LAG", "0")
    monkeypatch.setenv("KFAC_INV_GROUPS", "1")
    c = pk.Context(-1)
    try:
        assert c.get_option("factor_lag") == 1 and c.get_option("inv_groups") == 2
        c.kfac_update_factors(L, [1], [1], [1], [1], 0.5, check=False)
        with_lag = c.plan_stats(0)
        c.set_option("factor_lag", 0)
        c.kfac_update_factors(L, [1], [1], [1], [1], 0.5, check=False)
        without = c.plan_stats(0)
        assert with_lag["n_launches"] == 3 and without["n_launches"] == 1   # tiles + pair assembly + mirror; tiles alone
        assert with_lag["ws_bytes"] > without["ws_bytes"]
    finally:
        c.close()


@pytest.mark.parametrize("name", ["fc", "cnn", "r50", "r152", "bertl", "d201", "iv4"])
@pytest.mark.parametrize("opts", [{}, {"inv_groups": 1, "inv_agg": 2, "inv_agg_chain": 3, "inv_fuse": 0, "factor_lag": 0, "factor_xcd": 1, "factor_kjob": 1024}])
def test_host_only_planning_of_every_workload(name, opts):
    """Every workload's three schedules are built on a host-only context (all index arithmetic of the
    planners runs; nothing is launched), under the default and under non-default options.  This is
    also the case a host build with address / undefined-behaviour sanitizers is run on."""
    c = pk.Context(-1)
    try:
        for k, v in opts.items():
            c.set_option(k, v)
        ls = shapes.config_layers(name)
        n = len(ls)
        alg = shapes.flops(ls)
        assert c.kfac_update_factors(ls, [1] * n, [1] * n, [1] * n, [1] * n, 0.95, check=False) == pk.KFAC_ERR_DEVICE
        st = c.plan_stats(0)
        assert st["n_jobs"] > 0 and st["ws_bytes"] == c.workspace_bytes_factors(ls)
        assert 0.3 * (alg["factor_a"] + alg["factor_g"]) <= st["mfma_flops"]
        dims = [l.dA for l in ls] + [l.dG for l in ls]
        assert c.kfac_invert_batch(dims, [1] * 2 * n, [2] * 2 * n, 0.03, check=False) == pk.KFAC_ERR_DEVICE
        st = c.plan_stats(1)
        large = sum(d ** 3 for d in dims if d > 128)             # one-block matrices take the in-register path
        assert 0.9 * large <= st["mfma_flops"] and st["n_launches"] >= 1
        assert st["ws_bytes"] <= c.workspace_bytes_invert(dims)
        assert c.kfac_precondition([l.dG for l in ls], [l.dA for l in ls], [1] * n, [2] * n, [3] * n, [4] * n, check=False) == pk.KFAC_ERR_DEVICE
        assert alg["precondition"] <= c.plan_stats(2)["mfma_flops"]
        tot, off = c.packed_elems(dims)
        assert tot == sum(d * (d + 1) // 2 for d in dims) and len(off) >= 2 * n
    finally:
        c.close()
