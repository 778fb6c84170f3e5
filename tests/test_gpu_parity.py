"""GPU parity: every call of the C ABI against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from synth import shapes, inputs
from gpu_util import dev, host64, rel_fro, inv_residual, TOL_FACTOR, TOL_INVERSE, TOL_PRECOND

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(kfac_lib):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = kfac_lib.Context(0)
    yield c
    c.close()


def run_factors(ctx, layers, acts, gouts, A0, G0, xi, scale_a=0.0, scale_g=0.0):
    import torch
    a_d = [dev(a) if a is not None else None for a in acts]
    g_d = [dev(g) if g is not None else None for g in gouts]
    A_d = [dev(A.astype(np.float32)) for A in A0]
    G_d = [dev(G.astype(np.float32)) for G in G0]
    ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, xi, scale_a, scale_g)
    torch.cuda.synchronize()
    return A_d, G_d


def check_factor(got_t, want, what):
    got = host64(got_t)
    assert np.array_equal(got, got.T), f"{what}: not exactly symmetric"
    err = rel_fro(got, want)
    assert err <= TOL_FACTOR, f"{what}: rel Frobenius {err:.3e}"
    return err


# ------------------------------------------------------------------------------ factors
LINEAR_CASES = [
    (32, 64, 32, 1),        # the small FC workload's shape
    (1000, 300, 7, 1),      # ragged tiles, ragged k
    (257, 129, 130, 0),     # one past a tile edge, no bias
    (20000, 96, 200, 1),    # split reduction (R > one job)
    (1, 5, 3, 1),           # single row
]


@pytest.mark.parametrize("R,cin,cout,bias", LINEAR_CASES)
def test_linear_factors(ctx, R, cin, cout, bias):
    rng = np.random.default_rng(R + cin)
    layer = shapes.linear(R, cin, cout, bias)
    a = np.maximum(rng.standard_normal((R, cin)), 0).astype(np.float32)
    g = (1e-3 * rng.standard_normal((R, cout))).astype(np.float32)
    A0 = np.eye(layer.dA) + 0.1 * np.ones((layer.dA, layer.dA))
    G0 = np.eye(layer.dG)
    A_d, G_d = run_factors(ctx, [layer], [a], [g], [A0], [G0], 0.95)
    check_factor(A_d[0], oracle.update_factor_A(layer, a, A0.astype(np.float32), 0.95), "A")
    check_factor(G_d[0], oracle.update_factor_G(layer, g, G0, 0.95), "G")
    if bias:
        assert abs(float(A_d[0][-1, -1]) - (0.95 * 1.1 + 0.05)) < 1e-6


CONV_CASES = [
    # n, cin, h, w, cout, kh, kw, stride, pad, bias
    (2, 3, 5, 6, 4, 1, 1, 1, 0, 1),
    (4, 70, 9, 9, 130, 1, 1, 1, 0, 1),      # G spans two tiles
    (3, 16, 10, 10, 8, 1, 1, 2, 0, 1),      # strided 1x1 (projection shortcut)
    (2, 3, 8, 8, 5, 3, 3, 1, 1, 1),
    (2, 20, 12, 11, 6, 3, 3, 1, 1, 1),      # dA = 181: two tiles, ragged
    (2, 16, 13, 13, 6, 3, 3, 2, 1, 0),      # strided 3x3
    (2, 3, 23, 21, 6, 7, 7, 2, 3, 1),       # stem-like 7x7/2
    (2, 4, 9, 8, 3, 5, 5, 1, 2, 1),         # generic window
    (2, 4, 9, 8, 3, 2, 3, 1, 0, 1),         # rectangular window
    (2, 4, 9, 8, 3, 1, 1, 1, 1, 1),         # padded 1x1 goes through the generic window path
    (16, 8, 40, 40, 8, 3, 3, 1, 1, 1),      # R = 25600 > one job: split reduction with patches
    # 3x3 / stride 1 / pad 1 with >= 64 channels: built from lag products
    (2, 64, 5, 6, 4, 3, 3, 1, 1, 1),
    (2, 70, 2, 5, 4, 3, 3, 1, 1, 1),        # two rows: top and bottom strips touch
    (3, 64, 1, 1, 4, 3, 3, 1, 1, 1),        # single pixel: only the centre tap is ever inside
    (2, 130, 7, 7, 4, 3, 3, 1, 1, 0),       # channels span two tiles, no bias
    (2, 64, 1, 9, 4, 3, 3, 1, 1, 1),        # single row
    (9, 64, 31, 30, 4, 3, 3, 1, 1, 1),      # R = 8370 > one job: split reduction of the lag products
    (2, 64, 6, 6, 4, 3, 3, 1, 1, 1),        # 36 pixels per image: lag products read four pixels at a time
    # 1x1 / stride 1 with a pixel count divisible by four: four pixels per load
    (2, 70, 8, 6, 130, 1, 1, 1, 0, 1),
    (3, 5, 2, 2, 3, 1, 1, 1, 0, 0),
    (40, 16, 16, 16, 8, 1, 1, 1, 0, 1),     # R = 10240 > one job
    (5, 129, 4, 3, 257, 1, 1, 1, 0, 1),     # ragged channel tiles on both factors
    (7, 257, 3, 4, 300, 1, 1, 1, 0, 1),     # ones column alone in the third tile row; G ends on a 44-row tile; 84 rows
    (3, 80, 2, 2, 50, 1, 1, 1, 0, 0),       # single diagonal tiles of three and of two valid block rows
    # lag products whose channel count is no multiple of the assembly's pair tiles
    (2, 100, 6, 5, 4, 3, 3, 1, 1, 1),
    (2, 96, 3, 8, 4, 3, 3, 1, 1, 0),
]


@pytest.mark.parametrize("kh,kw,ph,pw,s,cin", [(1, 7, 0, 3, 1, 20), (7, 1, 3, 0, 1, 20), (1, 3, 0, 1, 1, 70), (3, 1, 1, 0, 1, 70), (3, 5, 0, 2, 2, 9)])
def test_conv_factors_rectangular_pads(ctx, kh, kw, ph, pw, s, cin):
    """1x7 / 7x1 / 1x3 / 3x1 windows padded along their long side only (Inception-style layers)."""
    rng = np.random.default_rng(kh * 10 + kw)
    layer = shapes.Layer(kind=1, n=3, c_in=cin, h=12, w=12, c_out=6, kh=kh, kw=kw, stride=s, pad=ph, pad_w=pw, has_bias=1)
    a = np.maximum(rng.standard_normal(layer.act_shape), 0).astype(np.float32)
    g = (1e-3 * rng.standard_normal(layer.gout_shape)).astype(np.float32)
    A0, G0 = np.eye(layer.dA), np.eye(layer.dG)
    A_d, G_d = run_factors(ctx, [layer], [a], [g], [A0], [G0], 0.9)
    check_factor(A_d[0], oracle.update_factor_A(layer, a, A0, 0.9), "A")
    check_factor(G_d[0], oracle.update_factor_G(layer, g, G0, 0.9), "G")


@pytest.mark.parametrize("n,cin,h,w,cout,kh,kw,s,p,bias", CONV_CASES)
def test_conv_factors(ctx, n, cin, h, w, cout, kh, kw, s, p, bias):
    rng = np.random.default_rng(n * 1000 + cin * 10 + kh)
    layer = shapes.Layer(kind=1, n=n, c_in=cin, h=h, w=w, c_out=cout, kh=kh, kw=kw, stride=s, pad=p, has_bias=bias)
    a = np.maximum(rng.standard_normal(layer.act_shape), 0).astype(np.float32)
    g = (1e-3 * rng.standard_normal(layer.gout_shape)).astype(np.float32)
    A0, G0 = np.eye(layer.dA), np.eye(layer.dG)
    A_d, G_d = run_factors(ctx, [layer], [a], [g], [A0], [G0], 0.9)
    check_factor(A_d[0], oracle.update_factor_A(layer, a, A0, 0.9), "A")
    check_factor(G_d[0], oracle.update_factor_G(layer, g, G0, 0.9), "G")


def test_factor_options(ctx):
    """Custom scales, xi = 0 and 1, skipping A or G."""
    import torch
    rng = np.random.default_rng(5)
    layer = shapes.linear(50, 20, 10, 1)
    a = rng.standard_normal((50, 20)).astype(np.float32)
    g = rng.standard_normal((50, 10)).astype(np.float32)
    A0, G0 = np.eye(21), 2 * np.eye(10)
    A_d, G_d = run_factors(ctx, [layer], [a], [g], [A0], [G0], 0.5, scale_a=0.25, scale_g=2.0)
    check_factor(A_d[0], oracle.update_factor_A(layer, a, A0, 0.5, scale=0.25), "A scaled")
    check_factor(G_d[0], oracle.update_factor_G(layer, g, G0, 0.5, scale=2.0), "G scaled")
    A_d, G_d = run_factors(ctx, [layer], [a], [g], [A0], [G0], 0.0)
    check_factor(A_d[0], oracle.update_factor_A(layer, a, A0, 0.0), "xi=0")
    A_d, G_d = run_factors(ctx, [layer], [a], [g], [A0], [G0], 1.0)
    assert np.array_equal(host64(A_d[0]), A0) and np.array_equal(host64(G_d[0]), G0)
    A_d, G_d = run_factors(ctx, [layer], [a], [None], [A0], [G0], 0.5)     # G skipped
    assert np.array_equal(host64(G_d[0]), G0)
    check_factor(A_d[0], oracle.update_factor_A(layer, a, A0, 0.5), "A only")
    # xi = 0 must not read the old factor (NaN would propagate)
    Anan = torch.full((21, 21), float("nan"), device="cuda")
    ctx.kfac_update_factors([layer], [dev(a)], None, [Anan], None, 0.0)
    torch.cuda.synchronize()
    check_factor(Anan, oracle.update_factor_A(layer, a, A0, 0.0), "xi=0 over NaN")


# ------------------------------------------------------------------------------ inverse
def spd(d, seed, cond):
    rng = np.random.default_rng(seed)
    r = rng.standard_normal((max(d // 2, 1), d))
    F = r.T @ r / r.shape[0]                      # rank-deficient PSD, like a factor with few rows
    F *= cond / max(np.linalg.eigvalsh(F).max(), 1e-30)
    return F


def run_invert(ctx, Fs, gamma):
    import torch
    F_d = [dev(F.astype(np.float32)) for F in Fs]
    X_d = [torch.full_like(f, float("nan")) for f in F_d]
    info = torch.full((len(Fs),), -7, dtype=torch.int32, device="cuda")
    ctx.kfac_invert_batch([F.shape[0] for F in Fs], F_d, X_d, gamma, info)
    torch.cuda.synchronize()
    return F_d, X_d, info.cpu().numpy()


def test_invert_batch_mixed_sizes(ctx):
    # incl. short last pivot blocks that join the previous outer block (513, 1025, 1040) and ones that do not (641, 1060)
    dims = [1, 2, 3, 17, 64, 65, 127, 128, 129, 148, 256, 257, 300, 513, 640, 641, 1025, 1040, 1060]
    gamma = 0.03
    Fs = [spd(d, d, 5.0) + 0.5 * np.eye(d) for d in dims]
    F_d, X_d, info = run_invert(ctx, Fs, gamma)
    assert np.all(info == 0)
    for d, F, Fd, Xd in zip(dims, Fs, F_d, X_d):
        F32 = host64(Fd)                       # the fp32 bytes both sides see
        X = host64(Xd)
        assert np.array_equal(X, X.T), f"d={d}: inverse not exactly symmetric"
        res = inv_residual(F32, gamma, X)
        assert res <= TOL_INVERSE, f"d={d}: residual {res:.3e}"
        want = oracle.damped_inverse(F32, gamma)
        assert rel_fro(X, want) <= 1e-4, f"d={d}: rel error vs oracle {rel_fro(X, want):.3e}"
        np.testing.assert_array_equal(host64(Fd), F.astype(np.float32).astype(np.float64))   # F untouched


@pytest.mark.parametrize("opts", [
    {"inv_agg": 4, "inv_agg_chain": 4},                   # the outer block size of a throughput-bound group
    {"inv_agg": 5, "inv_agg_chain": 5, "inv_fuse": 0},    # separate pivot and update launches
    {"inv_agg": 3, "inv_agg_chain": 3, "inv_groups": 1},
    {"inv_groups": 3},
    {"inv_side_pad": 0},
])
def test_invert_batch_other_schedules(kfac_lib, opts):
    """The schedule options of a context (outer block size, fused pivot/update launch, number of
    lockstep groups, occupancy of the off-chain products) change launch structure only: every
    setting meets the same bar."""
    c = kfac_lib.Context(0)
    try:
        for k, v in opts.items():
            c.set_option(k, v)
            assert c.get_option(k) == v
        dims = [5, 128, 129, 257, 513, 641, 777, 1025, 1040, 1300]
        gamma = 0.03
        Fs = [spd(d, d + 1, 5.0) + 0.5 * np.eye(d) for d in dims]
        F_d, X_d, info = run_invert(c, Fs, gamma)
        assert np.all(info == 0)
        for d, Fd, Xd in zip(dims, F_d, X_d):
            X = host64(Xd)
            assert np.array_equal(X, X.T), f"{opts} d={d}: inverse not exactly symmetric"
            res = inv_residual(host64(Fd), gamma, X)
            assert res <= TOL_INVERSE, f"{opts} d={d}: residual {res:.3e}"
    finally:
        c.close()


def test_invert_identity_and_diagonal(ctx):
    Fs = [np.eye(200), np.diag(np.arange(1.0, 131.0))]
    _, X_d, info = run_invert(ctx, Fs, 0.03)
    assert np.all(info == 0)
    np.testing.assert_allclose(host64(X_d[0]), np.eye(200) / 1.03, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(host64(X_d[1]), np.diag(1 / (np.arange(1.0, 131.0) + 0.03)), rtol=1e-6, atol=1e-9)


def test_invert_uses_lower_triangle_only(ctx):
    F = spd(150, 3, 4.0) + np.eye(150)
    Fu = F.copy()
    Fu[np.triu_indices(150, 1)] = 1e6           # garbage above the diagonal must not matter
    _, X_d, _ = run_invert(ctx, [F, Fu], 0.03)
    assert np.array_equal(host64(X_d[0]), host64(X_d[1]))


def test_invert_not_spd_info(ctx):
    good = spd(300, 1, 3.0) + np.eye(300)
    bad_small = np.diag([1.0, 2.0, -1.0, 3.0])
    bad_large = good.copy()
    bad_large[200, 200] = -50.0                  # leading minor 201 fails
    _, X_d, info = run_invert(ctx, [good, bad_small, bad_large, good[:100, :100]], 0.5)
    assert info[0] == 0 and info[3] == 0
    assert info[1] == 3
    assert info[2] == 201
    st, host = ctx.kfac_check_info(4, dev(info.astype(np.int32)))
    assert st == 2 and host == [0, 3, 201, 0]
    assert inv_residual(good, 0.5, host64(X_d[0])) <= TOL_INVERSE        # the others are still valid


# ------------------------------------------------------------------------------ precondition
@pytest.mark.parametrize("dG,dA", [(32, 65), (1, 1), (10, 129), (130, 300), (257, 64), (64, 577)])
def test_precondition(ctx, dG, dA):
    import torch
    rng = np.random.default_rng(dG * 1000 + dA)
    XG = rng.standard_normal((dG, dG)); XG = XG @ XG.T / dG + np.eye(dG)
    XA = rng.standard_normal((dA, dA)); XA = XA @ XA.T / dA + np.eye(dA)
    V = (1e-2 * rng.standard_normal((dG, dA)))
    XG_d, XA_d, V_d = dev(XG.astype(np.float32)), dev(XA.astype(np.float32)), dev(V.astype(np.float32))
    out = torch.full((dG, dA), float("nan"), device="cuda")
    ctx.kfac_precondition([dG], [dA], [XG_d], [XA_d], [V_d], [out])
    torch.cuda.synchronize()
    want = oracle.precondition(host64(XG_d), host64(XA_d), host64(V_d))
    assert rel_fro(host64(out), want) <= 1e-5
    # in place
    ctx.kfac_precondition([dG], [dA], [XG_d], [XA_d], [V_d], [V_d])
    torch.cuda.synchronize()
    assert np.array_equal(host64(V_d), host64(out))


def test_precondition_nonsymmetric_inverse_is_used_as_stored(ctx):
    import torch
    rng = np.random.default_rng(9)
    XG, XA, V = rng.standard_normal((40, 40)), rng.standard_normal((70, 70)), rng.standard_normal((40, 70))
    out = torch.empty((40, 70), device="cuda")
    t = [dev(x.astype(np.float32)) for x in (XG, XA, V)]
    ctx.kfac_precondition([40], [70], [t[0]], [t[1]], [t[2]], [out])
    torch.cuda.synchronize()
    assert rel_fro(host64(out), oracle.precondition(host64(t[0]), host64(t[1]), host64(t[2]))) <= 1e-5


# ------------------------------------------------------------------------------ whole steps
def run_config_steps(ctx, name, steps, batch=None):
    import torch
    hp = shapes.config_hparams(name)
    layers = shapes.config_layers(name, batch)
    A_ref = [np.eye(l.dA) for l in layers]
    G_ref = [np.eye(l.dG) for l in layers]
    A_d = [dev(np.eye(l.dA, dtype=np.float32)) for l in layers]
    G_d = [dev(np.eye(l.dG, dtype=np.float32)) for l in layers]
    XA_d = [torch.empty_like(t) for t in A_d]
    XG_d = [torch.empty_like(t) for t in G_d]
    n = len(layers)
    info = torch.zeros(2 * n, dtype=torch.int32, device="cuda")
    worst = dict(factor=0.0, inverse=0.0, precond=0.0)
    for step in range(steps):
        ins = [inputs.layer_inputs(l, hp["cid"], step, i, hp["relu"]) for i, l in enumerate(layers)]
        acts, gouts, grads = zip(*ins)
        a_d, g_d, v_d = [dev(x) for x in acts], [dev(x) for x in gouts], [dev(x) for x in grads]
        P_d = [torch.empty_like(v) for v in v_d]
        ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, hp["xi"])
        ctx.kfac_invert_batch([l.dA for l in layers] + [l.dG for l in layers], A_d + G_d, XA_d + XG_d, hp["gamma"], info)
        ctx.kfac_precondition([l.dG for l in layers], [l.dA for l in layers], XG_d, XA_d, v_d, P_d)
        torch.cuda.synchronize()
        assert int(info.abs().sum()) == 0
        A_ref, G_ref, XA_ref, XG_ref, P_ref = oracle.kfac_step(layers, acts, gouts, grads, A_ref, G_ref, hp["xi"], hp["gamma"])
        for i in range(n):
            worst["factor"] = max(worst["factor"], check_factor(A_d[i], A_ref[i], f"step {step} A[{i}]"),
                                  check_factor(G_d[i], G_ref[i], f"step {step} G[{i}]"))
            for X_t, F_ref in ((XA_d[i], A_ref[i]), (XG_d[i], G_ref[i])):
                X = host64(X_t)
                assert np.array_equal(X, X.T)
                res = inv_residual(F_ref, hp["gamma"], X)
                assert res <= TOL_INVERSE, f"step {step} layer {i}: inverse residual {res:.3e}"
                worst["inverse"] = max(worst["inverse"], res)
            e = rel_fro(host64(P_d[i]), P_ref[i])
            assert e <= TOL_PRECOND, f"step {step} layer {i}: preconditioned gradient rel err {e:.3e}"
            worst["precond"] = max(worst["precond"], e)
    return worst


def test_fc_config_three_steps(ctx):
    print(run_config_steps(ctx, "fc", 3))


def test_cnn_config(ctx):
    print(run_config_steps(ctx, "cnn", 2))


def test_cnn_config_on_user_stream(ctx):
    """The same step issued on a caller-created (non-default) stream: the inverse forks its internal
    streams from that stream and joins them back into it."""
    import torch
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        print(run_config_steps(ctx, "cnn", 1))


def test_empty_calls_are_noops(ctx):
    assert ctx.kfac_update_factors([], None, None, None, None, 0.95) == 0
    assert ctx.kfac_invert_batch([], None, None, 0.03) == 0
    assert ctx.kfac_precondition([], [], None, None, None, None) == 0


# ------------------------------------------------------------------------------ packed triangles
def test_pack_and_unpack_triangles_bit_exact(ctx):
    """Data movement: every packed element and every unpacked element must equal the oracle's bit for bit."""
    import torch
    dims = [1, 2, 31, 32, 33, 64, 100, 257, 1000]
    rng = np.random.default_rng(11)
    Ms = [rng.standard_normal((d, d)).astype(np.float32) for d in dims]       # not symmetric: only the upper triangle may be read
    tot, off = ctx.packed_elems(dims)
    assert tot == sum(oracle.packed_size(d) for d in dims)
    M_d = [dev(M) for M in Ms]
    packed = torch.full((tot,), float("nan"), device="cuda")
    ctx.kfac_pack_triangles(dims, M_d, packed)
    torch.cuda.synchronize()
    got = packed.cpu().numpy()
    for d, M, o in zip(dims, Ms, off):
        assert np.array_equal(got[o:o + oracle.packed_size(d)], oracle.pack_upper(M)), f"pack d={d}"
    for M, Md in zip(Ms, M_d):
        assert np.array_equal(Md.cpu().numpy(), M)                             # inputs untouched
    out_d = [torch.full((d, d), float("nan"), device="cuda") for d in dims]
    ctx.kfac_unpack_triangles(dims, packed, out_d)
    torch.cuda.synchronize()
    for d, M, X in zip(dims, Ms, out_d):
        assert np.array_equal(X.cpu().numpy(), oracle.unpack_upper(oracle.pack_upper(M), d)), f"unpack d={d}"


def test_packed_round_trip_of_a_whole_factor_set(ctx):
    """The ResNet-50 set's 108 factors: pack, unpack, compare with the mirrored upper triangles."""
    import torch
    layers = shapes.config_layers("r50")
    dims = [l.dA for l in layers] + [l.dG for l in layers]
    tot, off = ctx.packed_elems(dims)
    assert tot == sum(d * (d + 1) // 2 for d in dims)
    g = torch.Generator(device="cuda").manual_seed(1)
    M_d = [torch.randn((d, d), device="cuda", generator=g) for d in dims]
    packed = torch.empty((tot,), device="cuda")
    out_d = [torch.empty_like(M) for M in M_d]
    ctx.kfac_pack_triangles(dims, M_d, packed)
    ctx.kfac_unpack_triangles(dims, packed, out_d)
    torch.cuda.synchronize()
    for d, M, X, o in zip(dims, M_d, out_d, off):
        U = torch.triu(M)
        assert torch.equal(X, U + torch.triu(M, 1).T), f"d={d}"
        iu = torch.triu_indices(d, d, device="cuda")
        assert torch.equal(packed[o:o + d * (d + 1) // 2], M[iu[0], iu[1]]), f"d={d}"


def test_invert_batch_packed_output(ctx):
    """kfac_invert_batch_packed: the packed triangles written with the inverses are, bit for bit, the
    oracle's packing of the inverses the same call returns, and those meet the usual bar."""
    import torch
    dims = [1, 3, 31, 33, 64, 128, 129, 257, 300, 641, 1025]
    gamma = 0.03
    Fs = [spd(d, d + 7, 5.0) + 0.5 * np.eye(d) for d in dims]
    F_d = [dev(F.astype(np.float32)) for F in Fs]
    X_d = [torch.full_like(f, float("nan")) for f in F_d]
    tot, off = ctx.packed_elems(dims)
    packed = torch.full((tot,), float("nan"), device="cuda")
    info = torch.full((len(dims),), -7, dtype=torch.int32, device="cuda")
    ctx.kfac_invert_batch_packed(dims, F_d, X_d, packed, gamma, info)
    torch.cuda.synchronize()
    assert int(info.abs().sum()) == 0
    got = packed.cpu().numpy()
    for d, Fd, Xd, o in zip(dims, F_d, X_d, off):
        X32 = Xd.cpu().numpy()
        assert np.array_equal(got[o:o + oracle.packed_size(d)], oracle.pack_upper(X32)), f"d={d}: packed != pack_upper(X)"
        assert inv_residual(host64(Fd), gamma, X32.astype(np.float64)) <= TOL_INVERSE, f"d={d}"
    assert ctx.kfac_invert_batch_packed(dims, F_d, X_d, None, gamma, info, check=False) == 1   # packed is required


# ------------------------------------------------------------------------------ stale inverses
def test_precondition_with_last_inverses_while_inverting(ctx):
    """Inverse update interval > 1 on one GPU: the new inverses are computed on one stream while the
    gradients are preconditioned with the previous ones on another (calls of different kinds own
    separate workspaces).  Both results must match the oracle."""
    import torch
    hp = shapes.config_hparams("cnn")
    layers = shapes.config_layers("cnn")
    n = len(layers)
    dims = [l.dA for l in layers] + [l.dG for l in layers]
    dG, dA = [l.dG for l in layers], [l.dA for l in layers]
    A_ref, G_ref = [np.eye(l.dA) for l in layers], [np.eye(l.dG) for l in layers]
    A_d = [dev(np.eye(l.dA, dtype=np.float32)) for l in layers]
    G_d = [dev(np.eye(l.dG, dtype=np.float32)) for l in layers]
    X_old = [torch.empty((d, d), device="cuda") for d in dims]
    X_new = [torch.empty((d, d), device="cuda") for d in dims]
    # step 0: ordinary step, gives the inverses that step 1 reuses
    ins = [inputs.layer_inputs(l, hp["cid"], 0, i, hp["relu"]) for i, l in enumerate(layers)]
    acts, gouts, grads = zip(*ins)
    ctx.kfac_update_factors(layers, [dev(x) for x in acts], [dev(x) for x in gouts], A_d, G_d, hp["xi"])
    ctx.kfac_invert_batch(dims, A_d + G_d, X_old, hp["gamma"])
    torch.cuda.synchronize()
    A_ref, G_ref, XA0, XG0, _ = oracle.kfac_step(layers, acts, gouts, grads, A_ref, G_ref, hp["xi"], hp["gamma"])
    # step 1: new factors; invert on s1 while preconditioning with the old inverses on s2
    ins = [inputs.layer_inputs(l, hp["cid"], 1, i, hp["relu"]) for i, l in enumerate(layers)]
    acts, gouts, grads = zip(*ins)
    v_d = [dev(x) for x in grads]
    P_d = [torch.empty_like(v) for v in v_d]
    ctx.kfac_update_factors(layers, [dev(x) for x in acts], [dev(x) for x in gouts], A_d, G_d, hp["xi"])
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ctx.kfac_invert_batch(dims, A_d + G_d, X_new, hp["gamma"], stream=s1)
    ctx.kfac_precondition(dG, dA, X_old[n:], X_old[:n], v_d, P_d, stream=s2)
    torch.cuda.synchronize()
    A_ref, G_ref, XA1, XG1, _ = oracle.kfac_step(layers, acts, gouts, grads, A_ref, G_ref, hp["xi"], hp["gamma"])
    for i in range(n):
        want = oracle.precondition(XG0[i], XA0[i], grads[i])
        e = rel_fro(host64(P_d[i]), want)
        assert e <= TOL_PRECOND, f"layer {i}: preconditioning with the previous inverses, rel err {e:.3e}"
        for X_t, F_ref in ((X_new[i], A_ref[i]), (X_new[n + i], G_ref[i])):
            res = inv_residual(F_ref, hp["gamma"], host64(X_t))
            assert res <= TOL_INVERSE, f"layer {i}: new inverse residual {res:.3e}"


# ------------------------------------------------------------------------------ packed factor output
def test_update_factors_packed_output(ctx):
    """kfac_update_factors_packed: the packed triangles written with the factors (all A in layer order,
    then all G) are, bit for bit, the oracle's packing of the factors the same call returns, on every
    kernel that writes a factor: tiles written directly, split reductions, lag-product assembly,
    linear layers; the factors themselves meet the usual bar against the oracle's factors, and the
    segment of a skipped factor is left untouched."""
    import torch
    layers = [shapes.linear(50, 70, 33, name="lin"),                      # direct tiles, ones column
              shapes.conv(2, 20, 12, 11, 200, 3, 1, 1, name="c3"),        # 3x3 patch product, dA = 181
              shapes.conv(2, 64, 6, 6, 16, 3, 1, 1, name="lag"),          # lag products, dA = 577
              shapes.conv(40, 4, 16, 16, 140, 1, 1, 0, name="split"),     # R = 10240: split reduction of G (140) and A (5)
              shapes.conv(3, 16, 10, 10, 130, 1, 2, 0, name="s2")]        # strided 1x1
    hp = dict(cid=9, relu=True)
    ins = [inputs.layer_inputs(l, hp["cid"], 0, i, hp["relu"]) for i, l in enumerate(layers)]
    acts, gouts, _ = zip(*ins)
    gouts = [g * 1e3 for g in gouts]                                       # gradients of size one: the new term counts
    xi = 0.3
    rng = np.random.default_rng(5)
    def old(d):
        B = rng.standard_normal((d, d)).astype(np.float32)
        return ((B @ B.T) / d).astype(np.float32)
    A0, G0 = [old(l.dA) for l in layers], [old(l.dG) for l in layers]
    a_d, g_d = [dev(x) for x in acts], [dev(x) for x in gouts]
    A_d, G_d = [dev(x) for x in A0], [dev(x) for x in G0]
    dims = [l.dA for l in layers] + [l.dG for l in layers]
    tot, off = ctx.packed_elems(dims)
    packed = torch.full((tot,), float("nan"), device="cuda")
    g_skip = list(g_d)
    g_skip[1] = None                                                       # G of layer 1 is not updated
    ctx.kfac_update_factors_packed(layers, a_d, g_skip, A_d, G_d, xi, packed)
    torch.cuda.synchronize()
    got = packed.cpu().numpy()
    n = len(layers)
    for i, l in enumerate(layers):
        A32, G32 = A_d[i].cpu().numpy(), G_d[i].cpu().numpy()
        assert np.array_equal(got[off[i]:off[i] + oracle.packed_size(l.dA)], oracle.pack_upper(A32)), f"{l.name}: packed A"
        wantA = oracle.update_factor_A(l, acts[i], A0[i].astype(np.float64), xi)
        assert rel_fro(A32.astype(np.float64), wantA) <= TOL_FACTOR, l.name
        seg = got[off[n + i]:off[n + i] + oracle.packed_size(l.dG)]
        if i == 1:
            assert np.all(np.isnan(seg)), "segment of a skipped factor was written"
            assert np.array_equal(G32, G0[i])
            continue
        assert np.array_equal(seg, oracle.pack_upper(G32)), f"{l.name}: packed G"
        wantG = oracle.update_factor_G(l, gouts[i], G0[i].astype(np.float64), xi)
        assert rel_fro(G32.astype(np.float64), wantG) <= TOL_FACTOR, l.name
    assert ctx.kfac_update_factors_packed(layers, a_d, g_d, A_d, G_d, xi, None, check=False) == 1   # packed is required


def test_chain_products_as_blocks_match_tile_jobs(kfac_lib):
    """Option inv_quarter: the two products on the sweep chain of the long-chain group run as 32 x 32
    blocks per wave fed from memory instead of 128 x 128 tile jobs.  Same contraction order, so the
    inverses must agree bit for bit, ragged sizes and one-row tails included."""
    import torch
    dims = [1300, 1153, 1025, 641, 513, 257, 129, 64]     # the first three form the long-chain group
    gamma = 0.03
    Fs = [spd(d, 7 * d + 1, 5.0) + 0.5 * np.eye(d) for d in dims]
    results = []
    for quarter in (1, 0):
        c = kfac_lib.Context(0)
        try:
            c.set_option("inv_quarter", quarter)
            c.set_option("inv_agg_chain", 3)               # several outer blocks at these sizes
            F_d, X_d, info = run_invert(c, Fs, gamma)
            assert np.all(info == 0)
            results.append(X_d)
        finally:
            c.close()
    for d, a, b in zip(dims, *results):
        assert torch.equal(a, b), f"d={d}: block products and tile jobs disagree"
        assert inv_residual(host64(dev(Fs[dims.index(d)].astype(np.float32))), gamma, host64(a)) <= 1e-4
