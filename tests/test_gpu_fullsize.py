"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: one
kfac_update_factors + kfac_invert_batch + kfac_precondition over the whole layer set, each a
single call on the current stream with identity factors as the running-average start.

ResNet-50 set: every output of every layer is compared with the fp64 oracle element by element.
ResNet-152 and BERT-large sets: the oracle is run on one layer of every distinct shape class plus
the last layer (whole step for those layers, compared element by element); every other output is
covered by properties that hold at any size, evaluated in fp64 with torch on the device:
exact symmetry, the damped-inverse residual against the factor the GPU produced, and the
two-sided product recomputed from the GPU's own inverses.
"""
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle
from synth import shapes, inputs
from gpu_util import host64, rel_fro, inv_residual, TOL_FACTOR, TOL_INVERSE, TOL_PRECOND

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.fixture(scope="module")
def ctx(kfac_lib):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = kfac_lib.Context(0)
    yield c
    c.close()


def upload_inputs(name):
    """Seeded inputs of a whole configuration, generated on the host and uploaded once."""
    import torch
    hp = shapes.config_hparams(name)
    layers = shapes.config_layers(name)
    with ThreadPoolExecutor(max_workers=8) as ex:
        ins = list(ex.map(lambda il: inputs.layer_inputs(il[1], hp["cid"], 0, il[0], hp["relu"]), enumerate(layers)))
    up = lambda x: torch.from_numpy(x).cuda()
    return hp, layers, ins, ([up(x[0]) for x in ins], [up(x[1]) for x in ins], [up(x[2]) for x in ins])


def run_step(ctx, hp, layers, dev_inputs):
    """One step as bench.py issues it, on fresh output buffers (identity factors as the running-average start)."""
    import torch
    a_d, g_d, v_d = dev_inputs
    n = len(layers)
    A_d = [torch.eye(l.dA, device="cuda") for l in layers]
    G_d = [torch.eye(l.dG, device="cuda") for l in layers]
    XA_d = [torch.full_like(t, float("nan")) for t in A_d]
    XG_d = [torch.full_like(t, float("nan")) for t in G_d]
    P_d = [torch.full_like(v, float("nan")) for v in v_d]
    info = torch.full((2 * n,), -1, dtype=torch.int32, device="cuda")
    dims = [l.dA for l in layers] + [l.dG for l in layers]
    stream = torch.cuda.current_stream()
    ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, hp["xi"], stream=stream)
    ctx.kfac_invert_batch(dims, A_d + G_d, XA_d + XG_d, hp["gamma"], info, stream=stream)
    ctx.kfac_precondition([l.dG for l in layers], [l.dA for l in layers], XG_d, XA_d, v_d, P_d, stream=stream)
    torch.cuda.synchronize()
    assert int(info.abs().sum()) == 0, "a factor was reported not positive definite"
    return dict(A=A_d, G=G_d, XA=XA_d, XG=XG_d, P=P_d, V=v_d)


def gpu_step(ctx, name):
    """Upload the seeded inputs of a whole configuration and run one step as bench.py does."""
    hp, layers, ins, dev_inputs = upload_inputs(name)
    return hp, layers, ins, run_step(ctx, hp, layers, dev_inputs)


def check_layer_against_oracle(i, l, ins_i, hp, out):
    """Whole step of one layer in the oracle, compared element by element."""
    a, g, v = ins_i
    A, G, XA, XG, P = oracle.kfac_step([l], [a], [g], [v], [np.eye(l.dA)], [np.eye(l.dG)], hp["xi"], hp["gamma"])
    worst = {}
    for key, ref in (("A", A[0]), ("G", G[0])):
        got = host64(out[key][i])
        assert np.array_equal(got, got.T), f"layer {i} {key}: not exactly symmetric"
        e = rel_fro(got, ref)
        assert e <= TOL_FACTOR, f"layer {i} ({l.name}) {key}: rel Frobenius {e:.3e}"
        worst["factor"] = max(worst.get("factor", 0.0), e)
    for key, F in (("XA", A[0]), ("XG", G[0])):
        X = host64(out[key][i])
        assert np.array_equal(X, X.T), f"layer {i} {key}: not exactly symmetric"
        r = inv_residual(F, hp["gamma"], X)
        assert r <= TOL_INVERSE, f"layer {i} ({l.name}) {key}: residual {r:.3e}"
        worst["inverse"] = max(worst.get("inverse", 0.0), r)
    e = rel_fro(host64(out["P"][i]), P[0])
    assert e <= TOL_PRECOND, f"layer {i} ({l.name}) preconditioned gradient: rel err {e:.3e}"
    worst["precond"] = e
    return worst


def check_layer_properties(i, l, hp, out):
    """Size-independent properties in fp64 on the device (no oracle): symmetry, residual of the
    inverse against the GPU's own factor, two-sided product from the GPU's own inverses."""
    import torch
    for fk, xk in (("A", "XA"), ("G", "XG")):
        F, X = out[fk][i], out[xk][i]
        assert torch.equal(F, F.T) and torch.equal(X, X.T), f"layer {i} {fk}/{xk}: not exactly symmetric"
        d = F.shape[0]
        M = F.double()
        M.diagonal().add_(hp["gamma"])
        R = M @ X.double()
        R.diagonal().sub_(1.0)
        r = float(torch.linalg.norm(R) / np.sqrt(d))
        assert r <= TOL_INVERSE, f"layer {i} ({l.name}) {xk}: residual {r:.3e}"
    want = out["XG"][i].double() @ out["V"][i].double() @ out["XA"][i].double()
    e = float(torch.linalg.norm(out["P"][i].double() - want) / torch.linalg.norm(want))
    assert e <= 1e-5, f"layer {i} ({l.name}): two-sided product differs from its fp64 recomputation by {e:.3e}"


def merge(w, x):
    for k, v in x.items():
        w[k] = max(w.get(k, 0.0), v)


@pytest.fixture(scope="module")
def r50(kfac_lib):
    return upload_inputs("r50")


def test_r50_every_layer_against_oracle(ctx, r50):
    t0 = time.perf_counter()
    hp, layers, ins, dev_inputs = r50
    out = run_step(ctx, hp, layers, dev_inputs)
    print(f"\nr50: GPU step {time.perf_counter() - t0:.1f} s", flush=True)
    worst = {}
    t0 = time.perf_counter()
    for i, l in enumerate(layers):
        merge(worst, check_layer_against_oracle(i, l, ins[i], hp, out))
    print(f"r50: oracle over {len(layers)} layers {time.perf_counter() - t0:.1f} s, worst {worst}", flush=True)


@pytest.mark.parametrize("groups", [2, 1])
def test_r50_step_is_bit_reproducible(kfac_lib, r50, groups):
    """The whole step run three times on fresh output buffers gives the same bits every time: every
    sum is taken in a fixed order, and no kernel reads what another stream has not finished writing
    (kfac_invert_batch orders up to two sweep chains and two side streams with events).  Checked for
    the default two lockstep groups and for one."""
    import torch
    hp, layers, ins, dev_inputs = r50
    c = kfac_lib.Context(0)
    try:
        c.set_option("inv_groups", groups)
        first = run_step(c, hp, layers, dev_inputs)
        for rep in range(2):
            again = run_step(c, hp, layers, dev_inputs)
            for key in ("A", "G", "XA", "XG", "P"):
                for i, (x, y) in enumerate(zip(first[key], again[key])):
                    assert torch.equal(x, y), f"groups={groups} run {rep + 2}: {key}[{i}] ({layers[i].name}) differs from the first run"
            del again
    finally:
        c.close()


def sampled_layers(layers, cap=28):
    """First layer of every distinct shape class plus the last layer; when there are more classes
    than `cap` (DenseNet: every dense layer has its own input width), an even subsample of them."""
    first = {}
    for i, l in enumerate(layers):
        first.setdefault((l.kind, l.dA, l.dG, l.R, l.kh, l.kw, l.stride), i)
    idx = sorted(first.values())
    if len(idx) > cap:
        idx = [idx[round(k * (len(idx) - 1) / (cap - 1))] for k in range(cap)]
    return sorted(set(idx) | {len(layers) - 1})


@pytest.mark.parametrize("name", ["r152", "bertl", "d201", "iv4"])
def test_large_sets_sampled_against_oracle(ctx, name):
    t0 = time.perf_counter()
    hp, layers, ins, out = gpu_step(ctx, name)
    print(f"\n{name}: inputs + GPU step {time.perf_counter() - t0:.1f} s", flush=True)
    sample = sampled_layers(layers)
    worst = {}
    t0 = time.perf_counter()
    for i in sample:
        merge(worst, check_layer_against_oracle(i, layers[i], ins[i], hp, out))
    print(f"{name}: oracle on layers {sample}: {time.perf_counter() - t0:.1f} s, worst {worst}", flush=True)
    t0 = time.perf_counter()
    for i, l in enumerate(layers):
        if i not in sample:
            check_layer_properties(i, l, hp, out)
    print(f"{name}: properties of the other {len(layers) - len(sample)} layers {time.perf_counter() - t0:.1f} s", flush=True)


def test_invert_largest_dimension(ctx):
    """d = 16384, the largest matrix kfac_invert_batch accepts: checked by the properties that hold at
    any size (exact symmetry, damped-inverse residual in fp64 on the device); the oracle would need
    minutes for this one matrix."""
    import torch
    d, gamma = 16384, 0.03
    g = torch.Generator(device="cuda").manual_seed(210706533)
    B = torch.randn((d, 256), device="cuda", generator=g)
    F = 0.05 * (B @ B.T) / 256.0                # one running-average step from the identity, as every factor here
    F.diagonal().add_(0.95)
    F = torch.tril(F) + torch.tril(F, -1).T
    X = torch.empty_like(F)
    info = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    del B
    ctx.kfac_invert_batch([d], [F], [X], gamma, info)
    torch.cuda.synchronize()
    assert int(info[0]) == 0
    assert torch.equal(X, X.T)
    res = 0.0
    for c0 in range(0, d, 4096):                # residual column block by column block (bounded fp64 temporaries)
        Rb = F.double() @ X[:, c0:c0 + 4096].double() + gamma * X[:, c0:c0 + 4096].double()
        Rb[c0:c0 + 4096, :].diagonal().sub_(1.0)
        res += float((Rb * Rb).sum())
    res = (res / d) ** 0.5
    print(f"\nd={d}: residual {res:.3e}", flush=True)
    assert res <= TOL_INVERSE


def test_factor_largest_operand(ctx):
    """A linear layer whose activation tensor has 2^28 elements (1 GiB, the largest operand the library
    accepts): sampled entries of A against the oracle's definition evaluated one entry at a time."""
    import torch
    rows, cin = 65536, 4096
    layer = shapes.linear(rows, cin, 8, has_bias=1)
    rng = np.random.default_rng(7)
    a = rng.standard_normal((rows, cin), dtype=np.float32)
    np.maximum(a, 0.0, out=a)
    a_d = torch.from_numpy(a).cuda()
    A_d = torch.eye(layer.dA, device="cuda")
    ctx.kfac_update_factors([layer], [a_d], None, [A_d], None, 0.95)
    torch.cuda.synchronize()
    assert torch.equal(A_d, A_d.T)
    idx = rng.integers(0, layer.dA, size=(300, 2))
    idx[:20, 1] = layer.dA - 1                   # bias column
    idx[20:30, 0] = idx[20:30, 1]                # diagonal
    idx[30] = (layer.dA - 1, layer.dA - 1)
    got = A_d[torch.from_numpy(idx[:, 0]).cuda(), torch.from_numpy(idx[:, 1]).cuda()].cpu().numpy().astype(np.float64)
    col = lambda q: np.ones(rows) if q == cin else a[:, q].astype(np.float64)
    want = np.array([0.95 * (i == j) + 0.05 * float(col(i) @ col(j)) / rows for i, j in idx])
    err = np.linalg.norm(got - want) / np.linalg.norm(want)
    print(f"\nlargest operand: sampled rel error {err:.3e}", flush=True)
    assert err <= TOL_FACTOR
