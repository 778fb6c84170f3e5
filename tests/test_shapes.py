"""Layer enumerators against the sizes the paper prints (Table II, Sec. IV-A)."""
import os

import pytest

from synth import shapes

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_table2_factor_sizes.txt")


def _gold():
    rows = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        m, L, a, g, lo, hi = line.split()
        rows[m] = (int(L), float(a), float(g), int(lo), int(hi))
    return rows


@pytest.mark.parametrize("model,blocks", [("resnet50", (3, 4, 6, 3)), ("resnet152", (3, 8, 36, 3))])
def test_resnet_matches_paper_table(model, blocks):
    L, As, Gs, lo, hi = _gold()[model]
    ls = shapes.resnet_layers(blocks, conv_bias=0)
    # the paper counts the FC layer's A without the bias column too: try both, require one to match
    assert len(ls) == L
    tri = lambda d: d * (d + 1) // 2
    a_tot = sum(tri(l.c_in * l.kh * l.kw) for l in ls) / 1e6
    g_tot = sum(tri(l.dG) for l in ls) / 1e6
    assert abs(a_tot - As) < 0.06
    assert abs(g_tot - Gs) < 0.06
    if lo > 0:
        sizes = [tri(l.c_in * l.kh * l.kw) for l in ls] + [tri(l.dG) for l in ls]
        assert min(sizes) == lo and max(sizes) == hi


def test_densenet201_matches_paper_table():
    L, As, Gs, _, _ = _gold()["densenet201"]
    ls = shapes.densenet_layers(conv_bias=0)
    assert len(ls) == L
    tri = lambda d: d * (d + 1) // 2
    assert abs(sum(tri(l.c_in * l.kh * l.kw) for l in ls) / 1e6 - As) < 0.06
    assert abs(sum(tri(l.dG) for l in ls) / 1e6 - Gs) < 0.06
    cfg = shapes.config_layers("d201")
    assert len(cfg) == 201 and cfg[0].n == 16                       # the paper's per-GPU batch for this model
    assert cfg[-1].dA == 1921 and max(l.dA for l in cfg) == 1921
    assert sum(l.kind == 1 and l.kh == 3 and l.dA == 1153 for l in cfg) == 98


def test_inception_v4_matches_paper_table():
    L, As, Gs, _, _ = _gold()["inceptionv4"]
    ls = shapes.inception_v4_layers(conv_bias=0)
    assert len(ls) == L
    tri = lambda d: d * (d + 1) // 2
    assert abs(sum(tri(l.c_in * l.kh * l.kw) for l in ls) / 1e6 - As) < 0.06
    assert abs(sum(tri(l.dG) for l in ls) / 1e6 - Gs) < 0.06
    cfg = shapes.config_layers("iv4")
    assert len(cfg) == 150 and cfg[0].n == 16
    by = {l.name: l for l in cfg}
    # 224 -> 111 -> 109 -> 54 -> 52 -> 25 (Inception-A) -> 12 (B) -> 5 (C); padded 1x7 / 7x1 keep the size
    assert (by["stem.c2"].h, by["stem.3a"].h, by["stem.4a.b0c1"].h, by["stem.5a"].h) == (111, 109, 54, 52)
    assert (by["A0.b0"].h, by["B0.b0"].h, by["C0.b0"].h) == (25, 12, 5)
    l17 = by["B3.b1c2"]
    assert (l17.kh, l17.kw, l17.ph, l17.pw, l17.oh, l17.ow) == (1, 7, 0, 3, 12, 12)


def test_r50_config_dims():
    ls = shapes.config_layers("r50")
    assert len(ls) == 54
    assert ls[0].dA == 148 and ls[0].R == 32 * 112 * 112
    assert max(l.dA for l in ls) == 4609
    assert (ls[-1].dA, ls[-1].dG, ls[-1].R) == (2049, 1000, 32)
    f = shapes.flops(ls)
    assert abs(f["inverse"] / 1e12 - 0.453) < 1e-3
    assert abs((f["factor_a"] + f["factor_g"]) / 1e12 - 0.805) < 1e-3
    assert abs(f["precondition"] / 1e12 - 0.156) < 1e-3


def test_other_configs():
    assert [(l.dA, l.dG) for l in shapes.config_layers("fc")] == [(65, 32)]
    cnn = shapes.config_layers("cnn")
    assert [l.dA for l in cnn] == [28, 289, 577, 1153, 129]
    assert [l.dG for l in cnn] == [32, 64, 128, 128, 10]
    assert all(l.R == 32 * 32 * 32 for l in cnn[:4]) and cnn[4].R == 32
    assert len(shapes.config_layers("r152")) == 156
    b = shapes.config_layers("bertl")
    assert len(b) == 144 and {(l.dA, l.dG) for l in b} == {(1025, 1024), (1025, 4096), (4097, 1024)}
    assert all(l.R == 4096 for l in b)
