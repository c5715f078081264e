"""The synthetic payload shapes: counts that the published architectures fix, and seeding."""
import numpy as np

from paper_1711_00705_amd import workloads as wl


def test_payload_shapes():
    r = wl.resnet50_sizes()
    assert len(r) == 161 and sum(r) == 25_557_032 and min(r) == 64 and max(r) == 2_359_296
    assert all(s % 4 == 0 for s in r)
    v = wl.vgg16_sizes()
    assert len(v) == 32 and sum(v) == 138_357_544 and max(v) == 25088 * 4096
    g = wl.googlenet_sizes()
    assert len(g) == 116 and sum(g) == 6_998_552 and min(g) == 16 and max(g) == 1_024_000
    t, seed = wl.tiny_sizes()
    assert len(t) == 12 and sum(t) <= 262_144 and all(1 <= s <= 65536 for s in t)
    assert any(s % 4 for s in t), "Tiny must exercise misaligned offsets"
    assert wl.tiny_sizes() == (t, seed)


def test_configurations():
    cfg = {n: wl.workload(n) for n in wl.WORKLOADS}
    assert (cfg["tiny"].P, cfg["tiny"].k) == (4, 2)
    assert (cfg["resnet50"].P, cfg["resnet50"].k, cfg["resnet50"].lr, cfg["resnet50"].wd) == (4, 4, 0.1, 1e-4)
    assert (cfg["resnet50_heavy"].P, cfg["resnet50_heavy"].k, cfg["resnet50_heavy"].heavy_tail) == (8, 8, True)
    assert (cfg["vgg16"].P, cfg["vgg16"].k, cfg["vgg16"].lr, cfg["vgg16"].wd) == (4, 4, 0.01, 5e-4)
    assert (cfg["googlenet"].P, cfg["googlenet"].k, cfg["googlenet"].steps) == (4, 8, 100)


def test_values_are_seeded_and_distinct():
    sizes = [1000, 3, 50000]
    a = wl.contribution_tensors(sizes, 0)
    b = wl.contribution_tensors(sizes, 0)
    c = wl.contribution_tensors(sizes, 1)
    d = wl.contribution_tensors(sizes, 0, step=1)
    for x, y in zip(a, b):
        assert np.array_equal(x, y) and x.dtype == np.float32
    assert not np.array_equal(a[2], c[2]) and not np.array_equal(a[2], d[2])
    big = np.concatenate(a)
    assert abs(float(big.std()) - 1e-3) < 5e-5 and abs(float(big.mean())) < 2e-5
    h = np.concatenate(wl.contribution_tensors([400000], 2, heavy_tail=True))
    frac = float((np.abs(h) > 6e-3).mean())          # 100x outliers: about 1 % of the elements
    assert 0.005 < frac < 0.015
    w = np.concatenate(wl.weight_tensors(sizes))
    assert abs(float(w.std()) - 0.05) < 2e-3
    o = wl.rotation_order(5, 4)
    assert o.shape == (5, 4) and all(sorted(r) == [0, 1, 2, 3] for r in o.tolist()) and o[1].tolist() == [1, 2, 3, 0]
