"""CPU checks of the synthetic workloads (layout totals of the models the
configurations stand for) and of two repository rules: the product never
reaches into the oracle, and the oracle never into the product."""
import os
import re

import numpy as np

from workloads import CONFIGS, distinct_population, get_config, host_population, layouts

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_layout_totals():
    r18, r50, vit = layouts.resnet18_cifar(), layouts.resnet50_imagenet(), layouts.vit_b16()
    assert (len(r18), sum(t.numel for t in r18)) == (62, 11_173_962)
    assert (len(r50), sum(t.numel for t in r50)) == (161, 25_557_032)
    assert (len(vit), sum(t.numel for t in vit)) == (152, 86_567_656)
    assert min(t.numel for t in r18) == 10 and max(t.numel for t in r18) == 2_359_296
    assert sum(1 for t in r18 if t.numel < 4096) == 42 and sum(1 for t in r50 if t.numel < 4096) == 107
    assert r18[0].shape == (64, 3, 3, 3) and r50[0].shape == (64, 3, 7, 7) and vit[2].shape == (768, 3, 16, 16)
    flat = layouts.flat(1_100_000_000, 200)
    assert len(flat) == 200 and all(t.numel == 5_500_000 for t in flat)


def test_configs_as_listed():
    assert [c.N for c in CONFIGS] == [4, 5, 10, 20, 8]
    assert [c.P for c in CONFIGS] == [1 << 20, 11_173_962, 25_557_032, 86_567_656, 1_100_000_000]
    assert [c.momentum for c in CONFIGS] == [False, False, True, False, True]
    assert get_config(4).p_sweep == (1e-4, 1e-3, 1e-2, 1e-1)
    segs = get_config(5).segments()
    assert len(segs) == 200 and segs[0][2] == 0.05 and abs(segs[-1][2] - 0.001) < 1e-15
    assert abs(sum(p for _, _, p in segs) / 200 - 0.0255) < 1e-12
    for c in CONFIGS:                                    # segments tile the row without gaps
        s = c.segments()
        assert s[0][0] == 0 and s[-1][0] + s[-1][1] == c.P
        assert all(s[k][0] + s[k][1] == s[k + 1][0] for k in range(len(s) - 1))
    assert all(p == 0.001 for _, _, p in get_config(2).segments())
    assert all(p == 0.3 for _, _, p in get_config(2).segments(0.3))


def test_generators_are_seeded_and_shaped():
    t = layouts.resnet18_cifar()
    a, m = host_population(t, 3, "kaiming", seed=7, momentum=True)
    b, _ = host_population(t, 3, "kaiming", seed=7)
    assert a.shape == (3, 11_173_962) and a.dtype == np.float32 and np.array_equal(a, b)
    assert abs(m.std() - 1e-3) < 2e-5
    conv1 = a[:, :1728]                                  # 64x3x3x3, fan_out = 64*9
    assert abs(conv1.std() - np.sqrt(2.0 / 576)) < 0.005
    assert np.all(a[:, 1728:1792] == 1.0) and np.all(a[:, 1792:1856] == 0.0)     # bn1 weight, bias
    assert not np.array_equal(a[0, :1728], a[1, :1728])  # rows drawn independently
    v, _ = host_population([layouts.Tensor("w", (50, 100), "linear")], 2, "trunc002", seed=1)
    assert np.abs(v).max() <= 0.04 + 1e-7
    d = distinct_population(3, 1000)
    assert len(np.unique(d.view(np.uint32))) == 3000 and np.isfinite(d).all()


def _python_sources(folder):
    for dirpath, _, files in os.walk(os.path.join(ROOT, folder)):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".c")):
                yield os.path.join(dirpath, f)


def test_product_and_oracle_do_not_touch_each_other():
    for path in _python_sources("paper_2405_17517_amd"):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "wash_ref" not in text and "libwash_ref" not in text, path
    for path in _python_sources("oracle"):
        text = open(path).read()
        assert "paper_2405_17517_amd" not in text and "libwash_hip" not in text, path
        assert "hip/hip_runtime" not in text, path
    for path in _python_sources("workloads"):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+(oracle|paper_2405_17517_amd)\b", text, re.M), path


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr + res.stdout


def test_bench_store_unit_model():
    # expected distinct 64-byte half lines written by one shuffle launch: closed-form corner cases
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    units = bench._expected_store_units
    assert units([(0, 1600, 1.0)], 4, 1) == 100 * 3            # every half line of N - 1 rows
    assert units([(0, 1600, 0.0)], 4, 2) == 0
    small = units([(0, 16_000_000, 1e-6)], 2, 1)               # rare selections never share a half line
    assert abs(small - 16.0) < 1e-3
    assert abs(units([(0, 160, 0.5), (160, 160, 0.5)], 3, 2) - 2 * units([(0, 160, 0.5)], 3, 2)) < 1e-12
