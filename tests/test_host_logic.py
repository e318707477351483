"""Host-side logic that needs no GPU: the seeded input generators, the bench's argument
handling and byte accounting, and the rule that the product path never touches the oracle."""
import ast
import json
import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2305_16513_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("cfg,shape,wshape", [(1, (1, 1, 4096), (1, 1, 5)), (2, (2, 64, 128), (64, 64, 3)),
                                              (3, (1, 2, 16, 16), None), (4, (1, 64, 8, 8), (64, 64, 3, 3)),
                                              (5, (2, 128, 256), (128, 1, 31)), (6, (2, 1, 512), (1, 1, 51)),
                                              (7, (1, 4, 900), (4, 1, 51))])
def test_generators_are_seeded_clean_and_shaped(cfg, shape, wshape):
    x1, w1 = workloads.make(cfg, x_shape=shape, wgt_shape=wshape)
    x2, w2 = workloads.make(cfg, x_shape=shape, wgt_shape=wshape)
    assert x1.dtype == np.float32 and x1.shape == shape and np.array_equal(x1, x2)
    workloads.check_clean(x1)
    if wshape:
        assert w1.shape == wshape and np.array_equal(w1, w2)
        workloads.check_clean(w1)
    x3, _ = workloads.make(cfg, x_shape=shape, wgt_shape=wshape, seed_offset=1)
    assert not np.array_equal(x1, x3)                       # another seed, other bits
    if workloads.CONFIGS[cfg].x_dist == "uniform":
        assert -1.0 <= x1.min() and x1.max() < 1.0
    if workloads.CONFIGS[cfg].x_dist == "relu":
        assert x1.min() == 0.0


def test_full_size_shapes_match_the_named_configurations():
    c = workloads.CONFIGS
    assert c[1].x_shape == (1, 1, 1048576) and c[2].x_shape == (16, 64, 4096) and c[2].wgt_shape == (64, 64, 3)
    assert c[3].x_shape == (32, 64, 112, 112) and c[4].wgt_shape == (64, 64, 3, 3)
    assert c[5].x_shape == (256, 128, 16384) and c[5].wgt_shape == (128, 1, 31)
    assert abs(c[5].wgt_std ** 2 - 1 / 31) < 1e-12 and abs(c[4].wgt_std ** 2 - 2 / 576) < 1e-12


def test_pair_generator_keeps_long_products_in_range():
    u, v = workloads.make_pairs((4, 4096))
    u2, _ = workloads.make_pairs((4, 4096))
    assert np.array_equal(u, u2) and u.dtype == np.float32 and v.dtype == np.float32
    workloads.check_clean(u)
    workloads.check_clean(v)
    assert 0.97 <= np.abs(u).min() and np.abs(u).max() <= 1.03 + 1e-6
    assert 0.1 < (u < 0).mean() < 0.3
    assert np.isfinite(np.prod(np.abs(u[:, :961]).astype(np.float32), axis=1)).all()


def test_check_clean_rejects_negative_zero_and_non_finite():
    with pytest.raises(ValueError):
        workloads.check_clean(np.array([1.0, -0.0], np.float32))
    with pytest.raises(ValueError):
        workloads.check_clean(np.array([np.inf], np.float32))
    workloads.check_clean(workloads.integer_valued((3, 7), -4, 4, seed=1))


def test_bench_refuses_more_than_one_gpu():
    env = dict(os.environ, WORLD_SIZE="1")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       env=env, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
    assert not any(line.startswith("{") for line in r.stdout.splitlines())


def test_bench_byte_accounting():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.slide_bytes(32768, 16384, 16) == 4293001216          # the per-launch figures of configuration 5
    assert bench.slide_bytes(32768, 16384, 64) == 4286709760
    assert bench.slide_bytes(32768, 16384, 255) == 4261675008
    assert bench.slide_bytes(32768, 16384, 31) + 4 * 128 * 31 == 4291051008
    assert bench.read_traffic("no_such_profile.txt") is None
    t = bench.read_traffic("slide_scan_cfg5_hbm_traffic.txt")
    assert t is None or 4.2e9 < t < 4.6e9


def _imports(path):
    tree = ast.parse(open(path).read())
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
            names.add(node.module.split(".")[0])
    return names


def test_product_path_never_imports_the_oracle_and_the_oracle_never_imports_the_product():
    pkg = os.path.join(ROOT, "paper_2305_16513_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            assert "oracle" not in _imports(os.path.join(pkg, f)), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2305_16513_amd" not in _imports(os.path.join(ROOT, "oracle", f)), f
    csrc = os.path.join(pkg, "csrc")
    for f in os.listdir(csrc):
        assert "sws_ref" not in open(os.path.join(csrc, f)).read(), f


def test_missing_library_is_an_error_not_a_fallback(tmp_path, monkeypatch):
    from paper_2305_16513_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libsws.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()
