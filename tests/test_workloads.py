"""The synthetic input recipes have the stated shapes and structure."""
import numpy as np

import workloads


def test_resnet50_tensor_table():
    shapes = workloads.resnet50_tensor_shapes()
    sizes = [int(np.prod(s)) for s in shapes]
    assert len(shapes) == 161 and sum(sizes) == 25557032
    assert min(sizes) == 64 and max(sizes) == 2359296 and all(s % 4 == 0 for s in sizes)
    assert shapes[0] == (64, 3, 7, 7) and shapes[-2] == (2048, 1000)


def test_mlp_param_counts_and_init():
    assert workloads.mlp_param_count([784, 256, 10]) == 203530
    assert workloads.mlp_param_count([3072, 1024, 1024, 10]) == 4206602
    t = workloads.mlp_init([784, 256, 10], np.random.default_rng(0))
    assert t.dtype == np.float32 and t.shape == (203530,)
    w1 = t[:784 * 256]
    assert abs(w1.std() - np.sqrt(2 / 784)) < 1e-3 and np.all(t[784 * 256:784 * 256 + 256] == 0)


def test_configs_are_seeded_and_shaped():
    a = workloads.config1(n_data=512, batch=64); b = workloads.config1(n_data=512, batch=64)
    assert np.array_equal(a["data"], b["data"]) and np.array_equal(a["idx"], b["idx"])
    assert len(set(a["idx"].tolist())) == 64          # permutation prefix: no duplicates
    c = workloads.config4(n_data=20, batch=16, chw=(3, 8, 8))
    assert c["data"].dtype == np.uint8 and c["data"].shape == (20, 3, 8, 8) and c["mean"].shape == (3,)
    d = workloads.config5(rows=256, classes=50, n_slices=4)
    assert d["logits"].shape == (256, 50) and abs(d["logits"].std() - 2.0) < 0.1
    e = workloads.config3(n_params=4096, n_workers=3)
    assert len(e["grads"]) == 3 and abs(e["grads"][0].std() - 1e-3) < 1e-4
