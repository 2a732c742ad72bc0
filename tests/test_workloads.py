"""Shapes and seeds of the synthetic workloads (Table 2 for the model sizes)."""
import os

import numpy as np

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table2_param_counts.txt")


def _table2():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, depth, n = line.split()
        out[name] = (int(depth), int(n))
    return out


def test_model_sizes_match_table2():
    t = _table2()
    assert sum(wl.alexnet_counts()) == t["AlexNet"][1] == wl.ALEXNET_PARAMS
    assert len(wl.ALEXNET_SHAPES) == 2 * t["AlexNet"][0]
    assert sum(wl.vggnet_counts()) == t["VGGNet"][1] == wl.VGGNET_PARAMS
    assert wl.GOOGLENET_PARAMS == t["GoogLeNet"][1]
    assert sum(wl.googlenet_scale_counts(1)) == t["GoogLeNet"][1]


def test_many_small_recipe():
    c = wl.many_small_counts(wl.BASE_SEED + 4)
    assert len(c) == 116 and sum(c) == 7_000_000 and min(c) >= 1
    assert c == wl.many_small_counts(wl.BASE_SEED + 4)          # reproducible
    assert c != wl.many_small_counts(wl.BASE_SEED + 5)
    assert sum(1 for x in c if x % 8) > 50                      # ragged on purpose


def test_draws_are_seeded_and_distinct():
    counts = [1000, 7, 333]
    a = wl.gaussian_tensors(counts, 0.01, 5, "grad", worker=1, step=2)
    b = wl.gaussian_tensors(counts, 0.01, 5, "grad", worker=1, step=2)
    c = wl.gaussian_tensors(counts, 0.01, 5, "grad", worker=2, step=2)
    assert [x.size for x in a] == counts
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not np.array_equal(a[0], c[0])
    big = wl.gaussian_tensors([400_000], 0.01, 9, "grad")[0]
    assert big.dtype == np.float32 and abs(big.std() - 0.01) < 2e-4 and abs(big.mean()) < 1e-4


def test_worker_orders_are_permutations():
    o = wl.worker_orders(3, 8, 100)
    assert o.shape == (100, 8)
    assert all(sorted(r) == list(range(8)) for r in o.tolist())
    assert len({tuple(r) for r in o.tolist()}) > 90


def test_five_configs():
    for i in range(1, 6):
        c = wl.config(i)
        assert c.n == sum(c.counts)
    assert wl.config(1).n == 1_048_576 and wl.config(1).k == 2
    assert wl.config(3).k == 8 and wl.config(3).transfer == "f16"
    assert wl.config(5).alpha == 0.0625 and wl.config(5).rounds == 100
