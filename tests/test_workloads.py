"""The seeded input generators (shared by the oracle and the HIP path; they hold none of the
method's arithmetic): shapes, determinism, topology builders.  No GPU needed."""
import numpy as np
import pytest

import workloads as W


@pytest.mark.parametrize("k, n, P, B, total", [
    (1, 4, 7850, 1, 8400),
    (2, 16, 101770, 32, 678400),
    (3, 64, 44426, 16, 880640),
])
def test_config_sizes_match_the_scope_table(k, n, P, B, total):
    wl = W.CONFIGS[k]()
    assert wl.n_clients == n and wl.model.n_params() == P and wl.model.batch == B
    assert wl.total_client_samples() == total
    assert len(wl.X) == n and all(x.dtype == np.float32 and x.flags.c_contiguous for x in wl.X)
    assert all(y.dtype == np.int32 and y.min() >= 0 and y.max() < 10 for y in wl.y)
    assert wl.w0.dtype == np.float32 and wl.w0.size == P
    for i in range(wl.rounds):
        assert (wl.a * i + wl.b) % B == 0


def test_big_configs_shapes_without_building_them():
    m4 = W.cnn32_model(64)
    assert m4.n_params() == 1116970 and m4.in_size() == 3072
    m5 = W.softmax_model(3072, 10, 1)
    assert m5.n_params() == 30730


def test_generators_are_deterministic_and_seeded_per_config():
    a, b = W.config2(n_clients=4, n_total=400), W.config2(n_clients=4, n_total=400)
    for x, y in zip(a.X, b.X):
        assert np.array_equal(x, y)
    assert np.array_equal(a.w0, b.w0)
    c = W.config3(n_clients=4, n_per=100)
    assert a.seed != c.seed


def test_config3_is_non_iid_with_two_classes_per_client():
    wl = W.config3(n_clients=10, n_per=100)
    for c in range(10):
        assert set(np.unique(wl.y[c])) == {2 * (c % 5), 2 * (c % 5) + 1}


@pytest.mark.parametrize("n", [1, 2, 3, 7, 64])
def test_topology_builders_give_sorted_symmetric_lists(n):
    for build in (W.ring_topology, W.line_topology, W.complete_topology):
        off, nbr = build(n)
        assert off.dtype == np.int32 and nbr.dtype == np.int32 and off[0] == 0 and off[-1] == nbr.size
        for c in range(n):
            mine = nbr[off[c]:off[c + 1]]
            assert np.all(np.diff(mine) > 0) and c not in mine
            for v in mine:
                assert c in nbr[off[v]:off[v + 1]]
    off, _ = W.ring_topology(n)
    assert list(np.diff(off)) == [min(2, n - 1)] * n
    off, _ = W.complete_topology(n)
    assert list(np.diff(off)) == [n - 1] * n
