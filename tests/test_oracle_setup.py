"""Pins for the oracle's Setup (Algorithm 1): each recursion of global round i is assigned to
node c with probability p_c, and s_{i,c} counts node c's share.  No GPU needed."""
import ctypes as C

import numpy as np
import pytest

import workloads as W
from oracle import Oracle


def cum(weights):
    return np.cumsum(np.asarray(weights, dtype=np.uint64)).astype(np.uint64)


def owners(lib, seed, weights, i, count):
    cw = cum(weights)
    ptr = cw.ctypes.data_as(C.c_void_p)
    return np.array([lib.orc_setup_owner(C.c_uint64(seed), ptr, len(weights), i, t)
                     for t in range(count)], dtype=np.int64)


def small_softmax(n=4, rounds=5, a=8, b=12, **kw):
    wl = W.config1(n_clients=n, n_per=40, d=12, rounds=rounds, a=a, b=b)
    for k, v in kw.items():
        setattr(wl, k, v)
    return wl


def test_two_equal_nodes_follow_the_top_bit_of_the_hash(oracle_libs):
    """n = 2, equal weights: the multiply-shift onto [0, 2) is the top bit of the stream
    value (the stream itself is pinned by the SplitMix64 golden values)."""
    lib = oracle_libs.load("f64")
    seed = 4242
    got = owners(lib, seed, [1, 1], 3, 500)
    want = np.array([lib.orc_stream(C.c_uint64(seed), 2, 3, t) >> 63 for t in range(500)])
    assert np.array_equal(got, want)
    assert 0 < got.sum() < 500


def test_scaling_the_weights_changes_nothing(oracle_libs):
    """p_c depends on the ratios only: floor(h W / 2^32) >= cum  <=>  h >= cum 2^32 / W."""
    lib = oracle_libs.load("f64")
    a = owners(lib, 7, [1, 2, 5], 0, 3000)
    b = owners(lib, 7, [3, 6, 15], 0, 3000)
    c = owners(lib, 7, [1000, 2000, 5000], 0, 3000)
    assert np.array_equal(a, b) and np.array_equal(a, c)


def test_zero_weight_nodes_get_nothing_and_one_node_can_get_all(oracle_libs):
    lib = oracle_libs.load("f64")
    o = owners(lib, 1, [0, 3, 0, 1, 0], 2, 4000)
    assert set(np.unique(o)) == {1, 3}
    assert np.all(owners(lib, 1, [0, 0, 9], 5, 1000) == 2)
    assert np.all(owners(lib, 1, [9, 0, 0], 5, 1000) == 0)


def test_frequencies_follow_the_weights(oracle_libs):
    """E[s_{i,c}] = p_c s_i: chi-square of 200,000 flips against the weights (3 degrees of
    freedom; 30 is far beyond the 1e-5 quantile), and no memory between consecutive flips."""
    lib = oracle_libs.load("f64")
    w = np.array([1, 2, 5, 8])
    N = 200000
    o = owners(lib, 99, w, 11, N)
    cnt = np.bincount(o, minlength=4)
    exp = N * w / w.sum()
    assert ((cnt - exp) ** 2 / exp).sum() < 30.0
    pair = np.zeros((4, 4))
    np.add.at(pair, (o[:-1], o[1:]), 1)
    exp2 = (N - 1) * np.outer(w, w) / w.sum() ** 2
    assert ((pair - exp2) ** 2 / exp2).sum() < 60.0     # 9 degrees of freedom
    # different rounds and different seeds are different streams
    assert not np.array_equal(o[:1000], owners(lib, 99, w, 12, 1000))
    assert not np.array_equal(o[:1000], owners(lib, 98, w, 11, 1000))


@pytest.mark.parametrize("batch_case", ["per_sample", "mini_batch"])
def test_node_rounds_add_up_to_the_global_round(oracle_libs, batch_case):
    """sum_c s_{i,c} = s_i for every round; with mini-batches the unit handed out is one
    recursion, so every s_{i,c} is a multiple of the batch; the node's share is what
    orc_setup_owner says; delays and compute factors do not change it."""
    lib = oracle_libs.load("f64")
    if batch_case == "per_sample":
        wl = small_softmax(n=4, rounds=5, a=8, b=12)
    else:
        wl = W.config2(n_clients=4, n_total=200, d=20, hidden=8, batch=4, rounds=5, a=16, b=24)
    weights = np.array([1, 3, 0, 2], dtype=np.uint32)
    B = wl.model.batch
    lengths = []
    for variant in range(2):
        if variant == 1:
            wl.compute_factor = np.array([2, 1, 1, 3], dtype=np.int32)
            wl.is_straggler = np.array([0, 1, 0, 0], dtype=np.uint8)
            wl.delay_min, wl.delay_max, wl.delay_seed = 1, 2, 5
        o = Oracle(wl)
        o.set_setup(weights, 31337)
        o.run_all()
        tab = np.array([[o.round_info(c, i)["s"] for c in range(4)] for i in range(wl.rounds)])
        lengths.append(tab)
        for i in range(wl.rounds):
            s_i = wl.a * i + wl.b
            assert tab[i].sum() == s_i
            assert np.all(tab[i] % B == 0)
            own = owners(lib, 31337, weights, i, s_i // B)
            assert np.array_equal(tab[i], B * np.bincount(own, minlength=4))
            assert tab[i][2] == 0                      # weight 0
            for c in range(4):
                info = o.round_info(c, i)
                assert info["m"] * B == info["s"]
        # an empty round still posts a message, with U = 0 and nothing sampled
        assert o.history(2) == wl.rounds
        assert o.round_info(2, wl.rounds - 1)["q0"] == 0
    assert np.array_equal(lengths[0], lengths[1])


def test_sample_counters_follow_the_ragged_rounds(oracle_libs):
    """q0 and t0 of a round are the node's own running sums of s_{i,c} and m_{i,c}; the step
    size uses the node's own t."""
    wl = small_softmax(n=3, rounds=6, a=6, b=9, beta=0.1, power=0.5)
    o = Oracle(wl)
    o.set_setup(np.array([5, 1, 2], dtype=np.uint32), 8)
    o.run_all()
    for c in range(3):
        q = t = 0
        for i in range(6):
            info = o.round_info(c, i)
            assert info["q0"] == q and info["t0"] == t
            assert info["eta"] == pytest.approx(wl.eta0 / (1 + wl.beta * t ** wl.power), rel=1e-15)
            q += info["s"]
            t += info["m"]


def test_setup_errors(oracle_libs):
    wl = small_softmax(n=3, rounds=2)
    o = Oracle(wl)
    with pytest.raises(RuntimeError):
        o.set_setup(np.array([0, 0, 0], dtype=np.uint32), 1)
    with pytest.raises(RuntimeError):
        o.set_setup(np.array([2**31, 2**31, 1], dtype=np.uint32), 1)
    o.run_round()
    with pytest.raises(RuntimeError):
        o.set_setup(np.array([1, 1, 1], dtype=np.uint32), 1)
