"""Pins for the oracle's integer side: counter hash, sample indices, thresholds,
step-size schedule.  None of these tests needs a GPU."""
import math
import os

import numpy as np
import pytest

import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")
M64 = (1 << 64) - 1


def _lines(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_splitmix64_published_vector(oracle_libs):
    """The hash underneath every index is SplitMix64: its first outputs for seed 1234567
    are published."""
    lib = oracle_libs.load("f64")
    want = [int(v[0]) for v in _lines("splitmix64_seed1234567.txt")]
    got = [lib.orc_draw(1234567, k) for k in range(len(want))]
    assert got == want


def test_stream_is_three_nested_draws(oracle_libs):
    """stream(seed, tag, c, ctr) = draw(draw(draw(seed, tag), c), ctr), checked with
    Python's unbounded integers reduced mod 2^64."""
    lib = oracle_libs.load("f64")

    def draw(seed, k):
        z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & M64
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)

    rng = np.random.default_rng(0)
    for _ in range(200):
        seed = int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2))
        tag, c, ctr = int(rng.integers(0, 4)), int(rng.integers(0, 2000)), int(rng.integers(0, 2**40))
        assert lib.orc_stream(seed, tag, c, ctr) == draw(draw(draw(seed, tag), c), ctr)


def test_sample_index_range_purity_and_map(oracle_libs):
    lib = oracle_libs.load("f64")
    seed = 99
    for N in (1, 2, 3, 500, 1000, 3750, 2**31 - 1):
        idx = [lib.orc_sample_index(seed, 3, q, N) for q in range(300)]
        assert min(idx) >= 0 and max(idx) < N
        # pure function of (seed, c, q): asking again, in another order, changes nothing
        again = [lib.orc_sample_index(seed, 3, q, N) for q in reversed(range(300))]
        assert again[::-1] == idx
        # multiply-shift map of the hash's top 32 bits, in exact integer arithmetic
        for q in (0, 7, 299):
            h = lib.orc_stream(seed, 0, 3, q)
            assert idx[q] == ((h >> 32) * N) >> 32
    # different clients and different seeds give different streams
    a = [lib.orc_sample_index(seed, 0, q, 1000) for q in range(64)]
    b = [lib.orc_sample_index(seed, 1, q, 1000) for q in range(64)]
    c = [lib.orc_sample_index(seed + 1, 0, q, 1000) for q in range(64)]
    assert a != b and a != c


def test_sample_index_uniform(oracle_libs):
    """Algorithm 2, sampling step (a uniform draw from the client's shard): chi-square on 200,000 draws over 100 bins
    (99 degrees of freedom; 160 is far beyond the 99.99th percentile)."""
    lib = oracle_libs.load("f64")
    N, draws = 100, 200000
    counts = np.zeros(N)
    for q in range(draws):
        counts[lib.orc_sample_index(12345, 7, q, N)] += 1
    chi2 = ((counts - draws / N) ** 2 / (draws / N)).sum()
    assert chi2 < 160.0
    # consecutive draws are not correlated in the crudest way: lag-1 pairs cover the grid
    pairs = {(lib.orc_sample_index(12345, 7, q, 10), lib.orc_sample_index(12345, 7, q + 1, 10))
             for q in range(5000)}
    assert len(pairs) == 100


def test_net_delay_range_and_purity(oracle_libs):
    lib = oracle_libs.load("f64")
    seen = set()
    for c in range(40):
        for k in range(40):
            d = lib.orc_net_delay(5, c, k, 1, 3)
            assert 1 <= d <= 3
            assert d == lib.orc_net_delay(5, c, k, 1, 3)
            seen.add(d)
    assert seen == {1, 2, 3}
    assert all(lib.orc_net_delay(5, c, 0, 2, 2) == 2 for c in range(10))


def test_threshold_is_linear(oracle_libs):
    lib = oracle_libs.load("f64")
    for a, b in ((10, 10), (32, 64), (16, 32), (64, 128), (5, 5), (10, 0), (0, 7)):
        s = [lib.orc_threshold(a, b, i) for i in range(70)]
        assert s == [a * i + b for i in range(70)]
        # closed form of the total: a R (R-1)/2 + b R
        for R in (1, 20, 60):
            assert sum(s[:R]) == a * R * (R - 1) // 2 + b * R


def test_config_totals_match_closed_forms(oracle_libs):
    """Samples per client of the five configurations: 2100, 42400, 13760, 31680, 9150."""
    lib = oracle_libs.load("f64")
    cases = {(10, 10, 20): 2100, (32, 64, 50): 42400, (16, 32, 40): 13760,
             (64, 128, 30): 31680, (5, 5, 60): 9150}
    for (a, b, R), want in cases.items():
        assert sum(lib.orc_threshold(a, b, i) for i in range(R)) == want


def test_round_counts_printed_in_the_paper(oracle_libs):
    lib = oracle_libs.load("f64")
    for a, b, K, rounds, where in _lines("paper_round_counts.txt"):
        got = lib.orc_rounds_needed(int(a), int(b), int(K))
        if where == "table1_threshold6":
            assert got in (int(rounds) - 1, int(rounds)), where
        else:
            assert got == int(rounds), where
    # T grows like sqrt(K) for the linear sequence and like K for a constant one
    assert lib.orc_rounds_needed(10, 0, 4 * 60000) < 2.05 * lib.orc_rounds_needed(10, 0, 60000)
    assert lib.orc_rounds_needed(0, 100, 4 * 60000) == 4 * lib.orc_rounds_needed(0, 100, 60000)
    # K = ceil(K_total / n) iterations per node (caption of the node-count table)
    for n, want in ((1, 60000), (2, 30000), (5, 12000), (10, 6000), (15, 4000)):
        assert math.ceil(60000 / n) == want


def test_eta_schedule(oracle_libs):
    lib = oracle_libs.load("f64")
    # beta = 0: constant
    assert all(lib.orc_eta(0.01, 0.0, 0.5, t) == 0.01 for t in (0, 1, 10**6))
    # the paper's scheme eta0 / (1 + beta sqrt(t)), Table 5 values
    assert lib.orc_eta(0.01, 0.01, 0.5, 0) == 0.01
    assert lib.orc_eta(0.01, 0.01, 0.5, 10000) == pytest.approx(0.01 / 2.0, rel=1e-15)
    assert lib.orc_eta(0.01, 0.01, 0.5, 60000) == pytest.approx(0.01 / (1 + 0.01 * math.sqrt(60000)),
                                                                rel=1e-15)
    # power = 1 (the MLP configuration): 0.05 / (1 + 0.001 t)
    assert lib.orc_eta(0.05, 0.001, 1.0, 1000) == pytest.approx(0.025, rel=1e-15)
    seq = [lib.orc_eta(0.05, 0.001, 1.0, t) for t in range(0, 2000, 37)]
    assert all(x > y for x, y in zip(seq, seq[1:]))


def test_param_counts(oracle_libs):
    """Parameter counts of the five models: 7850, 101770, 44426, 1116970, 30730."""
    from oracle.oracle import _c_model
    import ctypes as C
    lib = oracle_libs.load("f64")
    cases = [(W.softmax_model(784, 10), 7850), (W.mlp_model(784, 128, 10, 32), 101770),
             (W.lenet_model(16), 44426), (W.cnn32_model(64), 1116970),
             (W.softmax_model(3072, 10), 30730)]
    for model, want in cases:
        cm = _c_model(model)
        assert lib.orc_n_params(C.byref(cm)) == want
        assert model.n_params() == want
