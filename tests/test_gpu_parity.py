"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Run with  -m gpu  on an MI355X."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the parity tests need the HIP path")
    from paper_2112_13935_amd import load_library
    load_library()
    from paper_2112_13935_amd.runner import Run
    return Run


def _both(gpu, wl, **kw):
    from oracle import Oracle
    return gpu(wl, **kw), Oracle(wl, "f64")


def report(name, worst):
    print(f"\n[parity] {name}: " + ", ".join(f"{k} {v:.2e}" if isinstance(v, float) else f"{k} {v}"
                                             for k, v in worst.items()), flush=True)


def test_sample_indices_bit_exact(gpu, oracle_libs):
    lib = oracle_libs.load("f64")
    wl = W.config1(n_clients=5, n_per=1000, d=16, rounds=2)
    sizes = [1, 2, 500, 999, 1000]
    for c, N in enumerate(sizes):
        wl.X[c] = wl.X[c][:N].copy()
        wl.y[c] = wl.y[c][:N].copy()
    run = gpu(wl)
    for c, N in enumerate(sizes):
        for q0, count in ((0, 4096), (123456789012, 1000), (2**40 + 5, 257), (7, 1)):
            got = run.lib.aet_debug_sample_indices(c, q0, count)
            want = np.array([lib.orc_sample_index(wl.seed, c, q0 + j, N) for j in range(count)],
                            dtype=np.int32)
            assert np.array_equal(got, want), (c, N, q0)
    run.close()


def small_cases():
    cases = {}
    wl = W.config1(n_clients=5, n_per=60, d=37, rounds=6, a=3, b=2)
    wl.compute_factor = np.array([1, 2, 1, 3, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 0, 1, 0, 1], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 3, 77
    cases["softmax_ragged_delays"] = wl
    wl = W.config2(n_clients=5, n_total=5 * 70, d=50, hidden=24, batch=4, rounds=6, a=4, b=8)
    wl.is_straggler = np.array([1, 0, 0, 1, 0], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 0, 2, 78
    cases["mlp_ragged_stragglers"] = wl
    wl = W.config3(n_clients=6, n_per=40, hw=16, batch=4, rounds=4, a=4, b=8)
    wl.compute_factor = np.array([1, 1, 2, 1, 4, 1], dtype=np.int32)
    cases["lenet16_factors_stragglers"] = wl
    wl = W.config4(n_clients=3, n_per=40, hw=8, width=8, fc=32, batch=4, rounds=3, a=4, b=8)
    cases["cnn8_factors"] = wl
    wl = W.config1(n_clients=3, n_per=30, d=20, rounds=4, a=5, b=0)
    cases["softmax_empty_first_round"] = wl
    wl = W.config2(n_clients=4, n_total=200, d=30, hidden=10, batch=2, rounds=5, a=2, b=2)
    wl.compute_factor = np.array([1, 3, 1, 2], dtype=np.int32)
    wl.d_max = 1
    cases["mlp_delay_checkpoint_d1"] = wl
    wl = W.config1(n_clients=1, n_per=50, d=10, rounds=5, a=2, b=3)
    wl.agg_scale = 1.0
    cases["one_client_plain_sgd"] = wl
    # shapes the fused dense-ReLU-dense kernel takes (hidden a multiple of 16, batch 16/32)
    wl = W.config2(n_clients=5, n_total=5 * 70, d=50, hidden=32, batch=16, rounds=5, a=16, b=32)
    wl.is_straggler = np.array([1, 0, 0, 1, 0], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 0, 2, 78
    wl.compute_factor = np.array([1, 2, 1, 1, 3], dtype=np.int32)
    cases["mlp_fused_b16_ragged_d"] = wl
    wl = W.config2(n_clients=11, n_total=11 * 90, d=100, hidden=48, batch=32, rounds=4, a=32, b=64)
    cases["mlp_fused_b32_11_clients"] = wl
    wl = W.config2(n_clients=3, n_total=3 * 200, d=784, hidden=128, batch=32, rounds=3, a=32, b=32)
    wl.compute_factor = np.array([1, 2, 1], dtype=np.int32)
    cases["mlp_fused_full_width"] = wl
    # the limits of the fused kernels: widest input and most unit groups of the
    # dense-ReLU-dense kernel (896 columns, 256 hidden units = 16 workgroups per client) ...
    wl = W.config2(n_clients=2, n_total=2 * 120, d=896, hidden=256, batch=16, rounds=3, a=16, b=16)
    cases["mlp_fused_widest"] = wl
    # wide inputs run two workgroups per unit group (half of the columns each): a width that
    # is not a multiple of 16 (ragged last tile in the second half), B = 16, and more clients
    # than fit one launch that way (20 x 8 x 2 workgroups: falls back to one per unit group)
    wl = W.config2(n_clients=3, n_total=3 * 100, d=777, hidden=64, batch=32, rounds=3, a=32, b=32)
    cases["mlp_fused_pair_ragged_width"] = wl
    wl = W.config2(n_clients=2, n_total=2 * 100, d=530, hidden=32, batch=16, rounds=3, a=16, b=16)
    cases["mlp_fused_pair_b16_ragged"] = wl
    wl = W.config2(n_clients=20, n_total=20 * 64, d=784, hidden=128, batch=32, rounds=2, a=32, b=32)
    cases["mlp_fused_wide_20_clients"] = wl
    # ... and of the softmax-regression kernel: 6 columns per thread with a ragged tail,
    # exactly 2 columns per thread, one column more than 1 per thread
    wl = W.config1(n_clients=3, n_per=40, d=3000, rounds=3, a=2, b=2)
    cases["softmax_3000_columns"] = wl
    wl = W.config1(n_clients=2, n_per=40, d=1024, rounds=3, a=2, b=2)
    cases["softmax_1024_columns"] = wl
    wl = W.config1(n_clients=2, n_per=40, d=513, rounds=3, a=2, b=2)
    cases["softmax_513_columns"] = wl
    # layer engine, dense layers with 16-byte aligned rows (the float4 kernels) and mini-batches
    # of 32 (two of four sample tiles real) and 64 (all four)
    wl = W.config2(n_clients=3, n_total=3 * 90, d=52, hidden=24, batch=32, rounds=3, a=32, b=32)
    cases["mlp_layers_aligned_b32"] = wl
    wl = W.config2(n_clients=2, n_total=2 * 150, d=36, hidden=40, batch=64, rounds=3, a=64, b=64)
    cases["mlp_layers_aligned_b64"] = wl
    # dense layers with aligned rows and small mini-batches (one sample tile), narrow and wide
    wl = W.config2(n_clients=5, n_total=5 * 60, d=36, hidden=20, batch=4, rounds=4, a=4, b=8)
    wl.compute_factor = np.array([1, 2, 1, 1, 3], dtype=np.int32)
    cases["mlp_layers_aligned_b4"] = wl
    wl = W.config2(n_clients=3, n_total=3 * 80, d=256, hidden=120, batch=16, rounds=3, a=16, b=16)
    cases["mlp_layers_256_120_b16"] = wl
    # shapes the fused LeNet round kernel takes (mini-batch 16, a cluster of four workgroups per
    # client): 16 x 16 images (one pooled pixel per channel in front of the dense layers) with
    # compute factors and stragglers, and the full 28 x 28 shape
    wl = W.config3(n_clients=5, n_per=60, hw=16, batch=16, rounds=4, a=16, b=32)
    wl.compute_factor = np.array([1, 2, 1, 3, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 1, 0, 0, 1], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 2, 11
    cases["lenet_fused_16x16_factors_stragglers"] = wl
    wl = W.config3(n_clients=3, n_per=80, hw=28, batch=16, rounds=3, a=16, b=16)
    cases["lenet_fused_28x28"] = wl
    wl = W.config3(n_clients=9, n_per=50, hw=20, batch=16, rounds=3, a=16, b=0)
    cases["lenet_fused_20x20_empty_first_round"] = wl
    # convolutions with 6 and 12 channels on 12 x 12 images: ragged channel groups in the
    # staging code, a pooling layer whose input rows are not 16-byte aligned (6 wide)
    wl = W.config4(n_clients=2, n_per=30, hw=12, width=6, fc=16, batch=4, rounds=3, a=4, b=4)
    cases["cnn12_six_channels"] = wl
    return cases


@pytest.mark.parametrize("name", list(small_cases()))
def test_small_cases_every_tick(gpu, oracle_libs, name):
    """Sizes the oracle finishes at once, ragged in every dimension (feature counts that
    are no multiple of the wavefront, odd client counts), with delays, compute factors,
    stragglers, an empty round, the delay checkpoint and the one-client case; U, w_c, the
    losses and the global model are compared after every tick."""
    from parity import lockstep
    wl = small_cases()[name]
    run, orc = _both(gpu, wl)
    worst = lockstep(wl, run, orc)
    report(name, worst)
    run.close()


@pytest.fixture
def select_kernels():
    """aet_test_select_kernels for one test; the defaults come back afterwards."""
    from paper_2112_13935_amd import load_library
    lib = load_library()
    yield lib.aet_test_select_kernels
    lib.aet_test_select_kernels(0, 0)


def test_layer_engine_on_fused_shapes(gpu, oracle_libs, select_kernels):
    """The layer-by-layer engine on a shape the fused kernel would take: both code paths
    have to match the oracle."""
    from parity import lockstep
    select_kernels(1, 0)
    wl = small_cases()["mlp_fused_b16_ragged_d"]
    run, orc = _both(gpu, wl)
    report("layer engine on mlp_fused_b16_ragged_d", lockstep(wl, run, orc))
    run.close()


@pytest.mark.parametrize("name", ["lenet16_factors_stragglers", "cnn8_factors", "mlp_ragged_stragglers"])
def test_plain_layer_kernels(gpu, oracle_libs, select_kernels, name):
    """The plain FMA layer kernels (the matrix-core ones switched off) against the oracle."""
    from parity import lockstep
    select_kernels(0, 1)
    wl = small_cases()[name]
    run, orc = _both(gpu, wl)
    report("plain layer kernels on " + name, lockstep(wl, run, orc))
    run.close()


def test_U_invariant_on_gpu(gpu):
    """w_start - w_end = eta_i U_i holds for the GPU's own numbers (fp32 rounding)."""
    wl = small_cases()["mlp_fused_b16_ragged_d"]
    run = gpu(wl)
    while not run.lib.aet_all_done(wl.rounds):
        w_start = run.lib.aet_get_weights(-1).astype(np.float64)
        for c, k in run.run_round():
            info = run.lib.aet_get_round_info(c, k)
            U = run.lib.aet_get_U(c, k).astype(np.float64)
            w_end = run.lib.aet_get_weights(c).astype(np.float64)
            err = np.abs((w_start - w_end) / info["eta"] - U).max()
            assert err <= 1e-4 * max(1.0, np.abs(U).max())
        run.server_aggregate()
    run.close()


def test_run_ticks_equals_tick_by_tick(gpu):
    """aet_run_ticks is the same loop as calling the two entry points per tick."""
    wl = small_cases()["mlp_fused_b16_ragged_d"]
    a = gpu(wl)
    ticks_a = a.run_all()
    b = gpu(wl)
    ticks_b = b.run_ticks()
    assert ticks_a == ticks_b
    assert np.array_equal(a.lib.aet_get_weights(-1), b.lib.aet_get_weights(-1))
    assert b.lib.aet_all_done(wl.rounds)
    # a second job after aet_reset gives the same bits again
    b.lib.aet_reset()
    assert b.run_ticks() == ticks_b
    assert np.array_equal(a.lib.aet_get_weights(-1), b.lib.aet_get_weights(-1))
    a.close()
    b.close()


def test_deterministic_rerun(gpu):
    """Two runs of the same workload give bit-identical results."""
    wl = small_cases()["lenet16_factors_stragglers"]
    out = []
    for _ in range(2):
        run = gpu(wl)
        run.run_all()
        out.append(run.lib.aet_get_weights(-1))
        run.close()
    assert np.array_equal(out[0], out[1])


def test_config1_full(gpu, oracle_libs):
    from parity import lockstep
    wl = W.config1()
    run, orc = _both(gpu, wl)
    report("config 1 (4 clients, 20 rounds)", lockstep(wl, run, orc))
    run.close()


def test_config2_full_clients_20_rounds(gpu, oracle_libs):
    from parity import TOL, lockstep
    wl = W.config2()
    run, orc = _both(gpu, wl)
    worst = lockstep(wl, run, orc, rounds=20, check_every=5)
    report("config 2 (16 clients, 20 rounds; U and w_c every fifth tick)", worst)
    assert worst["Wg"] <= TOL          # the global model meets the flat bar after 20 rounds
    run.close()


@pytest.mark.timeout(600)
def test_config3_full_clients_20_rounds(gpu, oracle_libs):
    from parity import TOL, lockstep
    wl = W.config3()
    run, orc = _both(gpu, wl)
    worst = lockstep(wl, run, orc, rounds=20, check_every=5)
    report("config 3 (64 clients, 20 rounds; U and w_c every fifth tick)", worst)
    assert worst["Wg"] <= TOL          # the global model meets the flat bar after 20 rounds
    run.close()


def test_config3_every_recursion_from_a_common_start(gpu, oracle_libs):
    """LeNet at its full layer shapes, all 64 clients: rounds of one recursion each (a = 0,
    b = B), every tick restarted from the oracle's global model, so each mini-batch gradient,
    update and aggregation is compared on its own."""
    from parity import lockstep
    wl = W.config3(rounds=6, a=0, b=16)
    run, orc = _both(gpu, wl)
    report("config 3, single recursions from a common start", lockstep(wl, run, orc, resync=True))
    run.close()


def test_config4_full_layer_shapes(gpu, oracle_libs):
    """The full 32x32x3 network and mini-batch 64, at 3 clients and 2 rounds (the oracle
    needs 0.1 s per sample for this model)."""
    from parity import lockstep
    wl = W.config4(n_clients=3, n_per=200, rounds=2)
    wl.compute_factor = np.array([1, 2, 1], dtype=np.int32)
    run, orc = _both(gpu, wl)
    report("config 4 shapes (3 clients, 2 rounds)", lockstep(wl, run, orc))
    run.close()


def test_config4_every_recursion_from_a_common_start(gpu, oracle_libs):
    """The CNN at its full layer shapes and B = 64: rounds of one recursion each, restarted
    from the oracle's global model after every tick."""
    from parity import lockstep
    wl = W.config4(n_clients=4, n_per=300, rounds=3, a=0, b=64)
    wl.compute_factor = None
    run, orc = _both(gpu, wl)
    report("config 4, single recursions from a common start", lockstep(wl, run, orc, resync=True))
    run.close()


@pytest.mark.timeout(900)
def test_config4_full_size_first_two_ticks(gpu, oracle_libs):
    """The CNN workload at full size in the launch configuration the benchmark times: all 32
    clients, B = 64.  Tick 0: round 0 of every client against the oracle (U, w_c, loss,
    bookkeeping), then the first aggregation at P = 1.12 M.  Tick 1: round 1 of the clients
    whose compute factor is 1, from the aggregated model, and the second aggregation."""
    from parity import lockstep
    wl = W.config4()
    run, orc = _both(gpu, wl)
    worst = lockstep(wl, run, orc, stop_after_ticks=2)
    report("config 4 at full size, ticks 0 and 1 (all 32 clients)", worst)
    assert orc.tick == 2 and sum(orc.history(c) for c in range(wl.n_clients)) > 0
    run.close()


@pytest.mark.timeout(900)
def test_config4_reduced_20_rounds(gpu, oracle_libs):
    """Same architecture at 16x16 images and half width, 6 clients with compute factors,
    20 rounds; all sides restart from the oracle's global model after every tick (a
    free-running CNN run of this length drifts by its own rounding: see parity.py)."""
    from parity import lockstep
    wl = W.config4(n_clients=6, n_per=300, hw=16, width=16, fc=64, batch=16, rounds=20, a=16, b=32)
    run, orc = _both(gpu, wl)
    report("config 4 reduced (6 clients, 20 rounds, common start per tick)",
           lockstep(wl, run, orc, resync=True))
    run.close()


def test_config4_reduced_free_running_8_rounds(gpu, oracle_libs):
    """The same workload left to itself for 8 rounds."""
    from parity import lockstep
    wl = W.config4(n_clients=6, n_per=300, hw=16, width=16, fc=64, batch=16, rounds=8, a=16, b=32)
    run, orc = _both(gpu, wl)
    report("config 4 reduced (6 clients, 8 rounds, free running)", lockstep(wl, run, orc, check_every=2))
    run.close()


@pytest.mark.timeout(900)
def test_config5_full_clients_20_rounds(gpu, oracle_libs):
    """All 1,024 clients and 3,072 features, the 20 rounds the tolerance is defined on
    (stragglers with delays up to 5 ticks are in flight throughout): losses of every round,
    U and w_c of every client every fifth tick, every client's model and the global model at
    the end."""
    from parity import lockstep
    wl = W.config5(rounds=20)
    run, orc = _both(gpu, wl)
    report("config 5 (1024 clients, 20 rounds)", lockstep(wl, run, orc, check_every=5))
    run.close()


def _final_state_check(wl, run, orc, name, clients):
    """Whole job through aet_run_ticks, twice (aet_reset in between, as the benchmark does),
    against the oracle's end state: global model, sampled clients' models, histories."""
    from parity import TOL, tensor_relerrs
    ticks_o = orc.run_all()
    worst = {}
    for attempt in range(2):
        if attempt:
            run.lib.aet_reset()
        assert run.run_ticks() == ticks_o
        assert run.lib.aet_all_done(wl.rounds) and run.lib.aet_inflight() == 0
        e = max(tensor_relerrs(wl.model, run.lib.aet_get_weights(-1), orc.get_weights(-1)))
        worst["Wg"] = max(worst.get("Wg", 0.0), e)
        for c in clients:
            e = max(tensor_relerrs(wl.model, run.lib.aet_get_weights(c), orc.get_weights(c)))
            worst["w_c"] = max(worst.get("w_c", 0.0), e)
            assert run.lib.aet_history(c) == orc.history(c) == wl.rounds
            for k in (0, wl.rounds - 1):
                io, ig = orc.round_info(c, k), run.lib.aet_get_round_info(c, k)
                for key in ("s", "m", "q0", "t0", "start_tick", "arrival"):
                    assert ig[key] == io[key], (c, k, key)
                worst["loss"] = max(worst.get("loss", 0.0), abs(ig["loss"] - io["loss"]) / max(abs(io["loss"]), 1e-12))
    report(name, worst)
    assert all(v <= TOL for v in worst.values()), worst


def test_config2_whole_job_as_benchmarked(gpu, oracle_libs):
    """The benchmark's workload at full size in the benchmark's launch configuration:
    all 16 clients, all 50 rounds, one aet_run_ticks call per job."""
    wl = W.config2()
    run, orc = _both(gpu, wl)
    _final_state_check(wl, run, orc, "config 2 whole job (16 clients, 50 rounds, aet_run_ticks)", range(16))
    run.close()


def test_config2_ring_whole_job_as_benchmarked(gpu, oracle_libs):
    wl = W.config2()
    wl.agg_scale = 1.0 / 3.0
    wl.topology = W.ring_topology(wl.n_clients)
    run, orc = _both(gpu, wl)
    _final_state_check(wl, run, orc, "config 2 on a ring, whole job (aet_run_ticks)", range(16))
    run.close()


def test_set_weights_round_trip(gpu):
    """aet_set_weights / aet_get_weights for the global model and a client's model."""
    wl = small_cases()["mlp_ragged_stragglers"]
    run = gpu(wl)
    rng = np.random.default_rng(5)
    a = rng.standard_normal(run.lib.P).astype(np.float32)
    b = rng.standard_normal(run.lib.P).astype(np.float32)
    run.lib.aet_set_weights(-1, a)
    run.lib.aet_set_weights(2, b)
    assert np.array_equal(run.lib.aet_get_weights(-1), a)
    assert np.array_equal(run.lib.aet_get_weights(2), b)
    assert np.array_equal(run.lib.aet_get_weights(1), wl.w0)
    # the next round starts from the imported global model
    run.run_round()
    assert not np.array_equal(run.lib.aet_get_weights(1), wl.w0)
    run.close()


def test_error_paths(gpu):
    """Bad arguments come back as status codes and leave the context usable."""
    from paper_2112_13935_amd import AetError
    wl = small_cases()["mlp_ragged_stragglers"]
    run = gpu(wl)
    with pytest.raises(AetError) as e:
        run.lib.aet_run_round(4, 6, wl.rounds, wl.eta0, wl.beta, wl.power)   # 6 % batch(4) != 0
    assert e.value.status == -1
    with pytest.raises(AetError):
        run.lib.aet_run_round(4, 8, wl.rounds, -1.0, 0.0, 1.0)
    with pytest.raises(AetError):
        run.lib.aet_run_round(4, 8, wl.rounds, 0.01, 0.0, 1.0, delay_min=2, delay_max=1)
    with pytest.raises(AetError) as e:
        run.lib.aet_get_U(0, 0)
    assert e.value.status == -4
    assert run.lib.aet_tick() == 0
    assert run.run_round() == [(c, 0) for c in range(5)]
    run.close()
