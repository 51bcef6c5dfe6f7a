"""GPU parity with round lengths from the coin flips of Algorithm 1 (Setup): ragged
s_{i,c}, empty rounds, inside the same launches.  Run with  -m gpu  on an MI355X."""
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


def report(name, worst):
    print(f"\n[parity] {name}: " + ", ".join(f"{k} {v:.2e}" if isinstance(v, float) else f"{k} {v}"
                                             for k, v in worst.items()), flush=True)


def setup_cases():
    cases = {}
    # per-sample softmax regression (fused round kernel), a node with weight 0
    wl = W.config1(n_clients=5, n_per=60, d=37, rounds=6, a=15, b=10)
    wl.compute_factor = np.array([1, 2, 1, 3, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 0, 1, 0, 1], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 3, 77
    wl.agg_scale = 1.0
    wl.setup_weights, wl.setup_seed = np.array([3, 1, 0, 2, 4], dtype=np.uint32), 1001
    cases["softmax_setup_delays"] = wl
    # fused dense-ReLU-dense rounds: the global round has 5 * (i + 2) mini-batch recursions
    wl = W.config2(n_clients=5, n_total=5 * 70, d=50, hidden=32, batch=16, rounds=5, a=80, b=160)
    wl.is_straggler = np.array([1, 0, 0, 1, 0], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 0, 2, 78
    wl.setup_weights, wl.setup_seed = np.array([1, 2, 3, 0, 4], dtype=np.uint32), 1002
    cases["mlp_fused_setup"] = wl
    # convolutions, equal probabilities (the paper's p_c = 1/n), on a ring
    wl = W.config3(n_clients=4, n_per=40, hw=16, batch=4, rounds=4, a=16, b=32)
    wl.compute_factor = np.array([1, 1, 2, 1], dtype=np.int32)
    wl.agg_scale = 0.5
    wl.setup_weights, wl.setup_seed = np.array([1, 1, 1, 1], dtype=np.uint32), 1003
    wl.topology = W.ring_topology(4)
    cases["lenet16_setup_ring"] = wl
    return cases


@pytest.mark.parametrize("name", list(setup_cases()))
def test_setup_cases_every_tick(gpu, oracle_libs, name):
    from oracle import Oracle
    from parity import lockstep
    wl = setup_cases()[name]
    run, orc = gpu(wl), Oracle(wl, "f64")
    report(name, lockstep(wl, run, orc))
    # the nodes' rounds add up to the global rounds (lockstep has compared every s_{i,c})
    for i in range(wl.rounds):
        assert sum(run.lib.aet_get_round_info(c, i)["s"] for c in range(wl.n_clients)) == wl.a * i + wl.b
    run.close()


def test_setup_error_paths(gpu):
    from paper_2112_13935_amd import AetError
    wl = W.config1(n_clients=3, n_per=30, d=10, rounds=2, a=2, b=2)
    run = gpu(wl)
    with pytest.raises(AetError) as e:
        run.lib.aet_set_setup(np.array([0, 0, 0], dtype=np.uint32), 1)
    assert e.value.status == -1
    with pytest.raises(AetError) as e:
        run.lib.aet_set_setup(np.array([2**31, 2**31, 1], dtype=np.uint32), 1)
    assert e.value.status == -1
    run.run_round()
    with pytest.raises(AetError) as e:
        run.lib.aet_set_setup(np.array([1, 1, 1], dtype=np.uint32), 1)
    assert e.value.status == -4
    run.close()
