"""GPU parity of the peer-to-peer form (own model per node, messages to the neighbours,
neighbour-only delay checkpoint): the HIP library through its C ABI against the CPU oracle.
Run with  -m gpu  on an MI355X."""
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


def p2p_cases():
    cases = {}
    # fused softmax-regression rounds, ring, everything ragged
    wl = W.config1(n_clients=5, n_per=60, d=37, rounds=6, a=3, b=2)
    wl.compute_factor = np.array([1, 2, 1, 3, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 0, 1, 0, 1], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 3, 77
    wl.agg_scale = 1.0                      # the paper's rule
    wl.topology = W.ring_topology(5)
    cases["softmax_ring_delays"] = wl
    # fused dense-ReLU-dense rounds, ring
    wl = W.config2(n_clients=5, n_total=5 * 70, d=50, hidden=32, batch=16, rounds=5, a=16, b=32)
    wl.is_straggler = np.array([1, 0, 0, 1, 0], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 0, 2, 78
    wl.compute_factor = np.array([1, 2, 1, 1, 3], dtype=np.int32)
    wl.agg_scale = 0.5
    wl.topology = W.ring_topology(5)
    cases["mlp_fused_ring_stragglers"] = wl
    # layer-by-layer engine, complete graph
    wl = W.config2(n_clients=4, n_total=4 * 70, d=50, hidden=24, batch=4, rounds=5, a=4, b=8)
    wl.agg_scale = 0.25
    wl.topology = W.complete_topology(4)
    cases["mlp_layers_complete"] = wl
    # convolutions, line, the delay checkpoint on neighbours
    wl = W.config3(n_clients=4, n_per=40, hw=16, batch=4, rounds=4, a=4, b=8)
    wl.compute_factor = np.array([1, 1, 3, 1], dtype=np.int32)
    wl.d_max = 1
    wl.agg_scale = 0.5
    wl.topology = W.line_topology(4)
    cases["lenet16_line_checkpoint"] = wl
    # two components and an isolated node
    wl = W.config1(n_clients=5, n_per=40, d=20, rounds=4, a=2, b=2)
    wl.agg_scale = 1.0
    wl.topology = W.topology_from_edges(5, [(0, 1), (2, 3)])
    cases["softmax_two_parts_and_a_loner"] = wl
    # more arrivals in a tick than travel in the kernel arguments
    wl = W.config1(n_clients=40, n_per=30, d=20, rounds=3, a=2, b=2)
    wl.agg_scale = 0.5
    wl.topology = W.ring_topology(40)
    cases["softmax_ring_40"] = wl
    # ... and more than one window of the arrival scan, with stragglers
    wl = W.config1(n_clients=300, n_per=20, d=8, rounds=3, a=1, b=2)
    wl.is_straggler = (np.arange(300) % 7 == 0).astype(np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 2, 5
    wl.agg_scale = 0.5
    wl.topology = W.ring_topology(300)
    cases["softmax_ring_300"] = wl
    return cases


@pytest.mark.parametrize("name", list(p2p_cases()))
def test_p2p_cases_every_tick(gpu, oracle_libs, name):
    """U, the losses, the finishing nodes' models after their rounds and EVERY node's model
    after each Receive are compared; starts, round numbers and deliveries bit-exactly."""
    from oracle import Oracle
    from parity import lockstep
    wl = p2p_cases()[name]
    run, orc = gpu(wl), Oracle(wl, "f64")
    assert run.p2p and orc.p2p
    report(name, lockstep(wl, run, orc))
    # no global model in this form: it stays what Setup gave
    assert np.array_equal(run.lib.aet_get_weights(-1), wl.w0)
    run.close()


def test_p2p_run_ticks_and_reset(gpu):
    """The driver loop takes the Receive form when a topology is set; a second job after
    aet_reset starts every node from w0 again and gives the same bits."""
    wl = p2p_cases()["mlp_fused_ring_stragglers"]
    a = gpu(wl)
    ticks_a = a.run_all()
    b = gpu(wl)
    assert b.run_ticks() == ticks_a
    for c in range(wl.n_clients):
        assert np.array_equal(a.lib.aet_get_weights(c), b.lib.aet_get_weights(c))
    first = [b.lib.aet_get_weights(c) for c in range(wl.n_clients)]
    b.lib.aet_reset()
    assert b.run_ticks() == ticks_a
    for c in range(wl.n_clients):
        assert np.array_equal(first[c], b.lib.aet_get_weights(c))
    a.close()
    b.close()


def test_p2p_config2_ring_20_rounds(gpu, oracle_libs):
    """The benchmark's model and client count on a ring, 20 rounds."""
    from oracle import Oracle
    from parity import lockstep
    wl = W.config2()
    wl.agg_scale = 1.0 / 3.0
    wl.topology = W.ring_topology(wl.n_clients)
    run, orc = gpu(wl), Oracle(wl, "f64")
    report("config 2 on a ring (16 nodes, 20 rounds)",
           lockstep(wl, run, orc, rounds=20, check_every=5))
    run.close()


def test_p2p_error_paths(gpu):
    from paper_2112_13935_amd import AetError
    wl = p2p_cases()["softmax_ring_delays"]
    run = gpu(wl)
    with pytest.raises(AetError) as e:       # a topology is set: no server step
        run.server_aggregate()
    assert e.value.status == -4
    run.run_round()
    with pytest.raises(AetError) as e:       # too late to change it
        run.lib.aet_set_topology(*W.line_topology(5))
    assert e.value.status == -4
    run.close()
    wl2 = W.config1(n_clients=3, n_per=30, d=10, rounds=2, a=2, b=2)
    run = gpu(wl2)
    with pytest.raises(AetError) as e:       # no topology: no Receive at neighbours
        run.receive()
    assert e.value.status == -4
    bad = [
        (np.array([0, 1, 1, 1], dtype=np.int32), np.array([1], dtype=np.int32)),            # one way only
        (np.array([0, 1, 1, 1], dtype=np.int32), np.array([0], dtype=np.int32)),            # self loop
        (np.array([0, 2, 4, 4], dtype=np.int32), np.array([1, 1, 0, 0], dtype=np.int32)),   # duplicate
        (np.array([0, 1, 2, 2], dtype=np.int32), np.array([5, 0], dtype=np.int32)),         # out of range
    ]
    for off, nbr in bad:
        with pytest.raises(AetError) as e:
            run.lib.aet_set_topology(off, nbr)
        assert e.value.status == -1
    # still usable, in the server form
    assert run.run_round() == [(c, 0) for c in range(3)]
    assert run.server_aggregate() == [(c, 0) for c in range(3)]
    run.close()
