"""aet_init_static (the entry point for callers that cannot allocate: the context lives on
the library's own device array) against aet_init with a caller's workspace: the same
kernels run, so every output has to agree bit for bit.  Three contexts in a row share the
array, each smaller than the one before, so stale contents of a larger run lie under the
next one."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2112_13935_amd import load_library
    load_library()
    from paper_2112_13935_amd.runner import Run
    return Run


def cases():
    out = []
    # the layer-by-layer engine (activations, pooling masks, partial sums in the workspace)
    wl = W.config3(n_clients=6, n_per=40, hw=16, batch=4, rounds=4, a=4, b=8)
    wl.compute_factor = np.array([1, 1, 2, 1, 4, 1], dtype=np.int32)
    out.append(("LeNet 16x16, 6 clients", wl))
    # the fused dense-ReLU-dense engine (tagged exchange records in the workspace)
    wl = W.config2(n_clients=5, n_total=5 * 70, d=50, hidden=32, batch=16, rounds=4, a=16, b=32)
    wl.compute_factor = np.array([1, 2, 1, 1, 3], dtype=np.int32)
    out.append(("MLP 50-32-10, 5 clients", wl))
    # 60 clients: more round records than one kernel-argument pack (48) and, with every
    # client arriving in the same tick, more arrivals than the by-value list (32)
    wl = W.config1(n_clients=60, n_per=40, d=37, rounds=4, a=3, b=2)
    wl.is_straggler = np.zeros(60, dtype=np.uint8)
    wl.is_straggler[::7] = 1
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 2, 5
    out.append(("softmax, 60 clients", wl))
    return out


def test_static_workspace_matches_caller_workspace(gpu):
    sizes = []
    for name, wl in cases():
        print(f"\n[no-alloc] {name}", flush=True)
        ref = gpu(wl)
        run = gpu(wl, shards=(ref.X, ref.y), static_workspace=True)
        sizes.append(run.lib.workspace_bytes)
        while not ref.lib.aet_all_done(wl.rounds):
            fin = ref.run_round()
            assert run.run_round() == fin
            for c, k in fin:
                assert run.lib.aet_get_round_info(c, k) == ref.lib.aet_get_round_info(c, k), (name, c, k)
                assert np.array_equal(run.lib.aet_get_U(c, k), ref.lib.aet_get_U(c, k)), (name, c, k)
                assert np.array_equal(run.lib.aet_get_weights(c), ref.lib.aet_get_weights(c)), (name, c, k)
            assert run.server_aggregate() == ref.server_aggregate()
            assert np.array_equal(run.lib.aet_get_weights(-1), ref.lib.aet_get_weights(-1)), name
        assert run.lib.aet_all_done(wl.rounds) and run.lib.aet_inflight() == 0
        # a second job on the same context
        run.lib.aet_reset()
        ref.lib.aet_reset()
        assert run.run_ticks() == ref.run_ticks()
        assert np.array_equal(run.lib.aet_get_weights(-1), ref.lib.aet_get_weights(-1)), name
        run.close()
        ref.close()
    assert sizes[0] > sizes[1] > sizes[2], sizes


def test_static_workspace_limits(gpu):
    from paper_2112_13935_amd import AetError
    small = cases()[1][1]
    a = gpu(small, static_workspace=True)
    with pytest.raises(AetError) as e:      # the array is taken
        gpu(small, shards=(a.X, a.y), static_workspace=True)
    assert e.value.status == -4
    a.close()
    b = gpu(small, shards=(a.X, a.y), static_workspace=True)   # free again after aet_destroy
    b.run_ticks()
    b.close()
    big = W.config3(n_clients=64, n_per=20)            # 64 LeNet replicas + U slots: beyond 64 MiB
    with pytest.raises(AetError) as e:
        gpu(big, static_workspace=True)
    assert e.value.status == -2 and "bytes" in str(e.value)
