"""Pins for the oracle's client/round/server loop: the per-round identity between U and
the weight displacement, the one-client reduction to plain SGD, brute-force server sums,
hand-computed event schedules, conservation of messages.  No GPU needed."""
import numpy as np
import pytest

import workloads as W
from oracle import Oracle
from oracle.oracle import batch_loss_grad


def small_softmax(n=3, n_per=40, d=12, rounds=5, a=2, b=3, **kw):
    wl = W.config1(n_clients=n, n_per=n_per, d=d, rounds=rounds, a=a, b=b)
    for k, v in kw.items():
        setattr(wl, k, v)
    return wl


def small_mlp(n=3, rounds=4, **kw):
    wl = W.config2(n_clients=n, n_total=n * 50, d=20, hidden=8, batch=4, rounds=rounds, a=4, b=8)
    for k, v in kw.items():
        setattr(wl, k, v)
    return wl


def small_lenet(n=4, rounds=3, **kw):
    wl = W.config3(n_clients=n, n_per=30, hw=16, batch=2, rounds=rounds, a=2, b=4)
    for k, v in kw.items():
        setattr(wl, k, v)
    return wl


@pytest.mark.parametrize("make", [small_softmax, small_mlp, small_lenet])
def test_U_equals_weight_displacement_over_eta(oracle_libs, make):
    """Within a round the step size is fixed and U is the sum of the gradients used, so
    w_start - w_end = eta_i * U_i (exactly in real arithmetic; to rounding in fp64)."""
    wl = make()
    o = Oracle(wl)
    while not o.all_done():
        w_start = o.get_weights(-1)
        for c, k in o.run_round():
            info = o.round_info(c, k)
            U = o.get_U(c, k)
            w_end = o.get_weights(c)
            assert info["m"] > 0 and np.abs(U).max() > 0
            assert np.abs((w_start - w_end) / info["eta"] - U).max() <= 1e-10 * max(1.0, np.abs(U).max())
        o.server_aggregate()


def test_round_lengths_follow_the_linear_threshold(oracle_libs):
    wl = small_mlp(rounds=6)
    o = Oracle(wl)
    o.run_all()
    B = wl.model.batch
    for c in range(wl.n_clients):
        q = t = 0
        for k in range(6):
            info = o.round_info(c, k)
            assert info["s"] == wl.a * k + wl.b
            assert info["m"] * B == info["s"]
            assert info["q0"] == q and info["t0"] == t
            assert info["eta"] == pytest.approx(wl.eta0 / (1 + wl.beta * t ** wl.power), rel=1e-15)
            q += info["s"]
            t += info["m"]


def test_round_length_not_multiple_of_batch_is_an_error(oracle_libs):
    wl = small_mlp()
    wl.b = 6          # batch is 4
    o = Oracle(wl)
    with pytest.raises(RuntimeError):
        o.run_round()


def test_one_client_zero_delay_is_plain_sgd(oracle_libs):
    """n = 1 'works as the traditional SGD method': with the paper's unscaled server rule
    the global model after every round equals sequential per-sample SGD on the same index
    stream.  The plain SGD here is written with numpy from the textbook softmax gradient."""
    wl = small_softmax(n=1, n_per=50, d=9, rounds=6, a=3, b=2, agg_scale=1.0)
    o = Oracle(wl)
    X, y = wl.X[0].astype(np.float64), wl.y[0]
    Wm = np.zeros((10, 9))
    bias = np.zeros(10)
    q = 0
    for i in range(6):
        o.run_round()
        o.server_aggregate()
        for _ in range(wl.a * i + wl.b):
            idx = o.sample_index(0, q, 50)
            q += 1
            z = Wm @ X[idx] + bias
            p = np.exp(z - z.max())
            p /= p.sum()
            p[y[idx]] -= 1.0
            Wm -= wl.eta0 * np.outer(p, X[idx])
            bias -= wl.eta0 * p
        wg = o.get_weights(-1)
        assert np.abs(wg[:90].reshape(10, 9) - Wm).max() <= 1e-13
        assert np.abs(wg[90:] - bias).max() <= 1e-13
    assert q == sum(wl.a * i + wl.b for i in range(6))


def test_first_step_of_first_round_is_one_sgd_recursion(oracle_libs):
    """a=0, b=B: one recursion per round; U is the batch gradient at w0 and the local
    model is w0 - eta * g (eq. 3)."""
    wl = small_mlp(n=2, rounds=1)
    wl.a, wl.b = 0, wl.model.batch
    o = Oracle(wl)
    o.run_round()
    for c in range(2):
        idx = [o.sample_index(c, j, wl.X[c].shape[0]) for j in range(wl.model.batch)]
        loss, g = batch_loss_grad(wl.model, wl.w0.astype(np.float64), wl.X[c][idx], wl.y[c][idx])
        assert np.array_equal(o.get_U(c, 0), g)
        assert np.array_equal(o.get_weights(c), wl.w0.astype(np.float64) - wl.eta0 * g)
        assert o.round_info(c, 0)["loss"] == loss


def test_server_sum_brute_force_and_order(oracle_libs):
    """Wg after a tick = Wg before - sum over arrivals of alpha * eta_k * U, and the log
    lists the arrivals in (round, client) order."""
    wl = small_mlp(n=5, rounds=3)
    o = Oracle(wl)
    for tick in range(3):
        before = o.get_weights(-1)
        fin = o.run_round()
        Us = {ck: o.get_U(*ck) for ck in fin}
        etas = {ck: o.round_info(*ck)["eta"] for ck in fin}
        applied = o.server_aggregate()
        assert applied == sorted(fin, key=lambda ck: (ck[1], ck[0]))
        want = before.copy()
        for ck in applied:
            want -= wl.agg_scale * etas[ck] * Us[ck]
        assert np.abs(o.get_weights(-1) - want).max() <= 1e-15
        assert np.abs(before - o.get_weights(-1)).max() > 0


def test_identical_shards_mean_aggregation_reproduces_a_client(oracle_libs):
    """Zero delay, alpha = 1/n and identical shards with identical index streams cannot be
    built (streams differ per client), but identical U's can: with one sample per shard
    every draw is index 0, so all clients compute the same U and the new global model is
    any client's end-of-round model."""
    wl = small_softmax(n=4, n_per=1, d=6, rounds=3, agg_scale=0.25)
    for c in range(1, 4):
        wl.X[c] = wl.X[0].copy()
        wl.y[c] = wl.y[0].copy()
    o = Oracle(wl)
    for _ in range(3):
        o.run_round()
        o.server_aggregate()
        wg = o.get_weights(-1)
        for c in range(4):
            assert np.abs(wg - o.get_weights(c)).max() <= 1e-15


def test_zero_delay_schedule(oracle_libs):
    """All factors 1 and no stragglers: tick t runs round t of every client and applies
    exactly {(c, t)} in client order."""
    wl = small_softmax(n=4, rounds=5)
    o = Oracle(wl)
    ticks = o.run_all()
    assert ticks == 5
    assert o.events() == [(t, c, t) for t in range(5) for c in range(4)]


def test_hand_computed_schedule_with_factors_and_a_straggler(oracle_libs):
    """n=3, R=3.  Client 1 takes 2 ticks per round; client 2 is a straggler whose messages
    spend exactly 2 extra ticks in the network (delay_min = delay_max = 2).
      client 0: starts rounds 0,1,2 at ticks 0,1,2, arrivals at 0,1,2
      client 1: starts at ticks 0,2,4, arrivals at 1,3,5
      client 2: starts at ticks 0,1,2, arrivals at 2,3,4
    Arrivals within a tick are applied in (round, client) order."""
    wl = small_softmax(n=3, rounds=3)
    wl.compute_factor = np.array([1, 2, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 0, 1], dtype=np.uint8)
    wl.delay_min = wl.delay_max = 2
    o = Oracle(wl)
    started = []
    while not o.all_done():
        t = o.tick
        started += [(t, c, k) for c, k in o.run_round()]
        o.server_aggregate()
    assert started == [(0, 0, 0), (0, 1, 0), (0, 2, 0), (1, 0, 1), (1, 2, 1), (2, 0, 2), (2, 1, 1),
                       (2, 2, 2), (4, 1, 2)]
    assert o.events() == [(0, 0, 0), (1, 1, 0), (1, 0, 1), (2, 2, 0), (2, 0, 2), (3, 1, 1), (3, 2, 1),
                          (4, 2, 2), (5, 1, 2)]
    assert o.tick == 6


def test_late_message_uses_the_senders_step_size(oracle_libs):
    """Receive applies eta_k of the SENDER's round k.  With a diminishing step size and a
    delayed message, the global model moves by alpha * eta_k * U with eta_k taken at the
    time the round ran, not at the time it arrives."""
    wl = small_mlp(n=2, rounds=3)
    wl.beta = 0.5
    wl.is_straggler = np.array([0, 1], dtype=np.uint8)
    wl.delay_min = wl.delay_max = 2
    o = Oracle(wl)
    pending = {}
    while not o.all_done():
        before = o.get_weights(-1)
        for ck in o.run_round():
            pending[ck] = (o.get_U(*ck), o.round_info(*ck)["eta"])
        applied = o.server_aggregate()
        want = before.copy()
        for ck in applied:
            U, eta = pending.pop(ck)
            want -= wl.agg_scale * eta * U
        assert np.abs(o.get_weights(-1) - want).max() <= 1e-15
    assert not pending
    etas = [o.round_info(1, k)["eta"] for k in range(3)]
    assert etas[0] > etas[1] > etas[2]


def test_every_message_is_applied_exactly_once(oracle_libs):
    """Messages may arrive out of order but are never lost (network setting)."""
    wl = small_lenet(n=8, rounds=4)
    wl.compute_factor = W.compute_factors(8, (1, 2, 4), 3)
    assert wl.is_straggler.sum() == 2
    o = Oracle(wl)
    o.run_all()
    ev = o.events()
    assert sorted((c, k) for _, c, k in ev) == [(c, k) for c in range(8) for k in range(4)]
    assert [t for t, _, _ in ev] == sorted(t for t, _, _ in ev)
    for c in range(8):
        assert o.history(c) == 4
        for k in range(4):
            info = o.round_info(c, k)
            f = int(wl.compute_factor[c])
            lo = info["start_tick"] + f - 1 + (wl.delay_min if wl.is_straggler[c] else 0)
            hi = info["start_tick"] + f - 1 + (wl.delay_max if wl.is_straggler[c] else 0)
            assert lo <= info["arrival"] <= hi
            if k:
                assert info["start_tick"] >= o.round_info(c, k - 1)["start_tick"] + f
    # a straggler's rounds are out of order relative to the others' in the log
    assert any(k1 > k2 for (_, _, k1), (_, _, k2) in zip(ev, ev[1:]))


def test_sample_stream_does_not_depend_on_schedule(oracle_libs):
    """q_c counts samples drawn, so delays and factors change WHEN a round runs, never
    which samples it draws."""
    wl1 = small_softmax(n=3, rounds=4)
    wl2 = small_softmax(n=3, rounds=4)
    wl2.compute_factor = np.array([2, 1, 4], dtype=np.int32)
    o1, o2 = Oracle(wl1), Oracle(wl2)
    o1.run_all()
    o2.run_all()
    for c in range(3):
        for k in range(4):
            assert o1.round_info(c, k)["q0"] == o2.round_info(c, k)["q0"]


def test_empty_round_posts_a_zero_message(oracle_libs):
    """The paper's s_i = 10 i makes round 0 empty: U = 0, the model does not move."""
    wl = small_softmax(n=2, rounds=2, a=3, b=0)
    o = Oracle(wl)
    fin = o.run_round()
    assert fin == [(0, 0), (1, 0)]
    assert not o.get_U(0, 0).any()
    assert o.round_info(0, 0)["m"] == 0
    o.server_aggregate()
    assert np.array_equal(o.get_weights(-1), wl.w0.astype(np.float64))
    o.run_round()
    assert o.get_U(1, 1).any()


def test_delay_checkpoint_d0_is_lock_step(oracle_libs):
    """Synchronize with d = 0: nobody starts round i before every other node's rounds
    < i have been received, so a slow client holds everybody back."""
    wl = small_softmax(n=3, rounds=3)
    wl.compute_factor = np.array([1, 3, 1], dtype=np.int32)
    wl.d_max = 0
    o = Oracle(wl)
    started = []
    while not o.all_done():
        t = o.tick
        started += [(t, c, k) for c, k in o.run_round()]
        o.server_aggregate()
    # client 1's round k arrives at tick 3k+2; the others may start round k+1 only then
    assert started == [(0, 0, 0), (0, 1, 0), (0, 2, 0), (3, 0, 1), (3, 1, 1), (3, 2, 1),
                       (6, 0, 2), (6, 1, 2), (6, 2, 2)]
    # with d large nothing waits
    wl.d_max = 10
    o = Oracle(wl)
    o.run_round(), o.server_aggregate()
    assert [c for c, _ in o.run_round()] == [0, 2]


def test_training_loss_goes_down(oracle_libs):
    """Sanity only (accuracy figures of the paper are out of reach without its data)."""
    wl = W.config2(n_clients=4, n_total=2000, d=64, hidden=16, batch=8, rounds=24, a=8, b=16)
    o = Oracle(wl)
    o.run_all()
    first = np.mean([o.round_info(c, 0)["loss"] for c in range(4)])
    last = np.mean([o.round_info(c, 23)["loss"] for c in range(4)])
    assert last < 0.5 * first


def test_f32_twin_tracks_f64_on_a_well_conditioned_run(oracle_libs):
    wl = small_mlp(n=3, rounds=6)
    o64, o32 = Oracle(wl, "f64"), Oracle(wl, "f32")
    o64.run_all()
    o32.run_all()
    a, b = o64.get_weights(-1), o32.get_weights(-1).astype(np.float64)
    assert np.abs(a - b).max() / np.abs(a).max() < 1e-5
    assert o64.events() == o32.events()


def test_delay_checkpoint_sweep(oracle_libs):
    """Synchronize with growing d on a schedule with slow nodes: the gate can only delay
    starts, so the number of ticks to finish does not grow with d; a large d is the ungated
    run; d = 0 lets nobody start round i before every other node has delivered i rounds;
    the models never depend on anything but the schedule (same events => same result)."""
    wl = small_mlp(n=4, rounds=5)
    wl.compute_factor = np.array([1, 1, 2, 4], dtype=np.int32)
    ticks = {}
    starts = {}
    for d in (0, 1, 2, 3, 50, -1):
        wl.d_max = d
        o = Oracle(wl)
        st = {}
        while not o.all_done():
            t = o.tick
            for c, k in o.run_round():
                st[(c, k)] = t
            o.server_aggregate()
            assert t < 1000
        ticks[d], starts[d] = o.tick, st
    assert ticks[0] >= ticks[1] >= ticks[2] >= ticks[3] >= ticks[50] == ticks[-1]
    # the gate does bite on this schedule: ungated, the fast node 0 is done after 5 ticks;
    # the slowest node sets the end of the run either way
    assert starts[-1][(0, 4)] == 4 and starts[0][(0, 4)] == 16 and ticks[-1] == 20
    assert starts[50] == starts[-1]
    # d = 0: the slowest node (factor 4) paces everybody: round i starts at tick 4 i
    for c in range(4):
        for k in range(5):
            assert starts[0][(c, k)] == 4 * k
    # every gated schedule starts each round no earlier than the ungated one
    for d in (0, 1, 2, 3):
        assert all(starts[d][ck] >= starts[-1][ck] for ck in starts[-1])
