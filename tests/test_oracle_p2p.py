"""Pins for the oracle's peer-to-peer form (Algorithm 2 as printed: every node keeps its
own model, sends (c, U_i, i) to its neighbours, applies what they send).  No GPU needed.

None of these retypes the oracle's loop: they check what the algorithm fixes from outside
(a conservation identity per node, reductions to cases pinned elsewhere, hand-computed
schedules, independence of disconnected parts)."""
import numpy as np
import pytest

import workloads as W
from oracle import Oracle


def small_softmax(n=4, n_per=40, d=12, rounds=4, a=2, b=3, **kw):
    wl = W.config1(n_clients=n, n_per=n_per, d=d, rounds=rounds, a=a, b=b)
    for k, v in kw.items():
        setattr(wl, k, v)
    return wl


def small_mlp(n=4, rounds=3, **kw):
    wl = W.config2(n_clients=n, n_total=n * 50, d=20, hidden=8, batch=4, rounds=rounds, a=4, b=8)
    for k, v in kw.items():
        setattr(wl, k, v)
    return wl


def neighbours(topo, c):
    off, nbr = topo
    return nbr[off[c]:off[c + 1]].tolist()


def run_collect(o, scale=None):
    """Tick to the end; returns {(c, k): (eta, U)} of every message and the delivery log."""
    msgs, log = {}, []
    while not o.all_done():
        for c, k in o.run_round():
            msgs[(c, k)] = (o.round_info(c, k)["eta"], o.get_U(c, k))
        t = o.tick
        for c, k in o.receive(scale):
            log.append((t, c, k))
    return msgs, log


@pytest.mark.parametrize("topo_name", ["ring", "line", "complete"])
@pytest.mark.parametrize("make", [small_softmax, small_mlp])
def test_every_node_ends_at_w0_minus_own_and_neighbour_messages(oracle_libs, make, topo_name):
    """Each recursion moves w_c by -eta_i g and U_i sums those g; each neighbour message
    moves it by -scale eta_k U_k.  So at the end, whatever the interleaving,
        w_c = w0 - sum_i eta_i U_{i,c} - scale * sum_{v in N(c)} sum_k eta_k U_{k,v}
    in real arithmetic (here to fp64 rounding).  Stragglers, compute factors and a
    non-trivial scale make sure the sender's eta_k (not the receiver's) and the right
    neighbour sets are what is used."""
    n = 5
    wl = make(n=n, beta=0.05, power=1.0)      # step size differs from round to round
    wl.compute_factor = np.array([1, 2, 1, 3, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 1, 0, 0, 1], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 3, 99
    topo = {"ring": W.ring_topology, "line": W.line_topology, "complete": W.complete_topology}[topo_name](n)
    o = Oracle(wl)
    o.set_topology(*topo)
    scale = 0.37
    msgs, log = run_collect(o, scale)
    assert len(msgs) == n * wl.rounds and len(log) == n * wl.rounds
    w0 = wl.w0.astype(np.float64)
    for c in range(n):
        expect = w0.copy()
        for k in range(wl.rounds):
            eta, U = msgs[(c, k)]
            expect -= eta * U
        for v in neighbours(topo, c):
            for k in range(wl.rounds):
                eta, U = msgs[(v, k)]
                expect -= scale * eta * U
        got = o.get_weights(c)
        assert np.abs(got - expect).max() <= 1e-12 * max(1.0, np.abs(expect).max()), (c, topo_name)
    # the step sizes did differ between rounds, so a receiver-side eta would have shown
    assert msgs[(0, 0)][0] != msgs[(0, wl.rounds - 1)][0]


def test_complete_graph_zero_delay_equals_the_server_form(oracle_libs):
    """All nodes neighbours of each other, no delays, scale 1: after every tick each node
    has applied its own U through its recursions and everybody else's through Receive,
    so all models agree and equal the server form's global model with the paper's
    unscaled rule (that form is pinned on its own)."""
    n = 4
    wl = small_softmax(n=n, rounds=4, agg_scale=1.0)
    srv = Oracle(wl)
    p2p = Oracle(wl)
    p2p.set_topology(*W.complete_topology(n))
    while not srv.all_done():
        assert srv.run_round() == p2p.run_round()
        assert srv.server_aggregate() == p2p.receive()
        wg = srv.get_weights(-1)
        for c in range(n):
            assert np.abs(p2p.get_weights(c) - wg).max() <= 1e-13 * max(1.0, np.abs(wg).max())
    assert p2p.all_done()


def test_no_neighbours_is_one_long_plain_sgd_run(oracle_libs):
    """A node without neighbours never receives anything and never adopts anything: its
    model after R rounds is plain per-sample SGD over all its samples in order (numpy,
    textbook softmax-regression gradient)."""
    wl = small_softmax(n=1, n_per=50, d=9, rounds=5, a=3, b=2)
    o = Oracle(wl)
    o.set_topology(*W.ring_topology(1))
    o.run_all()
    X, y = wl.X[0].astype(np.float64), wl.y[0]
    Wm, bias, q = np.zeros((10, 9)), np.zeros(10), 0
    for i in range(5):
        for _ in range(wl.a * i + wl.b):
            idx = o.sample_index(0, q, 50)
            q += 1
            z = Wm @ X[idx] + bias
            p = np.exp(z - z.max())
            p /= p.sum()
            p[y[idx]] -= 1.0
            Wm -= wl.eta0 * np.outer(p, X[idx])
            bias -= wl.eta0 * p
    w = o.get_weights(0)
    assert np.abs(w[:90].reshape(10, 9) - Wm).max() <= 1e-13
    assert np.abs(w[90:] - bias).max() <= 1e-13
    assert np.array_equal(o.get_weights(-1), wl.w0.astype(np.float64))   # no global model moves


def test_two_node_ring_delivers_once(oracle_libs):
    """With n = 2 the left and the right neighbour are the same node: one delivery, not two
    (covered by the conservation identity with the de-duplicated neighbour list)."""
    wl = small_softmax(n=2, rounds=3)
    topo = W.ring_topology(2)
    assert neighbours(topo, 0) == [1] and neighbours(topo, 1) == [0]
    o = Oracle(wl)
    o.set_topology(*topo)
    msgs, _ = run_collect(o, 1.0)
    w0 = wl.w0.astype(np.float64)
    for c in (0, 1):
        expect = w0 - sum(msgs[(c, k)][0] * msgs[(c, k)][1] for k in range(3)) \
                    - sum(msgs[(1 - c, k)][0] * msgs[(1 - c, k)][1] for k in range(3))
        assert np.abs(o.get_weights(c) - expect).max() <= 1e-13


def test_hand_computed_schedule_on_a_ring(oracle_libs):
    """n = 3 ring, compute factors (1, 2, 1), node 2 a straggler with network delay 2,
    R = 2.  By hand:
      tick 0: all start round 0.  Node 0 done at 0 -> arrives 0.  Node 1 busy ticks 0-1 ->
              arrives 1.  Node 2 done at 0, delay 2 -> arrives 2.
      tick 1: nodes 0, 2 start round 1 (node 1 still busy).  0 -> arrives 1;
              2 -> arrives 1 + 2 = 3.
      tick 2: node 1 starts round 1, busy 2-3 -> arrives 3.
    Deliveries in (round, sender) order inside a tick."""
    wl = small_softmax(n=3, rounds=2)
    wl.compute_factor = np.array([1, 2, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 0, 1], dtype=np.uint8)
    wl.delay_min = wl.delay_max = 2
    o = Oracle(wl)
    o.set_topology(*W.ring_topology(3))
    starts = []
    log = []
    while not o.all_done():
        t = o.tick
        starts += [(t, c, k) for c, k in o.run_round()]
        log += [(t, c, k) for c, k in o.receive()]
    assert starts == [(0, 0, 0), (0, 1, 0), (0, 2, 0), (1, 0, 1), (1, 2, 1), (2, 1, 1)]
    assert log == [(0, 0, 0), (1, 1, 0), (1, 0, 1), (2, 2, 0), (3, 1, 1), (3, 2, 1)]
    assert o.events() == log
    assert [o.history(c) for c in range(3)] == [2, 2, 2]


def test_delay_checkpoint_looks_at_neighbours_only(oracle_libs):
    """Line 0 - 1 - 2, node 2 four times slower, d = 0: node c may start round i only when
    every NEIGHBOUR has delivered i rounds.  By hand (factor f: a round started at t is
    delivered in tick t + f - 1, usable from tick t + f):
      node 2 starts round 0 at 0 (delivered tick 3), round 1 at 4 (gated by node 1: H_1 >= 1 ok).
      node 1 starts round 0 at 0, round 1 when H_0 >= 1 and H_2 >= 1 -> tick 4.
      node 0 starts round 0 at 0, round 1 when H_1 >= 1 -> tick 1; round 2 when H_1 >= 2:
              node 1's round 1 runs in tick 4, delivered tick 4 -> node 0 starts round 2 at 5.
    Node 0 is never held back by node 2 directly: its round 1 starts at tick 1 although
    node 2 has delivered nothing by then."""
    wl = small_softmax(n=3, rounds=3)
    wl.compute_factor = np.array([1, 1, 4], dtype=np.int32)
    wl.d_max = 0
    o = Oracle(wl)
    o.set_topology(*W.line_topology(3))
    start = {}
    while not o.all_done():
        t = o.tick
        for c, k in o.run_round():
            start[(c, k)] = t
        o.receive()
        assert t < 100
    assert start[(0, 0)] == 0 and start[(1, 0)] == 0 and start[(2, 0)] == 0
    assert start[(0, 1)] == 1            # only node 1 matters for node 0
    assert start[(1, 1)] == 4            # waits for node 2's first delivery (tick 3)
    assert start[(2, 1)] == 4
    assert start[(0, 2)] == 5            # node 1's round 1 delivered in tick 4
    # the same run under the all-nodes map of the server form would hold node 0 until tick 4
    srv = Oracle(wl)
    s2 = {}
    while not srv.all_done():
        t = srv.tick
        for c, k in srv.run_round():
            s2[(c, k)] = t
        srv.server_aggregate()
    assert s2[(0, 1)] == 4


def test_disconnected_parts_do_not_influence_each_other(oracle_libs):
    """Two components {0,1} and {2,3}: replacing the data of nodes 2, 3 leaves the models of
    nodes 0, 1 bit-identical."""
    wl = small_mlp(n=4, rounds=3)
    topo = W.topology_from_edges(4, [(0, 1), (2, 3)])
    a = Oracle(wl)
    a.set_topology(*topo)
    a.run_all()
    wl2 = small_mlp(n=4, rounds=3)
    wl2.X[2] = wl2.X[2][::-1].copy()
    wl2.X[3] = wl2.X[3] * 0.5
    b = Oracle(wl2)
    b.set_topology(*topo)
    b.run_all()
    for c in (0, 1):
        assert np.array_equal(a.get_weights(c), b.get_weights(c))
    for c in (2, 3):
        assert not np.array_equal(a.get_weights(c), b.get_weights(c))


def test_bad_topologies_are_rejected(oracle_libs):
    wl = small_softmax(n=3, rounds=1)
    o = Oracle(wl)
    with pytest.raises(RuntimeError):      # directed edge 0 -> 1 only
        o.set_topology(np.array([0, 1, 1, 1], dtype=np.int32), np.array([1], dtype=np.int32))
    with pytest.raises(RuntimeError):      # self loop
        o.set_topology(np.array([0, 1, 1, 1], dtype=np.int32), np.array([0], dtype=np.int32))
    with pytest.raises(RuntimeError):      # duplicate neighbour
        o.set_topology(np.array([0, 2, 4, 4], dtype=np.int32), np.array([1, 1, 0, 0], dtype=np.int32))
    o.run_round()
    with pytest.raises(RuntimeError):      # too late
        o.set_topology(*W.ring_topology(3))
    with pytest.raises(RuntimeError):      # and the server form has no Receive at neighbours
        o.receive()
