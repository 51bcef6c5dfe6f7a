"""The comparison that the GPU parity tests rely on, exercised on the CPU: the oracle's fp32
build stands in for the library under test (tests/twin_adapter.py).  It has to pass the
bar; planted mistakes have to fail it; an error beyond the flat bar is accepted exactly
where a near-kink decision is booked."""
import numpy as np
import pytest

import workloads as W
from oracle import Oracle
from parity import KINK_SLACK, TOL, lockstep
from twin_adapter import OracleAsRun


def lenet16():
    wl = W.config3(n_clients=4, n_per=40, hw=16, batch=4, rounds=4, a=4, b=8)
    wl.compute_factor = np.array([1, 1, 2, 1], dtype=np.int32)
    wl.is_straggler = np.array([0, 1, 0, 0], dtype=np.uint8)
    wl.delay_min, wl.delay_max, wl.delay_seed = 1, 2, 9
    return wl


def mlp():
    return W.config2(n_clients=3, n_total=3 * 60, d=30, hidden=16, batch=4, rounds=4, a=4, b=8)


@pytest.mark.parametrize("make", [lenet16, mlp, lambda: W.config1(n_clients=3, n_per=30, d=20, rounds=4, a=2, b=2)])
def test_fp32_build_of_the_oracle_passes(oracle_libs, make):
    wl = make()
    out = lockstep(wl, OracleAsRun(Oracle(wl, "f32")), Oracle(wl, "f64"))
    assert out["Wg"] <= TOL and out["loss"] <= TOL


def test_fp32_build_passes_on_a_ring_and_under_resync(oracle_libs):
    wl = lenet16()
    lockstep(wl, OracleAsRun(Oracle(wl, "f32")), Oracle(wl, "f64"), resync=True)
    wl = mlp()
    wl.agg_scale = 0.5
    wl.topology = W.ring_topology(3)
    lockstep(wl, OracleAsRun(Oracle(wl, "f32")), Oracle(wl, "f64"))


class _Tampered(OracleAsRun):
    """Exact copy of the oracle whose reported values are changed by the test."""

    def __init__(self, orc, weights=None, U=None, order=False):
        super().__init__(orc)
        get_w, get_U = self.lib.aet_get_weights, self.lib.aet_get_U
        if weights:
            self.lib.aet_get_weights = lambda c=-1: weights(c, get_w(c).astype(np.float64))
        if U:
            self.lib.aet_get_U = lambda c, k: U(c, k, get_U(c, k).astype(np.float64))
        self.order = order

    def exchange(self):
        out = self.o.exchange()
        return out[::-1] if self.order and len(out) > 1 else out


def test_a_small_bias_error_fails(oracle_libs):
    """2e-4 of the tensor's scale in one entry of a small bias tensor, nothing booked."""
    wl = mlp()
    sl = wl.model.param_slices()[0]

    def bump(c, w):
        if c == 1:
            w[sl[2] + 3] += 2e-4 * np.abs(w[sl[2]:sl[2] + sl[3]]).max()
        return w
    with pytest.raises(AssertionError, match="no near-kink decision"):
        lockstep(wl, _Tampered(Oracle(wl, "f64"), weights=bump), Oracle(wl, "f64"), kink_eps=1e-12)


def test_wrong_aggregation_order_fails(oracle_libs):
    wl = mlp()
    with pytest.raises(AssertionError, match="aggregation order"):
        lockstep(wl, _Tampered(Oracle(wl, "f64"), order=True), Oracle(wl, "f64"))


def test_error_beyond_flat_bar_needs_a_booked_decision(oracle_libs):
    """The same displacement of one U tensor passes when the round has booked jumps that
    cover it and fails when the margin is so small that nothing is booked."""
    wl = lenet16()
    eps = 0.05                                  # wide margin: plenty of decisions are booked
    probe = Oracle(wl, "f64")
    probe.set_kink_eps(eps)
    probe.run_round()
    ev, allow = probe.round_kinks(2, 0)
    j = int(np.argmax(allow))
    assert ev > 0 and allow[j] > 0
    slices = []
    for sl in wl.model.param_slices():
        if sl is not None:
            slices += [slice(sl[0], sl[0] + sl[1]), slice(sl[2], sl[2] + sl[3])]
    U0 = probe.get_U(2, 0)
    shift = max(0.5 * KINK_SLACK * allow[j], 3 * TOL * np.abs(U0[slices[j]]).max())
    assert shift <= KINK_SLACK * allow[j]

    def bump(c, k, U):
        if (c, k) == (2, 0):
            U[slices[j].start] += shift
        return U
    lockstep(wl, _Tampered(Oracle(wl, "f64"), U=bump), Oracle(wl, "f64"), kink_eps=eps, stop_after_ticks=1)
    with pytest.raises(AssertionError, match="no near-kink decision"):
        lockstep(wl, _Tampered(Oracle(wl, "f64"), U=bump), Oracle(wl, "f64"), kink_eps=1e-12, stop_after_ticks=1)
