"""Helpers of the parity tests: drive the CPU oracle (fp64) and an implementation under test
(the HIP library through its C ABI) in lock step on the same seeded workload and compare.

Integer side, bit-exact: which clients run in a tick, their round numbers, round lengths
s_i and recursion counts, sample counters, start and arrival ticks, the sample indices,
the order in which arrivals are applied, the history H.  The round step size must be the
fp32 rounding of the oracle's double.

Floating point, per tensor (each layer's weights, each layer's bias, on their own):
    max|test - oracle| <= TOL * max|oracle|,   TOL = 1e-4,
for the global model, every client's w_c, every U and the losses (fp32 results after 20
rounds).  That is the whole bar for models without ReLU / max pooling.

Models with ReLU / max pooling.  Their gradient is discontinuous where a pre-activation
crosses zero or the two largest entries of a pooling window cross.  When rounding puts one
such decision of one sample on the other side than the fp64 oracle has it, that sample's
gradient jumps, and w and U with it, whatever the quality of the arithmetic; on a small
bias tensor one flip is already several 1e-4 of the tensor's scale.  The oracle therefore
books, per client and round, every decision whose relative margin is below KINK_EPS and
the jump of the mini-batch gradient that its flip would cause, per parameter tensor (the
section "Kinks" of oracle/aet_oracle.c, pinned by tests/test_oracle_kinks.py).  The bar of
a tensor becomes
    TOL * max|oracle| + KINK_SLACK * (jumps booked for that tensor on the way to this value
                                      + r * max|oracle|):
      U of a round          : the round's jumps
      w_c after a round     : eta_i * the round's jumps + what the model it started from carries
      a model after Receive : + scale * eta_k * the jumps of every message applied to it
      r                     : the largest of (booked jumps / max|w|) over the tensors of the
                              model: a flip moves the tensors at and below the flipped unit at
                              once and, through the recursions that follow it in the round,
                              every other tensor by about the same relative amount
so a tensor may leave the flat bar only where a near-kink decision was booked for the
client and round (or for a message that reached the model), and then by no more than the
booked jumps allow.  Without booked decisions the bar is TOL flat.

U of a round that the two sides did not start from the same model (a free-running run
after its first aggregation) is a function of two different inputs: its plain relative
error then measures how sensitive the oracle's own U is to its starting model (large for
the upper layers' small, cancelling sums), not the implementation.  Such a U is judged by
what it does when Receive applies it: eta_i * max|U_test - U_oracle| over a tensor against
TOL * max|w_c| of that tensor (plus the booked jumps).  U of rounds started from
bit-identical models (the first tick of every run, every tick under resync) is judged in
plain relative error.

resync=True: after every tick all sides restart from the oracle's global model (rounded
to fp32), so that every local round and every aggregation of a long run is compared from a
common starting point and what a model carries does not pile up over the run.
"""
from __future__ import annotations

import numpy as np

TOL = 1e-4
KINK_EPS = 1e-5     # relative margin below which a ReLU / pooling decision counts as near its kink
KINK_SLACK = 2.0    # a flipped decision also moves the recursions that follow it in the round


def relerr(test: np.ndarray, ref: np.ndarray) -> float:
    return float(np.abs(test.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-12))


def layer_slices(model):
    out = []
    for sl in model.param_slices():
        if sl is None:
            continue
        out.append(slice(sl[0], sl[0] + sl[1]))
        out.append(slice(sl[2], sl[2] + sl[3]))
    return out


def tensor_relerrs(model, test: np.ndarray, ref: np.ndarray):
    """Per-tensor relative errors; a tensor that is exactly zero on the oracle's side must be
    (almost) zero on the other side."""
    return [relerr(test[s], ref[s]) if np.abs(ref[s]).max() > 0 else float(np.abs(test[s]).max())
            for s in layer_slices(model)]


def tensor_relerr(model, test: np.ndarray, ref: np.ndarray) -> float:
    return max(tensor_relerrs(model, test, ref))


def has_kinks(model) -> bool:
    return any(L.relu or L.type == 1 for L in model.layers)


class Judge:
    """Compares tensors against the bar at once; keeps the worst figures for the report."""

    def __init__(self, model, tol):
        self.model, self.tol = model, tol
        self.slices = layer_slices(model)
        self.worst = {}        # quantity -> worst plain relative error
        self.compared = {}     # quantity -> tensor comparisons made
        self.beyond = {}       # quantity -> ... of which beyond the flat bar (inside the booked jumps)
        self.widest = {}       # quantity -> the widest bar that such a comparison was given
        self.fill = {}         # quantity -> the largest error / bar among them

    def tensors(self, quantity, what, test, ref, allow=None, events=0, scale_of=None, moved=0.0):
        """allow: per tensor, absolute, already in the units of `ref` (None: flat bar).
        scale_of: take each tensor's scale from this array instead of from `ref`.
        moved: the largest relative displacement that the booked jumps allow in any tensor
        of the model the value was computed from (follow-on of a flip on the other tensors)."""
        for j, s in enumerate(self.slices):
            scale = float(np.abs((ref if scale_of is None else scale_of)[s]).max())
            err = float(np.abs(test[s].astype(np.float64) - ref[s]).max())
            rel = err / max(scale, 1e-12) if scale > 0 else err
            self.worst[quantity] = max(self.worst.get(quantity, 0.0), rel)
            self.compared[quantity] = self.compared.get(quantity, 0) + 1
            flat = self.tol * scale if scale > 0 else self.tol
            if err <= flat:
                continue
            extra = 0.0 if allow is None else KINK_SLACK * (float(allow[j]) + moved * scale)
            self.widest[quantity] = max(self.widest.get(quantity, 0.0), (flat + extra) / max(scale, 1e-12))
            self.fill[quantity] = max(self.fill.get(quantity, 0.0), err / (flat + extra))
            assert err <= flat + extra, (
                f"{quantity}, tensor {j}, {what}: relerr {rel:.3e} > {self.tol:.0e}"
                + (" and no near-kink decision was booked on the way to it" if extra == 0.0 else
                   f"; the booked jumps ({events} decisions) allow {(flat + extra) / max(scale, 1e-12):.3e}"))
            self.beyond[quantity] = self.beyond.get(quantity, 0) + 1

    def scalar(self, quantity, what, test, ref):
        rel = abs(test - ref) / max(abs(ref), 1e-12)
        self.worst[quantity] = max(self.worst.get(quantity, 0.0), rel)
        assert rel <= self.tol, f"{quantity}, {what}: relerr {rel:.3e} > {self.tol:.0e}"

    def summary(self):
        out = dict(self.worst)
        for q, n in self.beyond.items():
            out[q + "_beyond_flat"] = n
            out[q + "_compared"] = self.compared[q]
            out[q + "_widest_bar"] = self.widest[q]
            out[q + "_err/bar"] = self.fill[q]
        return out


def lockstep(wl, run, orc, rounds=None, check_every=1, tol=TOL, max_ticks=10000,
             check_clients=None, resync=False, kink_eps=KINK_EPS, stop_after_ticks=None):
    """Tick both sides until done; asserts the bar on the way and returns the worst relative
    errors seen (plus, for ReLU / pooling models, how many tensor comparisons lay beyond the
    flat bar and inside the booked jumps).
    check_every: U and w_c of the finishing clients and the global model are compared in
    every check_every-th tick (0: only the losses on the way, the models at the end).
    resync: see the module docstring (server form only).
    stop_after_ticks: compare this many ticks of the run and stop (the models are compared
    where the run stands then)."""
    R = wl.rounds if rounds is None else rounds
    model = wl.model
    kinks = has_kinks(model)
    nt = len(layer_slices(model))
    judge = Judge(model, tol)
    if kinks:
        orc.set_kink_eps(kink_eps)
    # what each model carries: jumps booked on the way to its current value (weight units)
    zero = np.zeros(nt)
    carry = {c: zero.copy() for c in range(-1, orc.n)}
    events_on = {c: 0 for c in range(-1, orc.n)}
    inflight = {}   # (c, k) -> (jumps of the message in weight units, decisions)
    ticks = 0

    slices = layer_slices(model)

    def moved(c, ref_w):
        """largest relative displacement the booked jumps allow in any tensor of model c"""
        return max(float(carry[c][j]) / max(float(np.abs(ref_w[s]).max()), 1e-12) for j, s in enumerate(slices))

    def compare_model(c, what):
        test, ref = run.lib.aet_get_weights(c), orc.get_weights(c)
        judge.tensors("Wg" if c < 0 else "w_c", what, test, ref,
                      carry[c] if kinks else None, events_on[c], moved=moved(c, ref) if kinks else 0.0)

    while not orc.all_done(R):
        assert not run.lib.aet_all_done(R)
        assert run.lib.aet_tick() == orc.tick
        full = check_every > 0 and ticks % check_every == 0
        # do both sides start this tick's rounds from the same bits?  (server form: the global
        # model; peer-to-peer form: every node's own)
        same_start = full and kinks and all(
            np.array_equal(run.lib.aet_get_weights(c).astype(np.float64), orc.get_weights(c))
            for c in (range(orc.n) if orc.p2p else (-1,)))
        fin_o = orc.run_round(R)
        fin_g = run.run_round(R)
        assert fin_g == fin_o, f"tick {orc.tick}: clients/rounds differ"
        for c, k in fin_o:
            io = orc.round_info(c, k)
            if kinks:
                ev, allow = orc.round_kinks(c, k)
                start = carry[c] if orc.p2p else carry[-1]
                start_ev = events_on[c] if orc.p2p else events_on[-1]
                carry[c] = start + io["eta"] * allow
                events_on[c] = start_ev + ev
                inflight[(c, k)] = (io["eta"] * allow, ev)
            if check_clients is not None and c not in check_clients:
                continue
            ig = run.lib.aet_get_round_info(c, k)
            for key in ("s", "m", "q0", "t0", "start_tick", "arrival"):
                assert ig[key] == io[key], (c, k, key)
            assert ig["eta"] == float(np.float32(io["eta"])), (c, k, "eta")
            what = f"client {c} round {k}"
            if full:
                # U: the round's own jumps, and what the starting model carried, in units of g
                Ug, Uo = run.lib.aet_get_U(c, k), orc.get_U(c, k)
                wo = orc.get_weights(c)
                mv = moved(c, wo) if kinks else 0.0
                if same_start or not kinks:
                    judge.tensors("U", what, Ug, Uo, carry[c] / io["eta"] if kinks else None, events_on[c], moved=mv)
                else:
                    judge.tensors("U_weight_units", what, io["eta"] * Ug.astype(np.float64), io["eta"] * Uo,
                                  carry[c], events_on[c], scale_of=wo, moved=mv)
                compare_model(c, what)
            if io["m"] > 0:
                judge.scalar("loss", what, ig["loss"], io["loss"])
        app_o = orc.exchange()
        app_g = run.exchange()
        assert app_g == app_o, f"tick {orc.tick - 1}: aggregation order differs"
        if kinks:
            for c, k in app_o:
                a, ev = inflight.pop((c, k))
                targets = [int(r) for r in wl.topology[1][wl.topology[0][c]:wl.topology[0][c + 1]]] if orc.p2p else [-1]
                for r in targets:
                    carry[r] = carry[r] + abs(wl.agg_scale) * a
                    events_on[r] += ev
        if (full or resync) and not orc.p2p:
            compare_model(-1, f"after tick {orc.tick - 1}")
        if resync:
            assert not orc.p2p
            w32 = orc.get_weights(-1).astype(np.float32)
            orc.set_weights(-1, w32)
            run.lib.aet_set_weights(-1, w32)
            carry[-1], events_on[-1] = zero.copy(), 0
        if full and orc.p2p:   # Receive has moved the neighbours' models
            for c in (range(orc.n) if check_clients is None else check_clients):
                compare_model(c, f"client {c} after tick {orc.tick - 1}")
        ticks += 1
        assert ticks <= max_ticks
        if stop_after_ticks is not None and ticks >= stop_after_ticks:
            break
    if stop_after_ticks is None:
        assert run.lib.aet_all_done(R)
        assert run.lib.aet_inflight() == 0
    if not resync and not orc.p2p:
        compare_model(-1, "end of run")
    for c in range(orc.n):
        assert run.lib.aet_history(c) == orc.history(c)
        if check_clients is None or c in check_clients:
            compare_model(c, f"client {c} at the end")
    return judge.summary()
