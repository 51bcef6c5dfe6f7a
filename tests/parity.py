"""Helpers of the GPU parity tests: drive the CPU oracle (fp64) and the HIP library in
lock step on the same seeded workload and compare them.

Bars: bit-exact for everything integer (which clients run, round numbers, round lengths,
sample counters, ticks, sample indices, the order in which arrivals are applied); for
floating point, per tensor  max|gpu - cpu| / max(max|cpu|, 1e-12) <= tol  with tol = 1e-4
(fp32 results after 20 rounds), and the round step size must be the fp32 rounding of the
oracle's double."""
from __future__ import annotations

import numpy as np

TOL = 1e-4


def relerr(gpu: np.ndarray, cpu: np.ndarray) -> float:
    return float(np.abs(gpu.astype(np.float64) - cpu).max() / max(np.abs(cpu).max(), 1e-12))


def layer_slices(model):
    out = []
    for sl in model.param_slices():
        if sl is None:
            continue
        out.append(slice(sl[0], sl[0] + sl[1]))
        out.append(slice(sl[2], sl[2] + sl[3]))
    return out


def tensor_relerr(model, gpu: np.ndarray, cpu: np.ndarray) -> float:
    """Worst per-tensor relative error (each layer's weights and bias on their own);
    a tensor that is exactly zero on the CPU side must be (almost) zero on the GPU."""
    worst = 0.0
    for s in layer_slices(model):
        worst = max(worst, relerr(gpu[s], cpu[s]) if np.abs(cpu[s]).max() > 0 else float(np.abs(gpu[s]).max()))
    return worst


def lockstep(wl, run, orc, rounds=None, check_every_tick=True, tol=TOL, max_ticks=10000,
             check_clients=None):
    """Tick both sides until done.  Returns the worst relative errors seen."""
    R = wl.rounds if rounds is None else rounds
    model = wl.model
    worst = dict(U=0.0, W=0.0, Wg=0.0, loss=0.0)
    ticks = 0
    while not orc.all_done(R):
        assert not run.lib.aet_all_done(R)
        assert run.lib.aet_tick() == orc.tick
        fin_o = orc.run_round(R)
        fin_g = run.run_round(R)
        assert fin_g == fin_o, f"tick {orc.tick}: clients/rounds differ"
        for c, k in fin_o:
            if check_clients is not None and c not in check_clients:
                continue
            io, ig = orc.round_info(c, k), run.lib.aet_get_round_info(c, k)
            for key in ("s", "m", "q0", "t0", "start_tick", "arrival"):
                assert ig[key] == io[key], (c, k, key)
            assert ig["eta"] == float(np.float32(io["eta"])), (c, k, "eta")
            if check_every_tick:
                e = tensor_relerr(model, run.lib.aet_get_U(c, k), orc.get_U(c, k))
                worst["U"] = max(worst["U"], e)
                assert e <= tol, f"U of client {c} round {k}: relerr {e:.3e}"
                e = tensor_relerr(model, run.lib.aet_get_weights(c), orc.get_weights(c))
                worst["W"] = max(worst["W"], e)
                assert e <= tol, f"w_c of client {c} round {k}: relerr {e:.3e}"
            if io["m"] > 0:
                e = abs(ig["loss"] - io["loss"]) / max(abs(io["loss"]), 1e-12)
                worst["loss"] = max(worst["loss"], e)
                assert e <= tol, f"loss of client {c} round {k}: {ig['loss']} vs {io['loss']}"
        app_o = orc.server_aggregate()
        app_g = run.server_aggregate()
        assert app_g == app_o, f"tick {orc.tick - 1}: aggregation order differs"
        if check_every_tick:
            e = tensor_relerr(model, run.lib.aet_get_weights(-1), orc.get_weights(-1))
            worst["Wg"] = max(worst["Wg"], e)
            assert e <= tol, f"global model after tick {orc.tick - 1}: relerr {e:.3e}"
        ticks += 1
        assert ticks <= max_ticks
    assert run.lib.aet_all_done(R)
    assert run.lib.aet_inflight() == 0
    e = tensor_relerr(model, run.lib.aet_get_weights(-1), orc.get_weights(-1))
    worst["Wg"] = max(worst["Wg"], e)
    assert e <= tol, f"final global model: relerr {e:.3e}"
    for c in range(orc.n):
        assert run.lib.aet_history(c) == orc.history(c)
        if check_clients is not None and c not in check_clients:
            continue
        e = tensor_relerr(model, run.lib.aet_get_weights(c), orc.get_weights(c))
        worst["W"] = max(worst["W"], e)
        assert e <= tol, f"final w_c of client {c}: relerr {e:.3e}"
    return worst
