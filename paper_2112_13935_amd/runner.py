"""Drive a workload record (model, shards, schedule parameters) through the library:
upload the shards with PyTorch, then call aet_run_round and aet_server_aggregate (or
aet_receive, when the workload has a topology) per tick.
Marshalling only; used by the tests, the smoke check and the benchmark."""
from __future__ import annotations

from typing import Optional

import torch

from .binding import AetSgd


def upload(wl, device="cuda:0", n_clients: Optional[int] = None):
    n = wl.n_clients if n_clients is None else n_clients
    X = [torch.from_numpy(wl.X[c]).to(device) for c in range(n)]
    y = [torch.from_numpy(wl.y[c]).to(device) for c in range(n)]
    return X, y


class Run:
    def __init__(self, wl, device="cuda:0", shards=None, max_rounds: Optional[int] = None,
                 static_workspace: bool = False):
        self.wl = wl
        self.X, self.y = shards if shards is not None else upload(wl, device)
        self.n = len(self.X)
        self.lib = AetSgd(wl.model, self.X, self.y, wl.w0, wl.seed,
                          max_inflight=wl.delay_max + 1,
                          max_rounds=max(1, wl.rounds if max_rounds is None else max_rounds),
                          static_workspace=static_workspace)
        if getattr(wl, "setup_weights", None) is not None and self.n == wl.n_clients:
            self.lib.aet_set_setup(wl.setup_weights, wl.setup_seed)
        self.p2p = getattr(wl, "topology", None) is not None and self.n == wl.n_clients
        if self.p2p:
            self.lib.aet_set_topology(*wl.topology)

    def run_round(self, rounds: Optional[int] = None):
        wl = self.wl
        return self.lib.aet_run_round(
            wl.a, wl.b, wl.rounds if rounds is None else rounds, wl.eta0, wl.beta, wl.power,
            None if wl.compute_factor is None else wl.compute_factor[: self.n],
            None if wl.is_straggler is None else wl.is_straggler[: self.n],
            wl.delay_min, wl.delay_max, wl.delay_seed, wl.d_max)

    def server_aggregate(self):
        return self.lib.aet_server_aggregate(self.wl.agg_scale)

    def receive(self):
        return self.lib.aet_receive(self.wl.agg_scale)

    def exchange(self):
        """The tick's second half: Receive at the neighbours or at the server."""
        return self.receive() if self.p2p else self.server_aggregate()

    def run_all(self, rounds: Optional[int] = None, max_ticks: int = 100000) -> int:
        R = self.wl.rounds if rounds is None else rounds
        ticks = 0
        while not self.lib.aet_all_done(R):
            self.run_round(R)
            self.exchange()
            ticks += 1
            if ticks > max_ticks:
                raise RuntimeError("run did not finish")
        return ticks

    def run_ticks(self, rounds: Optional[int] = None, max_ticks: int = 1 << 30) -> int:
        """The same loop inside the library (one call for the whole job)."""
        wl = self.wl
        return self.lib.aet_run_ticks(
            wl.a, wl.b, wl.rounds if rounds is None else rounds, wl.eta0, wl.beta, wl.power,
            wl.agg_scale,
            None if wl.compute_factor is None else wl.compute_factor[: self.n],
            None if wl.is_straggler is None else wl.is_straggler[: self.n],
            wl.delay_min, wl.delay_max, wl.delay_seed, wl.d_max, max_ticks)

    def close(self):
        self.lib.aet_destroy()
