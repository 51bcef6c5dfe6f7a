"""Lets the parity helpers drive the oracle's fp32 build in the place of the library under
test: the CPU tests use it to exercise the comparison itself (bars, bookkeeping of booked
jumps, messages) without a GPU."""
from __future__ import annotations

import numpy as np


class _Lib:
    def __init__(self, orc):
        self.o = orc

    def aet_get_weights(self, c=-1):
        return self.o.get_weights(c).astype(np.float32)

    def aet_get_U(self, c, k):
        return self.o.get_U(c, k).astype(np.float32)

    def aet_set_weights(self, c, w):
        self.o.set_weights(c, np.asarray(w, dtype=np.float32))

    def aet_get_round_info(self, c, k):
        info = self.o.round_info(c, k)
        info["eta"] = float(np.float32(info["eta"]))
        return info

    def aet_all_done(self, R):
        return self.o.all_done(R)

    def aet_tick(self):
        return self.o.tick

    def aet_inflight(self):
        return int(self.o.lib.orc_queue_len(self.o.ctx))

    def aet_history(self, c):
        return self.o.history(c)


class OracleAsRun:
    def __init__(self, orc):
        self.o = orc
        self.lib = _Lib(orc)

    def run_round(self, R=None):
        return self.o.run_round(R)

    def exchange(self):
        return self.o.exchange()

    def close(self):
        self.o.close()
