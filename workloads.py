"""Seeded synthetic workloads: model descriptions, data shards, initial weights and
delay-schedule inputs for the five AET-SGD configurations.

This module is the only thing the CPU oracle and the HIP path have in common.  It holds
none of the method's arithmetic (no gradients, no thresholds, no step sizes, no sample
indexing, no aggregation): it only produces *inputs* — arrays and parameter records —
that both sides consume.  Everything is drawn from numpy's Philox counter generator with
a fixed seed, so the same call returns the same bytes on every machine.

The data stand in for MNIST-like (28x28x1) and CIFAR10-like (32x32x3) image sets that the
paper trains on (Appendix, "Data sets"); only their shapes and class counts are taken.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 211213935

# layer types (shared vocabulary of the two model descriptions)
CONV, POOL, DENSE = 0, 1, 2


@dataclass
class Layer:
    type: int          # CONV / POOL / DENSE
    cout: int = 0      # output channels (conv) or output features (dense)
    k: int = 0         # square kernel size (conv)
    pad: int = 0       # zero padding on each side (conv)
    relu: int = 0      # ReLU after the affine map


@dataclass
class Model:
    in_c: int
    in_h: int
    in_w: int
    layers: List[Layer]
    batch: int

    def shapes(self) -> List[Tuple[int, int, int]]:
        """Activation shape (C, H, W) before the first layer and after every layer."""
        c, h, w = self.in_c, self.in_h, self.in_w
        out = [(c, h, w)]
        for L in self.layers:
            if L.type == CONV:
                c, h, w = L.cout, h + 2 * L.pad - L.k + 1, w + 2 * L.pad - L.k + 1
            elif L.type == POOL:
                c, h, w = c, h // 2, w // 2
            else:
                c, h, w = L.cout, 1, 1
            out.append((c, h, w))
        return out

    def param_slices(self) -> List[Optional[Tuple[int, int, int, int]]]:
        """Per layer (w_off, w_count, b_off, b_count) in the canonical flat layout:
        layers in order, weights then bias; dense W[out][in]; conv W[cout][cin][kh][kw]."""
        shp = self.shapes()
        off = 0
        out = []
        for L, (c, h, w) in zip(self.layers, shp[:-1]):
            if L.type == CONV:
                nw = L.cout * c * L.k * L.k
            elif L.type == DENSE:
                nw = L.cout * c * h * w
            else:
                out.append(None)
                continue
            out.append((off, nw, off + nw, L.cout))
            off += nw + L.cout
        return out

    def n_params(self) -> int:
        return sum(s[1] + s[3] for s in self.param_slices() if s is not None)

    def in_size(self) -> int:
        return self.in_c * self.in_h * self.in_w

    def n_classes(self) -> int:
        return self.layers[-1].cout


def softmax_model(d: int, classes: int, batch: int = 1) -> Model:
    return Model(d, 1, 1, [Layer(DENSE, classes)], batch)


def mlp_model(d: int, hidden: int, classes: int, batch: int) -> Model:
    return Model(d, 1, 1, [Layer(DENSE, hidden, relu=1), Layer(DENSE, classes)], batch)


def lenet_model(batch: int, hw: int = 28) -> Model:
    return Model(1, hw, hw, [
        Layer(CONV, 6, 5, 0, 1), Layer(POOL),
        Layer(CONV, 16, 5, 0, 1), Layer(POOL),
        Layer(DENSE, 120, relu=1), Layer(DENSE, 84, relu=1), Layer(DENSE, 10)], batch)


def cnn32_model(batch: int, hw: int = 32, width: int = 32, fc: int = 256) -> Model:
    return Model(3, hw, hw, [
        Layer(CONV, width, 3, 1, 1), Layer(CONV, width, 3, 1, 1), Layer(POOL),
        Layer(CONV, 2 * width, 3, 1, 1), Layer(CONV, 2 * width, 3, 1, 1), Layer(POOL),
        Layer(DENSE, fc, relu=1), Layer(DENSE, 10)], batch)


@dataclass
class Workload:
    name: str
    model: Model
    n_clients: int
    X: List[np.ndarray]            # per client, float32 [N_c, in_size]
    y: List[np.ndarray]            # per client, int32 [N_c]
    w0: np.ndarray                 # float32 [P], canonical layout
    a: int                         # threshold s_i = a*i + b (samples)
    b: int
    rounds: int                    # local rounds per client
    eta0: float
    beta: float
    power: float
    agg_scale: float               # server scale on eta_k * U
    seed: int                      # seed of the sample-index streams
    compute_factor: Optional[np.ndarray] = None   # int32 [n], ticks per local round
    is_straggler: Optional[np.ndarray] = None     # uint8 [n]
    delay_min: int = 0
    delay_max: int = 0
    delay_seed: int = 0
    d_max: int = -1                # SYNCHRONIZE gate off
    notes: str = ""
    topology: Optional[tuple] = None   # (nbr_off, nbr) neighbour lists: peer-to-peer form
    setup_weights: Optional[np.ndarray] = None    # uint32 [n]: p_c = w_c / sum(w); the threshold
    setup_seed: int = 0                           # is then the global sequence s_i (Algorithm 1)

    def total_client_samples(self, rounds: Optional[int] = None) -> int:
        R = self.rounds if rounds is None else rounds
        if self.setup_weights is not None:      # the nodes share the global rounds
            return sum(self.a * i + self.b for i in range(R))
        return self.n_clients * sum(self.a * i + self.b for i in range(R))


def topology_from_edges(n: int, edges) -> tuple:
    """Neighbour lists (CSR: nbr_off int32 [n+1], nbr int32, ascending per node) of the
    undirected graph with the given edges; duplicates and self loops are dropped."""
    adj = [set() for _ in range(n)]
    for u, v in edges:
        u, v = int(u) % n, int(v) % n
        if u != v:
            adj[u].add(v)
            adj[v].add(u)
    off = np.zeros(n + 1, dtype=np.int32)
    for c in range(n):
        off[c + 1] = off[c] + len(adj[c])
    nbr = np.array([v for c in range(n) for v in sorted(adj[c])], dtype=np.int32)
    return off, nbr


def ring_topology(n: int) -> tuple:
    """Every node talks to its two ring neighbours (one neighbour when n = 2, none when n = 1)."""
    return topology_from_edges(n, [(c, c + 1) for c in range(n)])


def line_topology(n: int) -> tuple:
    return topology_from_edges(n, [(c, c + 1) for c in range(n - 1)])


def complete_topology(n: int) -> tuple:
    return topology_from_edges(n, [(u, v) for u in range(n) for v in range(u + 1, n)])


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), stream]))


def init_weights(model: Model, seed: int, zero: bool = False) -> np.ndarray:
    """U(-1/sqrt(fan_in), 1/sqrt(fan_in)) for weights and biases, or zeros."""
    P = model.n_params()
    w = np.zeros(P, dtype=np.float32)
    if zero:
        return w
    g = _rng(seed, 7)
    shp = model.shapes()
    for L, sl, (c, h, ww) in zip(model.layers, model.param_slices(), shp[:-1]):
        if sl is None:
            continue
        fan_in = c * L.k * L.k if L.type == CONV else c * h * ww
        bound = 1.0 / np.sqrt(fan_in)
        w[sl[0]:sl[0] + sl[1]] = g.uniform(-bound, bound, sl[1]).astype(np.float32)
        w[sl[2]:sl[2] + sl[3]] = g.uniform(-bound, bound, sl[3]).astype(np.float32)
    return w


def straggler_flags(n: int, frac: float, seed: int) -> np.ndarray:
    """First floor(frac*n) clients of a seeded permutation are stragglers."""
    perm = _rng(seed, 11).permutation(n)
    flags = np.zeros(n, dtype=np.uint8)
    flags[perm[: int(np.floor(frac * n))]] = 1
    return flags


def compute_factors(n: int, choices: Tuple[int, ...], seed: int) -> np.ndarray:
    return _rng(seed, 13).choice(np.array(choices, dtype=np.int32), size=n).astype(np.int32)


def class_gaussian(n: int, d: int, classes: int, seed: int, sigma: float, clip: bool,
                   labels: Optional[np.ndarray] = None, mean_lo: float = 0.0,
                   mean_hi: float = 1.0, means: Optional[np.ndarray] = None,
                   stream: int = 3):
    """x = mu[label] + sigma*N(0,1) (optionally clipped to [0,1]); labels uniform."""
    g = _rng(seed, stream)
    if means is None:
        means = _rng(seed, 5).uniform(mean_lo, mean_hi, (classes, d)).astype(np.float32)
    if labels is None:
        labels = g.integers(0, classes, n).astype(np.int32)
    X = g.standard_normal((n, d), dtype=np.float32)
    X *= np.float32(sigma)
    X += means[labels]
    if clip:
        np.clip(X, 0.0, 1.0, out=X)
    return X, labels.astype(np.int32), means


def teacher_labels(X: np.ndarray, classes: int, seed: int, noise: float) -> np.ndarray:
    """argmax of a seeded random linear teacher plus N(0, noise^2) on the scores."""
    g = _rng(seed, 17)
    T = g.standard_normal((classes, X.shape[1]))
    s = X.astype(np.float64) @ T.T + noise * g.standard_normal((X.shape[0], classes))
    return np.argmax(s, axis=1).astype(np.int32)


# ----------------------------------------------------------------------------------------
# The five configurations (scaled-down variants are made by passing smaller n / N / dims)
# ----------------------------------------------------------------------------------------

def config1(n_clients: int = 4, n_per: int = 1000, d: int = 784, rounds: int = 20,
            a: int = 10, b: int = 10) -> Workload:
    """Softmax regression, per-sample SGD, constant eta, zero delay.  The server averages
    the clients' displacements (agg_scale = 1/n): with the unscaled rule this data scale
    and step size leave the stable regime (the loss grows to ~280) and fp32 and fp64 runs
    drift apart by more than the parity tolerance."""
    seed = BASE_SEED + 1
    X, y = [], []
    for c in range(n_clients):
        Xc = _rng(seed, 100 + c).uniform(0.0, 1.0, (n_per, d)).astype(np.float32)
        X.append(Xc)
        y.append(teacher_labels(Xc, 10, seed, 0.1))
    m = softmax_model(d, 10, 1)
    return Workload("cfg1_softmax784", m, n_clients, X, y, init_weights(m, seed, zero=True),
                    a, b, rounds, 0.01, 0.0, 1.0, 1.0 / n_clients, seed)


def config2(n_clients: int = 16, n_total: int = 60000, d: int = 784, hidden: int = 128,
            batch: int = 32, rounds: int = 50, a: int = 32, b: int = 64) -> Workload:
    """MLP, iid split of one class-conditional Gaussian set, diminishing eta."""
    seed = BASE_SEED + 2
    Xall, yall, _ = class_gaussian(n_total, d, 10, seed, 0.3, True)
    perm = _rng(seed, 19).permutation(n_total)
    per = n_total // n_clients
    X = [np.ascontiguousarray(Xall[perm[c * per:(c + 1) * per]]) for c in range(n_clients)]
    y = [np.ascontiguousarray(yall[perm[c * per:(c + 1) * per]]) for c in range(n_clients)]
    m = mlp_model(d, hidden, 10, batch)
    return Workload("cfg2_mlp784", m, n_clients, X, y, init_weights(m, seed), a, b, rounds,
                    0.05, 0.001, 1.0, 1.0 / n_clients, seed)


def config3(n_clients: int = 64, n_per: int = 1000, hw: int = 28, batch: int = 16,
            rounds: int = 40, a: int = 16, b: int = 32) -> Workload:
    """LeNet-5-style CNN, non-iid label skew (2 classes per client), 25% stragglers whose
    messages arrive 1-3 rounds late."""
    seed = BASE_SEED + 3
    d = hw * hw
    means = _rng(seed, 5).uniform(0.0, 1.0, (10, d)).astype(np.float32)
    X, y = [], []
    for c in range(n_clients):
        lab = np.repeat(np.array([2 * (c % 5), 2 * (c % 5) + 1], dtype=np.int32), n_per // 2)
        lab = np.concatenate([lab, np.full(n_per - lab.size, 2 * (c % 5), np.int32)])
        Xc, yc, _ = class_gaussian(n_per, d, 10, seed, 0.3, True, labels=lab, means=means,
                                   stream=200 + c)
        X.append(Xc)
        y.append(yc)
    m = lenet_model(batch, hw)
    return Workload("cfg3_lenet", m, n_clients, X, y, init_weights(m, seed), a, b, rounds,
                    0.01, 0.0, 1.0, 1.0 / n_clients, seed,
                    is_straggler=straggler_flags(n_clients, 0.25, seed),
                    delay_min=1, delay_max=3, delay_seed=seed ^ 0xD1A7)


def config4(n_clients: int = 32, n_per: int = 1500, hw: int = 32, width: int = 32,
            fc: int = 256, batch: int = 64, rounds: int = 30, a: int = 64,
            b: int = 128) -> Workload:
    """Small 4-conv CNN on 3-channel images, per-class per-channel Gaussian means,
    compute-delay factors from {1,2,4}."""
    seed = BASE_SEED + 4
    ch_means = _rng(seed, 5).uniform(0.0, 1.0, (10, 3)).astype(np.float32)
    means = np.repeat(ch_means, hw * hw, axis=1)          # (10, 3*hw*hw), layout C,H,W
    X, y = [], []
    for c in range(n_clients):
        Xc, yc, _ = class_gaussian(n_per, 3 * hw * hw, 10, seed, 0.3, False, means=means,
                                   stream=300 + c)
        X.append(Xc)
        y.append(yc)
    m = cnn32_model(batch, hw, width, fc)
    return Workload("cfg4_cnn32", m, n_clients, X, y, init_weights(m, seed), a, b, rounds,
                    0.01, 0.0, 1.0, 1.0 / n_clients, seed,
                    compute_factor=compute_factors(n_clients, (1, 2, 4), seed))


def config5(n_clients: int = 1024, n_per: int = 500, d: int = 3072, rounds: int = 60,
            a: int = 5, b: int = 5) -> Workload:
    """Scale test: softmax regression, many small replicas, Gaussian mixture with the
    feature scale chosen so that E|x|^2 is O(1), 10% stragglers delayed 1-5 rounds."""
    seed = BASE_SEED + 5
    centres = (_rng(seed, 5).standard_normal((10, d)) * (2.0 / np.sqrt(d))).astype(np.float32)
    X, y = [], []
    for c in range(n_clients):
        Xc, yc, _ = class_gaussian(n_per, d, 10, seed, 1.0 / np.sqrt(d), False, means=centres,
                                   stream=400 + c)
        X.append(Xc)
        y.append(yc)
    m = softmax_model(d, 10, 1)
    return Workload("cfg5_softmax3072", m, n_clients, X, y, init_weights(m, seed, zero=True),
                    a, b, rounds, 0.01, 0.0, 1.0, 1.0 / n_clients, seed,
                    is_straggler=straggler_flags(n_clients, 0.10, seed),
                    delay_min=1, delay_max=5, delay_seed=seed ^ 0xD1A7)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
