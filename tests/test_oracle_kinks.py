"""Pins for the oracle's kink analysis (the bookkeeping behind the parity tolerance of ReLU /
max-pool networks): which decisions count as near a kink, and the jump of the sample's
gradient that a flipped decision causes, against the same quantities from PyTorch's CPU
autograd on a network whose ReLU masks and pooling choices are explicit tensors."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as W
from oracle import Oracle
from oracle.oracle import batch_loss_grad, sample_kinks

MODELS = {
    "mlp": W.mlp_model(6, 5, 3, batch=1),
    "lenet": W.Model(2, 8, 8, [W.Layer(W.CONV, 3, 3, 0, 1), W.Layer(W.POOL),
                                W.Layer(W.CONV, 4, 2, 0, 1), W.Layer(W.DENSE, 5, relu=1),
                                W.Layer(W.DENSE, 3)], 1),
    "cnn": W.Model(3, 8, 8, [W.Layer(W.CONV, 4, 3, 1, 1), W.Layer(W.CONV, 4, 3, 1, 1),
                              W.Layer(W.POOL), W.Layer(W.CONV, 5, 3, 1, 1), W.Layer(W.POOL),
                              W.Layer(W.DENSE, 6, relu=1), W.Layer(W.DENSE, 4)], 1),
}


def _sample(model, seed):
    g = np.random.default_rng(seed)
    x = g.uniform(-1, 1, model.in_size()).astype(np.float32)
    y = int(g.integers(0, model.n_classes()))
    w = g.uniform(-0.7, 0.7, model.n_params())
    return w, x, y


def _explicit_network(model, w, x, y):
    """Forward pass with every decision as data.  Returns per layer: the pre-activation z,
    the magnitude scale |b| + sum |w||x|, the layer's output `a` (a leaf-like tensor that
    keeps its gradient), for pooling layers the flat input index chosen per output and all
    four candidates; and the weight tensor."""
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(x, dtype=torch.float64).reshape(1, model.in_c, model.in_h, model.in_w)
    rec = []
    shp = model.shapes()
    for L, sl, (c, h, ww) in zip(model.layers, model.param_slices(), shp[:-1]):
        r = {"type": L.type, "relu": L.relu, "in": a}
        if L.type == W.CONV:
            Wt = wt[sl[0]:sl[0] + sl[1]].reshape(L.cout, c, L.k, L.k)
            b = wt[sl[2]:sl[2] + sl[3]]
            z = F.conv2d(a, Wt, b, padding=L.pad)
            r["scale"] = F.conv2d(a.abs(), Wt.abs(), b.abs(), padding=L.pad).detach().reshape(-1)
        elif L.type == W.DENSE:
            a = a.reshape(1, -1)
            r["in"] = a
            Wt = wt[sl[0]:sl[0] + sl[1]].reshape(L.cout, c * h * ww)
            b = wt[sl[2]:sl[2] + sl[3]]
            z = F.linear(a, Wt, b)
            r["scale"] = F.linear(a.abs(), Wt.abs(), b.abs()).detach().reshape(-1)
        else:
            win = a.reshape(c, h // 2, 2, ww // 2, 2).permute(0, 1, 3, 2, 4).reshape(c, h // 2, ww // 2, 4)
            flat = torch.arange(c * h * ww).reshape(c, h // 2, 2, ww // 2, 2).permute(0, 1, 3, 2, 4).reshape(c, h // 2, ww // 2, 4)
            vals = win.detach()
            # first maximum in window order
            choice = torch.zeros(vals.shape[:-1], dtype=torch.long)
            for j in range(1, 4):
                better = vals[..., j] > torch.gather(vals, -1, choice.unsqueeze(-1)).squeeze(-1)
                choice = torch.where(better, torch.full_like(choice, j), choice)
            z = torch.gather(win, -1, choice.unsqueeze(-1)).squeeze(-1).reshape(1, c, h // 2, ww // 2)
            r["choice"], r["flat"], r["vals"] = choice.reshape(-1), flat.reshape(-1, 4), vals.reshape(-1, 4)
        r["z"] = z
        if L.relu:
            mask = (z.detach() > 0).to(torch.float64)
            a = z * mask
        else:
            a = z
        a.retain_grad()
        r["a"] = a
        rec.append(r)
    loss = F.cross_entropy(a.reshape(1, -1), torch.tensor([y], dtype=torch.long))
    return wt, rec, loss


def _grad(scalar, wt):
    g, = torch.autograd.grad(scalar, wt, retain_graph=True, allow_unused=True)
    return np.zeros(wt.numel()) if g is None else g.numpy().copy()


def _expected_events(model, w, x, y, eps, guard=1e-9):
    """{(layer, unit): jump} from autograd; `unsure` holds decisions whose margin is within
    `guard` of eps (either side may count them)."""
    wt, rec, loss = _explicit_network(model, w, x, y)
    loss.backward(retain_graph=True)
    events, unsure = {}, set()
    for l, r in enumerate(rec):
        if r["type"] != W.POOL:
            if not r["relu"]:
                continue
            z = r["z"].reshape(-1)
            delta = r["a"].grad.reshape(-1)
            for o in range(z.numel()):
                margin = abs(float(z[o].detach())) / float(r["scale"][o])
                if abs(margin - eps) < guard:
                    unsure.add((l, o))
                elif margin < eps:
                    events[(l, o)] = float(delta[o]) * _grad(z[o], wt)
        else:
            below = rec[l - 1]
            a_in = below["a"].reshape(-1)
            delta = r["a"].grad.reshape(-1)
            for o in range(r["choice"].numel()):
                vals, flat, ch = r["vals"][o], r["flat"][o], int(r["choice"][o])
                if not float(vals[ch]) > 0:
                    continue
                others = [j for j in range(4) if j != ch]
                sec = others[0]
                for j in others[1:]:
                    if float(vals[j]) > float(vals[sec]):
                        sec = j
                sc = max(float(below["scale"][int(flat[ch])]), float(below["scale"][int(flat[sec])]))
                margin = (float(vals[ch]) - float(vals[sec])) / sc
                if abs(margin - eps) < guard:
                    unsure.add((l, o))
                elif margin < eps:
                    events[(l, o)] = float(delta[o]) * (_grad(a_in[int(flat[sec])], wt) - _grad(a_in[int(flat[ch])], wt))
    return events, unsure


@pytest.mark.parametrize("name", list(MODELS))
@pytest.mark.parametrize("eps", [0.02, 0.3])
def test_events_and_jumps_match_autograd(oracle_libs, name, eps):
    model = MODELS[name]
    found_any = False
    for seed in range(3):
        w, x, y = _sample(model, 10 + seed)
        want, unsure = _expected_events(model, w, x, y, eps)
        got, allow, n = sample_kinks(model, w, x, y, eps)
        assert n == len(got)
        got = {(l, o): j for l, o, j in got}
        assert set(got) - unsure == set(want) - unsure
        for key in set(want) - unsure:
            scale = max(1e-12, np.abs(want[key]).max())
            assert np.abs(got[key] - want[key]).max() <= 1e-11 * max(1.0, scale), key
            found_any = found_any or scale > 1e-6
        if not unsure:
            # per parameter tensor: sum over the events of the largest |entry| of the jump
            exp = []
            for sl in model.param_slices():
                if sl is None:
                    continue
                for a, nn in ((sl[0], sl[1]), (sl[2], sl[3])):
                    exp.append(sum(np.abs(j[a:a + nn]).max() for j in want.values()))
            assert np.allclose(allow, exp, rtol=1e-10, atol=1e-14)
    assert found_any, "no decision with a non-zero jump was exercised"


def test_a_unit_put_exactly_on_its_kink_is_found_and_the_jump_is_the_gradient_difference(oracle_libs):
    """Dense ReLU unit moved onto z = 0 through its bias: the gradient with the unit on (bias
    a hair above) minus the gradient with it off (a hair below) is the reported jump."""
    model = MODELS["mlp"]
    w, x, y = _sample(model, 3)
    sl = model.param_slices()[0]
    Wm = w[sl[0]:sl[0] + sl[1]].reshape(5, 6)
    unit = 2
    z = Wm[unit] @ x.astype(np.float64) + w[sl[2] + unit]
    w[sl[2] + unit] -= z
    ev, _, n = sample_kinks(model, w, x, y, 1e-9)
    assert n == 1 and ev[0][0] == 0 and ev[0][1] == unit
    h = 1e-7
    wp, wm = w.copy(), w.copy()
    wp[sl[2] + unit] += h
    wm[sl[2] + unit] -= h
    _, gp = batch_loss_grad(model, wp, x[None], np.array([y], dtype=np.int32))
    _, gm = batch_loss_grad(model, wm, x[None], np.array([y], dtype=np.int32))
    assert np.abs((gp - gm) - ev[0][2]).max() <= 1e-5 * np.abs(ev[0][2]).max()
    assert np.abs(ev[0][2]).max() > 1e-3


def test_no_relu_no_pool_no_events(oracle_libs):
    model = W.softmax_model(7, 4)
    w, x, y = _sample(model, 5)
    ev, allow, n = sample_kinks(model, w, x, y, 0.5)
    assert n == 0 and not ev and not allow.any()


def test_round_allowance_is_the_sum_over_its_samples(oracle_libs):
    """orc_run_round with the analysis on: the round's allowance equals the per-sample
    allowances at the weights of each recursion, divided by the mini-batch size; results of
    the round itself do not change."""
    wl = W.config3(n_clients=2, n_per=30, hw=16, batch=3, rounds=2, a=3, b=6)
    eps = 0.05
    plain, orc = Oracle(wl), Oracle(wl)
    orc.set_kink_eps(eps)
    assert orc.run_round() == plain.run_round() == [(0, 0), (1, 0)]
    B, model = wl.model.batch, wl.model
    for c in range(2):
        assert np.array_equal(orc.get_U(c, 0), plain.get_U(c, 0))
        assert np.array_equal(orc.get_weights(c), plain.get_weights(c))
        info = orc.round_info(c, 0)
        w = wl.w0.astype(np.float64)
        eta = info["eta"]
        tot, nev = 0.0, 0
        for u in range(info["m"]):
            idx = [orc.sample_index(c, info["q0"] + u * B + j, wl.X[c].shape[0]) for j in range(B)]
            for i in idx:
                _, allow, n = sample_kinks(model, w, wl.X[c][i], int(wl.y[c][i]), eps, cap=0)
                tot = tot + allow / B
                nev += n
            _, g = batch_loss_grad(model, w, wl.X[c][idx], wl.y[c][idx])
            w = w - eta * g
        ev, allow = orc.round_kinks(c, 0)
        assert ev == nev and nev > 0
        assert np.allclose(allow, tot, rtol=1e-12, atol=0)
    with pytest.raises(RuntimeError):
        plain.round_kinks(0, 0)
