"""Pins for the CPU oracle: every check compares the oracle with something
that is not the oracle (finite differences, a library LSTM, closed forms,
hand-computed scalars, invariants, values the paper prints)."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import lstm_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")


def _rand_params(rng, L, I, H, vocab=0, embed=0, scale=0.5):
    shapes = orc.param_shapes(L, I, H, vocab, embed)
    p = {n: rng.uniform(-scale, scale, s) for n, s in shapes}
    return p, shapes


def _targets(rng, head, T, B):
    if head == orc.HEAD_LAST_BCE:
        return (rng.random((B, 1)) < 0.5).astype(np.float64)
    if head == orc.HEAD_STEP_MSE:
        return rng.standard_normal((T, B, 1))
    return (rng.random((T, B, 1)) < 0.3).astype(np.float64)


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("L,head,vocab", [(1, 1, 0), (2, 1, 0), (1, 2, 0), (2, 3, 0), (1, 2, 11), (3, 2, 0)])
def test_backward_matches_central_differences(L, head, vocab):
    rng = np.random.default_rng(100 + 10 * L + head)
    T, B, I, H, E = 4, 3, 5, 4, 6
    p, shapes = _rand_params(rng, L, I, H, vocab, E if vocab else 0)
    x = rng.integers(0, vocab, (T, B)) if vocab else rng.standard_normal((T, B, I))
    if vocab:
        x[0, 0] = x[1, 1] = x[2, 2]          # repeated ids must accumulate
    y = _targets(rng, head, T, B)
    S = 8.0
    loss, cache = orc.forward(p, L, x, y, head)
    g = orc.backward(p, L, cache, S)
    eps = 1e-6
    for name, _ in shapes:
        flat = p[name].reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 12), replace=False)
        for k in idx:
            old = flat[k]
            flat[k] = old + eps
            lp, _ = orc.forward(p, L, x, y, head)
            flat[k] = old - eps
            lm, _ = orc.forward(p, L, x, y, head)
            flat[k] = old
            fd = S * (lp - lm) / (2 * eps)
            an = g[name].reshape(-1)[k]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 2e-8, (name, k, fd, an)


@pytest.mark.parametrize("L,head", [(1, 1), (2, 3), (3, 2)])
def test_backward_fd_with_initial_state(L, head):
    """Central differences of S * loss over EVERY element of every tensor with a non-zero initial state:
    the t = 0 contributions (dU from h_prev = h0, the forget-gate term dc * c0, the upper layers' own
    h0 / c0) are part of every difference, so a wrong or dropped one fails here."""
    rng = np.random.default_rng(50 + L)
    T, B, I, H = 3, 2, 3, 3
    p, shapes = _rand_params(rng, L, I, H)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, head, T, B)
    h0 = rng.uniform(-0.9, 0.9, (L, B, H)); c0 = rng.uniform(-1.5, 1.5, (L, B, H))
    S = 4.0
    l0, _ = orc.forward(p, L, x, y, head)
    l1, cache = orc.forward(p, L, x, y, head, h0, c0)
    assert abs(l0 - l1) > 1e-6
    assert np.array_equal(cache["layers"][0]["h"][0], h0[0])
    assert np.array_equal(cache["layers"][L - 1]["c"][0], c0[L - 1])
    g = orc.backward(p, L, cache, S)
    g_zero = orc.backward(p, L, orc.forward(p, L, x, y, head)[1], S)
    eps = 1e-6
    for name, _ in shapes:
        flat = p[name].reshape(-1)
        for k in range(flat.size):
            old = flat[k]
            flat[k] = old + eps
            lp, _ = orc.forward(p, L, x, y, head, h0, c0)
            flat[k] = old - eps
            lm, _ = orc.forward(p, L, x, y, head, h0, c0)
            flat[k] = old
            fd = S * (lp - lm) / (2 * eps)
            an = g[name].reshape(-1)[k]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 2e-8, (name, k, fd, an)
    # the state really enters the gradients (the pin above is not the zero-state pin in disguise)
    for l in range(L):
        assert np.max(np.abs(g[f"U{l}"] - g_zero[f"U{l}"])) > 1e-4


def test_single_step_gradients_come_from_the_initial_state_only():
    """T = 1: dU = dA^T h0 exists only because of h0, and the forget-gate rows of every gradient only
    because of c0 (df = dc * c0).  With c0 = 0 those rows vanish exactly; with h0 = 0, dU does."""
    rng = np.random.default_rng(61)
    L, T, B, I, H = 1, 1, 3, 2, 4
    p, shapes = _rand_params(rng, L, I, H)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 3, T, B)
    h0 = rng.uniform(-0.9, 0.9, (L, B, H)); c0 = rng.uniform(-1.5, 1.5, (L, B, H))
    _, ca = orc.forward(p, L, x, y, 3, h0, np.zeros_like(c0))
    ga = orc.backward(p, L, ca, 1.0)
    assert np.all(ga["b0"][H:2 * H] == 0.0) and np.all(ga["W0"][H:2 * H] == 0.0) and np.all(ga["U0"][H:2 * H] == 0.0)
    assert np.max(np.abs(ga["U0"][:H])) > 1e-6
    _, cb = orc.forward(p, L, x, y, 3, np.zeros_like(h0), c0)
    gb = orc.backward(p, L, cb, 1.0)
    assert np.all(gb["U0"] == 0.0)
    assert np.max(np.abs(gb["b0"][H:2 * H])) > 1e-6
    # hand-written single cell, one sample, against the oracle's df row: df = dc * c0, da_f = df f (1 - f)
    b = 1
    a = p["W0"] @ x[0, b] + p["U0"] @ h0[0, b] + p["b0"]
    i = 1 / (1 + np.exp(-a[:H])); f = 1 / (1 + np.exp(-a[H:2 * H])); gg = np.tanh(a[2 * H:3 * H]); o = 1 / (1 + np.exp(-a[3 * H:]))
    c = f * c0[0, b] + i * gg
    h = o * np.tanh(c)
    z = h @ p["w_head"] + p["b_head"][0]
    dz = 2.0 * (z - y[0, b, 0]) / (T * B)
    dc = dz * p["w_head"] * o * (1 - np.tanh(c) ** 2)
    da_f = dc * c0[0, b] * f * (1 - f)
    _, cc = orc.forward(p, L, x[:, b:b + 1], y[:, b:b + 1], 3, h0[:, b:b + 1], c0[:, b:b + 1])
    gc = orc.backward(p, L, cc, 1.0)
    np.testing.assert_allclose(gc["b0"][H:2 * H] / B, da_f, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(gc["U0"][H:2 * H] / B, np.outer(da_f, h0[0, b]), rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("L", [1, 2, 3])
def test_initial_state_matches_torch_lstm_autograd(L):
    """torch.nn.LSTM with (h0, c0) passed in, fp64, bias_hh = 0: loss, final states and every gradient."""
    rng = np.random.default_rng(70 + L)
    T, B, I, H = 5, 4, 3, 6
    p, shapes = _rand_params(rng, L, I, H, scale=0.4)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 3, T, B)
    h0 = rng.uniform(-0.9, 0.9, (L, B, H)); c0 = rng.uniform(-1.5, 1.5, (L, B, H))
    loss, cache = orc.forward(p, L, x, y, orc.HEAD_STEP_MSE, h0, c0)
    g = orc.backward(p, L, cache, 2.0)
    lstm = torch.nn.LSTM(I, H, num_layers=L, bias=True).double()
    with torch.no_grad():
        for l in range(L):
            getattr(lstm, f"weight_ih_l{l}").copy_(torch.from_numpy(p[f"W{l}"]))
            getattr(lstm, f"weight_hh_l{l}").copy_(torch.from_numpy(p[f"U{l}"]))
            getattr(lstm, f"bias_ih_l{l}").copy_(torch.from_numpy(p[f"b{l}"]))
            getattr(lstm, f"bias_hh_l{l}").zero_()
    wh = torch.from_numpy(p["w_head"]).requires_grad_()
    bh = torch.from_numpy(p["b_head"]).requires_grad_()
    out, (hT, cT) = lstm(torch.from_numpy(x), (torch.from_numpy(h0), torch.from_numpy(c0)))
    z = out @ wh + bh
    tl = torch.nn.functional.mse_loss(z, torch.from_numpy(y[..., 0]))
    (2.0 * tl).backward()
    assert abs(loss - tl.item()) < 1e-12
    for l in range(L):
        np.testing.assert_allclose(cache["layers"][l]["h"][-1], hT[l].detach().numpy(), atol=1e-13)
        np.testing.assert_allclose(cache["layers"][l]["c"][-1], cT[l].detach().numpy(), atol=1e-13)
        np.testing.assert_allclose(g[f"W{l}"], getattr(lstm, f"weight_ih_l{l}").grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(g[f"U{l}"], getattr(lstm, f"weight_hh_l{l}").grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(g[f"b{l}"], getattr(lstm, f"bias_ih_l{l}").grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(g["w_head"], wh.grad.numpy(), atol=1e-12)


# ---------------------------------------------------------------- library special case
@pytest.mark.parametrize("L", [1, 2, 3])
def test_matches_torch_lstm_autograd(L):
    rng = np.random.default_rng(7 + L)
    T, B, I, H = 9, 5, 6, 7
    p, shapes = _rand_params(rng, L, I, H, scale=0.4)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 1, T, B)
    loss, cache = orc.forward(p, L, x, y, orc.HEAD_STEP_BCE)
    g = orc.backward(p, L, cache, 1.0)

    lstm = torch.nn.LSTM(I, H, num_layers=L, bias=True).double()
    with torch.no_grad():
        for l in range(L):
            getattr(lstm, f"weight_ih_l{l}").copy_(torch.from_numpy(p[f"W{l}"]))
            getattr(lstm, f"weight_hh_l{l}").copy_(torch.from_numpy(p[f"U{l}"]))
            getattr(lstm, f"bias_ih_l{l}").copy_(torch.from_numpy(p[f"b{l}"]))
            getattr(lstm, f"bias_hh_l{l}").zero_()
    wh = torch.from_numpy(p["w_head"]).requires_grad_()
    bh = torch.from_numpy(p["b_head"]).requires_grad_()
    out, (hT, cT) = lstm(torch.from_numpy(x))
    z = out @ wh + bh
    tl = torch.nn.functional.binary_cross_entropy_with_logits(z, torch.from_numpy(y[..., 0]))
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    np.testing.assert_allclose(cache["layers"][-1]["h"][1:], out.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(cache["layers"][-1]["c"][-1], cT[-1].detach().numpy(), atol=1e-13)
    for l in range(L):
        np.testing.assert_allclose(g[f"W{l}"], getattr(lstm, f"weight_ih_l{l}").grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(g[f"U{l}"], getattr(lstm, f"weight_hh_l{l}").grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(g[f"b{l}"], getattr(lstm, f"bias_ih_l{l}").grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(g["w_head"], wh.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(g["b_head"], bh.grad.numpy(), atol=1e-13)


def test_matches_torch_embedding_last_step_and_mse():
    rng = np.random.default_rng(21)
    T, B, H, V, E = 6, 4, 5, 9, 3
    p, shapes = _rand_params(rng, 1, 0, H, V, E)
    ids = rng.integers(0, V, (T, B)); ids[0, :] = 2
    y = _targets(rng, orc.HEAD_LAST_BCE, T, B)
    loss, cache = orc.forward(p, 1, ids, y, orc.HEAD_LAST_BCE)
    g = orc.backward(p, 1, cache, 4.0)
    tp = {k: torch.from_numpy(v.copy()).requires_grad_() for k, v in p.items()}
    xs = tp["E"][torch.from_numpy(ids)]
    h = torch.zeros(B, H, dtype=torch.float64); c = torch.zeros(B, H, dtype=torch.float64)
    for t in range(T):
        a = xs[t] @ tp["W0"].T + h @ tp["U0"].T + tp["b0"]
        i, f, gg, o = a.chunk(4, dim=1)
        c = torch.sigmoid(f) * c + torch.sigmoid(i) * torch.tanh(gg)
        h = torch.sigmoid(o) * torch.tanh(c)
    z = h @ tp["w_head"] + tp["b_head"]
    tl = torch.nn.functional.binary_cross_entropy_with_logits(z, torch.from_numpy(y[:, 0]))
    (4.0 * tl).backward()
    assert abs(loss - tl.item()) < 1e-12
    for k in p:
        np.testing.assert_allclose(g[k], tp[k].grad.numpy(), atol=1e-12, err_msg=k)
    # MSE head against torch's mse_loss
    x = rng.standard_normal((T, B, 4)); p2, _ = _rand_params(rng, 1, 4, H)
    y2 = rng.standard_normal((T, B, 1))
    l2, c2 = orc.forward(p2, 1, x, y2, orc.HEAD_STEP_MSE)
    lstm = torch.nn.LSTM(4, H).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(p2["W0"])); lstm.weight_hh_l0.copy_(torch.from_numpy(p2["U0"]))
        lstm.bias_ih_l0.copy_(torch.from_numpy(p2["b0"])); lstm.bias_hh_l0.zero_()
    out, _ = lstm(torch.from_numpy(x))
    z2 = out @ torch.from_numpy(p2["w_head"]) + p2["b_head"][0]
    assert abs(l2 - torch.nn.functional.mse_loss(z2, torch.from_numpy(y2[..., 0])).item()) < 1e-12


# ---------------------------------------------------------------- closed forms
def test_zero_weights_closed_form():
    L, T, B, I, H = 2, 5, 3, 4, 6
    shapes = orc.param_shapes(L, I, H)
    p = {n: np.zeros(s) for n, s in shapes}
    rng = np.random.default_rng(0)
    x = rng.standard_normal((T, B, I))
    y = _targets(rng, 1, T, B)
    loss, cache = orc.forward(p, L, x, y, orc.HEAD_STEP_BCE)
    assert abs(loss - math.log(2.0)) < 1e-15
    for lay in cache["layers"]:
        assert np.all(lay["i"] == 0.5) and np.all(lay["f"] == 0.5) and np.all(lay["o"] == 0.5)
        assert np.all(lay["g"] == 0.0) and np.all(lay["c"] == 0.0) and np.all(lay["h"] == 0.0)
    ym = rng.standard_normal((T, B, 1))
    loss, _ = orc.forward(p, L, x, ym, orc.HEAD_STEP_MSE)
    assert abs(loss - float(np.mean(ym ** 2))) < 1e-15
    # sigmoid(0) = 1/2 and tanh is odd
    assert orc.sigmoid(0.0) == 0.5
    a = rng.standard_normal(50) * 20
    np.testing.assert_allclose(orc.sigmoid(a) + orc.sigmoid(-a), 1.0, atol=1e-15)
    assert np.all(np.isfinite(orc.sigmoid(np.array([-800.0, 800.0]))))


def test_scalar_cell_by_hand():
    """H = 1, two steps, computed with the math module from the cell's definition."""
    w = dict(wi=0.3, wf=-0.2, wg=0.7, wo=0.5, ui=0.1, uf=0.4, ug=-0.6, uo=0.25,
             bi=0.05, bf=0.9, bg=-0.1, bo=0.2)
    p = {"W0": np.array([[w["wi"]], [w["wf"]], [w["wg"]], [w["wo"]]]),
         "U0": np.array([[w["ui"]], [w["uf"]], [w["ug"]], [w["uo"]]]),
         "b0": np.array([w["bi"], w["bf"], w["bg"], w["bo"]]),
         "w_head": np.array([1.5]), "b_head": np.array([-0.3])}
    xs = [0.8, -1.1]
    sg = lambda v: 1.0 / (1.0 + math.exp(-v))
    h = c = 0.0
    hs = []
    for xv in xs:
        i = sg(w["wi"] * xv + w["ui"] * h + w["bi"])
        f = sg(w["wf"] * xv + w["uf"] * h + w["bf"])
        g = math.tanh(w["wg"] * xv + w["ug"] * h + w["bg"])
        o = sg(w["wo"] * xv + w["uo"] * h + w["bo"])
        c = f * c + i * g
        h = o * math.tanh(c)
        hs.append(h)
    x = np.array(xs).reshape(2, 1, 1)
    y = np.array([1.0, 0.0]).reshape(2, 1, 1)
    loss, cache = orc.forward(p, 1, x, y, orc.HEAD_STEP_BCE)
    np.testing.assert_allclose(cache["layers"][0]["h"][1:, 0, 0], hs, rtol=0, atol=1e-15)
    z = [1.5 * hv - 0.3 for hv in hs]
    want = 0.5 * (-math.log(sg(z[0])) - math.log(1.0 - sg(z[1])))
    assert abs(loss - want) < 1e-14


def test_tanh_odd_symmetry():
    """Flipping the sign of the g-gate input rows, of the recurrent columns
    acting on the other gates, and of the head weight flips h and c and leaves
    the loss unchanged."""
    rng = np.random.default_rng(3)
    T, B, I, H = 6, 3, 4, 5
    p, _ = _rand_params(rng, 1, I, H)
    q = {k: v.copy() for k, v in p.items()}
    gs = slice(2 * H, 3 * H)
    q["W0"][gs] *= -1; q["b0"][gs] *= -1            # a_g -> -a_g from the input side
    q["U0"] *= -1; q["U0"][gs] *= -1                # h -> -h: i,f,o rows negate, g rows keep
    q["w_head"] *= -1
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 1, T, B)
    l1, c1 = orc.forward(p, 1, x, y, 1)
    l2, c2 = orc.forward(q, 1, x, y, 1)
    assert abs(l1 - l2) < 1e-15
    np.testing.assert_allclose(c1["layers"][0]["h"], -c2["layers"][0]["h"], atol=1e-15)
    np.testing.assert_allclose(c1["layers"][0]["c"], -c2["layers"][0]["c"], atol=1e-15)
    g1 = orc.backward(p, 1, c1, 1.0); g2 = orc.backward(q, 1, c2, 1.0)
    np.testing.assert_allclose(g1["w_head"], -g2["w_head"], atol=1e-15)
    np.testing.assert_allclose(g1["W0"][gs], -g2["W0"][gs], atol=1e-15)
    np.testing.assert_allclose(g1["W0"][:2 * H], g2["W0"][:2 * H], atol=1e-15)


# ---------------------------------------------------------------- invariants
def test_loss_scale_invariance():
    rng = np.random.default_rng(11)
    L, T, B, I, H = 2, 5, 3, 4, 4
    p, shapes = _rand_params(rng, L, I, H)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 1, T, B)
    _, cache = orc.forward(p, L, x, y, 1)
    g1 = orc.flatten(orc.backward(p, L, cache, 1.0), shapes)
    for S in (1024.0, 32768.0):        # powers of two: scaling commutes with rounding
        gS = orc.flatten(orc.backward(p, L, cache, S), shapes)
        assert np.array_equal(gS / S, g1)
    g10 = orc.flatten(orc.backward(p, L, cache, 10.0), shapes)   # the paper's alpha = 10
    np.testing.assert_allclose(g10 / 10.0, g1, rtol=1e-12, atol=1e-16)
    avg, inf = orc.grad_average(np.stack([g10, g10]), 10.0)
    np.testing.assert_allclose(avg, g1, rtol=1e-12, atol=1e-16)
    assert not inf


def test_worker_average_equals_big_batch():
    """N workers with batch B each give, after averaging, the gradient of one
    batch of N*B samples (effective batch = N * batch, Section 'Learning rate
    schedule')."""
    rng = np.random.default_rng(13)
    L, T, B, I, H, N = 2, 4, 3, 3, 4, 5
    p, shapes = _rand_params(rng, L, I, H)
    xs = [rng.standard_normal((T, B, I)) for _ in range(N)]
    ys = [_targets(rng, 3, T, B) for _ in range(N)]
    S = 64.0
    wg = []
    for x, y in zip(xs, ys):
        _, c = orc.forward(p, L, x, y, 3)
        wg.append(orc.flatten(orc.backward(p, L, c, S), shapes))
    avg, inf = orc.grad_average(np.stack(wg), S)
    _, c = orc.forward(p, L, np.concatenate(xs, 1), np.concatenate(ys, 1), 3)
    big = orc.flatten(orc.backward(p, L, c, 1.0), shapes)
    np.testing.assert_allclose(avg, big, rtol=1e-12, atol=1e-15)
    assert not inf
    wg[2][7] = np.inf
    assert orc.grad_average(np.stack(wg), S)[1]
    wg[2][7] = np.nan
    assert orc.grad_average(np.stack(wg), S)[1]


def test_batch_permutation_and_independence():
    rng = np.random.default_rng(17)
    L, T, B, I, H = 2, 5, 4, 3, 4
    p, _ = _rand_params(rng, L, I, H)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 1, T, B)
    _, c1 = orc.forward(p, L, x, y, 1)
    perm = np.array([2, 0, 3, 1])
    _, c2 = orc.forward(p, L, x[:, perm], y[:, perm], 1)
    np.testing.assert_allclose(c1["layers"][1]["h"][:, perm], c2["layers"][1]["h"], atol=1e-15)
    x2 = x.copy(); x2[:, 1:] = rng.standard_normal((T, B - 1, I))
    _, c3 = orc.forward(p, L, x2, y, 1)
    np.testing.assert_allclose(c1["layers"][1]["h"][:, 0], c3["layers"][1]["h"][:, 0], atol=1e-15)


def test_chunked_sequence_consistency():
    rng = np.random.default_rng(19)
    L, T, B, I, H = 2, 8, 3, 3, 4
    p, _ = _rand_params(rng, L, I, H)
    x = rng.standard_normal((T, B, I)); y = _targets(rng, 1, T, B)
    _, full = orc.forward(p, L, x, y, 1)
    _, a = orc.forward(p, L, x[:4], y[:4], 1)
    h0 = np.stack([a["layers"][l]["h"][-1] for l in range(L)])
    c0 = np.stack([a["layers"][l]["c"][-1] for l in range(L)])
    _, b = orc.forward(p, L, x[4:], y[4:], 1, h0, c0)
    np.testing.assert_allclose(full["layers"][1]["h"][5:], b["layers"][1]["h"][1:], atol=1e-15)
    np.testing.assert_allclose(full["z"][4:], b["z"], atol=1e-15)


# ---------------------------------------------------------------- update + schedule
def test_sgd_momentum_closed_forms():
    rng = np.random.default_rng(23)
    W0 = rng.standard_normal(10); g1 = rng.standard_normal(10); g2 = rng.standard_normal(10)
    W1, H1 = orc.sgd_momentum_update(W0, np.zeros(10), g1, 0.01, 0.0)
    np.testing.assert_allclose(W1, W0 - 0.01 * g1, rtol=0, atol=1e-16)
    m, l1, l2 = 0.9, 0.01, 0.004
    W1, H1 = orc.sgd_momentum_update(W0, np.zeros(10), g1, l1, m)
    W2, H2 = orc.sgd_momentum_update(W1, H1, g2, l2, m)
    np.testing.assert_allclose(H2, -m * l1 * g1 - l2 * g2, rtol=1e-14)
    np.testing.assert_allclose(W2, W0 - l1 * g1 + H2, rtol=1e-14)


def test_sgd_momentum_equals_torch_for_constant_lr():
    rng = np.random.default_rng(29)
    W = rng.standard_normal(16); Hb = np.zeros(16)
    tw = torch.from_numpy(W.copy()).requires_grad_()
    opt = torch.optim.SGD([tw], lr=0.05, momentum=0.8)
    for _ in range(4):
        g = rng.standard_normal(16)
        W, Hb = orc.sgd_momentum_update(W, Hb, g, 0.05, 0.8)
        tw.grad = torch.from_numpy(g.copy()); opt.step()
    np.testing.assert_allclose(W, tw.detach().numpy(), rtol=1e-13)


def test_adam_equals_torch():
    rng = np.random.default_rng(31)
    W = rng.standard_normal(16); m = np.zeros(16); v = np.zeros(16)
    tw = torch.from_numpy(W.copy()).requires_grad_()
    opt = torch.optim.Adam([tw], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    for k in range(1, 5):
        g = rng.standard_normal(16)
        W, m, v = orc.adam_update(W, m, v, g, 0.01, k)
        tw.grad = torch.from_numpy(g.copy()); opt.step()
    np.testing.assert_allclose(W, tw.detach().numpy(), rtol=1e-12)


def test_lr_schedule_closed_forms():
    gold = json.load(open(GOLDEN))
    half = gold["lr_halved_at_N_equals_n"]["value"]
    cap = gold["eff_lr_max"]["value"]
    # N = n halves the base rate (Eq. 4)
    assert orc.lr_schedule(0.001, 8, 8, 1e9, 0, 1.0, 0) == pytest.approx(0.001 * half, rel=1e-15)
    # few workers: rate tends to lr0
    assert orc.lr_schedule(0.001, 1e-9, 8, 1e9, 0, 1.0, 0) == pytest.approx(0.001, rel=1e-8)
    # clip: lr0 = 0.05, N = n = 8 -> 0.025, times 8 = 0.2 > 0.1 -> 0.1 / 8
    assert orc.lr_schedule(0.05, 8, 8, cap, 0, 1.0, 0) == pytest.approx(cap / 8, rel=1e-15)
    # no clip when the product stays below the cap
    assert orc.lr_schedule(0.001, 64, 64, cap, 0, 1.0, 0) == pytest.approx(0.0005, rel=1e-15)
    # Eq. 3
    for i in range(6):
        assert orc.lr_schedule(0.02, 1, 1e12, 1e9, 0, 0.9, i) == pytest.approx(0.02 * 0.9 ** i, rel=1e-12)
    # warm-up (benchmark config 5): monotone, reaches the base rate at k = W-1, then decays
    vals = [orc.lr_schedule(1e-3, 64, 64, cap, 5, 0.97, k) for k in range(8)]
    assert all(b > a for a, b in zip(vals[:4], vals[1:5]))
    assert vals[4] == pytest.approx(5e-4, rel=1e-15)
    assert vals[5] == pytest.approx(5e-4 * 0.97, rel=1e-14)
    assert vals[7] == pytest.approx(5e-4 * 0.97 ** 3, rel=1e-14)


def test_loss_scale_policy():
    assert orc.loss_scale_policy(1024.0, 3, True, False) == (1024.0, 3)
    assert orc.loss_scale_policy(32768.0, 3, True, True) == (16384.0, 0)
    assert orc.loss_scale_policy(32768.0, 3, False, True) == (32768.0, 4)
    assert orc.loss_scale_policy(32768.0, 1999, False, True) == (65536.0, 0)


# ---------------------------------------------------------------- storage formats
def test_half_precision_facts_from_paper():
    gold = json.load(open(GOLDEN))
    mx = gold["fp16_max_finite"]["value"]
    assert orc.FP16_MAX == mx
    assert orc.round_fp16(mx) == mx
    assert np.isinf(orc.round_fp16(mx + 16.0))          # halfway to the next step rounds to even = inf
    assert orc.round_fp16(mx + 15.9) == mx
    mn = 2.0 ** -14
    assert abs(mn - gold["fp16_min_normal_approx"]["value"]) < 2e-6
    mb = gold["fp16_mantissa_bits"]["value"]
    assert orc.round_fp16(1.0 + 2.0 ** -mb) == 1.0 + 2.0 ** -mb
    assert orc.round_fp16(1.0 + 2.0 ** -(mb + 1)) == 1.0          # tie -> even
    assert orc.round_fp16(1.0 + 3 * 2.0 ** -(mb + 1)) == 1.0 + 2.0 ** -(mb - 1)


def test_bf16_rounding_matches_library_cast():
    rng = np.random.default_rng(37)
    v = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-20, 20, 4000),
                        [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.3895314e38, np.inf, -np.inf]])
    want = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_bf16(v)
    assert np.array_equal(got, want)
    v16 = torch.from_numpy(v.astype(np.float32)).to(torch.float16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_fp16(v.astype(np.float32)), v16)


def test_param_count_formula_and_table1():
    assert orc.param_count(1, 14, 32) == 4 * 32 * (14 + 32 + 1) + 33
    assert orc.param_count(3, 512, 2048) == 88_107_009
    assert orc.param_count(1, 0, 256, 20000, 128) == 2_954_497
    gold = json.load(open(GOLDEN))
    per_layer = orc.param_count(2, 200, 200) - orc.param_count(1, 200, 200)
    assert per_layer == 4 * 200 * (200 + 200 + 1)
    for row in gold["table1"]["rows"]:
        printed = row["n_par"] / row["n_layers"]
        assert abs(printed - per_layer) / per_layer < 0.05, row
    # flatten/unflatten round trip keeps order
    shapes = orc.param_shapes(2, 3, 2)
    flat = np.arange(orc.param_count(2, 3, 2), dtype=np.float64)
    t = orc.unflatten(flat, shapes)
    assert t["W0"][1, 2] == 5 and t["b_head"][0] == flat[-1]
    assert np.array_equal(orc.flatten(t, shapes), flat)


def test_training_step_matches_pieces():
    rng = np.random.default_rng(41)
    L, T, B, I, H = 1, 4, 2, 3, 3
    shapes = orc.param_shapes(L, I, H)
    flat = rng.uniform(-0.5, 0.5, orc.param_count(L, I, H))
    batches = [(rng.standard_normal((T, B, I)), _targets(rng, 1, T, B)) for _ in range(3)]
    out = orc.training_step(flat, shapes, L, batches, 1, 128.0, 0.01, 0.9)
    assert not out["found_inf"]
    np.testing.assert_allclose(out["W"], flat - 0.01 * out["avg_grad"], rtol=1e-14)
    np.testing.assert_allclose(out["avg_grad"], out["worker_grads"].mean(0) / 128.0, rtol=1e-13)


# ---------------------------------------------------------------- fault-tolerant average
def test_partial_average_by_hand_and_invariants():
    """Averaging only the workers that reported (Section "Distributed computing
    framework", closing paragraph)."""
    # worked by hand: workers 0 and 1 present, scale 2 -> ((2+6)/2/2, (4+8)/2/2)
    g = np.array([[2.0, 4.0], [6.0, 8.0], [100.0, -100.0]])
    avg, bad, n = orc.grad_average_partial(g, 2.0, [1, 1, 0])
    assert n == 2 and not bad
    np.testing.assert_array_equal(avg, [2.0, 3.0])
    # one participant: its own gradient over the scale
    avg, bad, n = orc.grad_average_partial(g, 4.0, [0, 0, 1])
    assert n == 1 and not bad
    np.testing.assert_array_equal(avg, [25.0, -25.0])
    # nobody: zero, no overflow flag
    avg, bad, n = orc.grad_average_partial(g, 4.0, [0, 0, 0])
    assert n == 0 and not bad and not avg.any()

    rng = np.random.default_rng(11)
    N, P, S = 9, 37, 128.0
    g = rng.normal(size=(N, P))
    mask = np.array([1, 0, 1, 1, 0, 1, 1, 1, 0])
    avg, bad, n = orc.grad_average_partial(g, S, mask)
    # library mean over the selected rows
    np.testing.assert_allclose(avg, g[mask.astype(bool)].mean(axis=0) / S, rtol=1e-14, atol=0)
    assert n == 6 and not bad
    # everybody present: the lock-step average
    full, bad_full = orc.grad_average(g, S)
    part, bad_part, n_all = orc.grad_average_partial(g, S, np.ones(N, dtype=int))
    np.testing.assert_allclose(part, full, rtol=1e-15, atol=0)
    assert n_all == N and bad_part == bad_full
    # what an absent worker holds is irrelevant, Inf and NaN included
    g2 = g.copy()
    g2[1] = np.inf
    g2[4] = np.nan
    g2[8] = -1e30
    avg2, bad2, _ = orc.grad_average_partial(g2, S, mask)
    np.testing.assert_array_equal(avg2, avg)
    assert not bad2
    # ... and an Inf in a present worker is reported
    g3 = g.copy()
    g3[3, 5] = np.inf
    assert orc.grad_average_partial(g3, S, mask)[1]
    # order of the workers does not matter beyond rounding
    perm = rng.permutation(N)
    avg_p, _, _ = orc.grad_average_partial(g[perm], S, mask[perm])
    np.testing.assert_allclose(avg_p, avg, rtol=1e-13, atol=1e-18)


# ---------------------------------------------------------------- the paper's own head (Fig. 2, Eq. 6)
def _fc_params(rng, L, I, H, F, scale=0.5):
    shapes = orc.param_shapes(L, I, H, 0, 0, F)
    return {n: rng.uniform(-scale, scale, s) for n, s in shapes}, shapes


def _pm_targets(rng, T, B):
    return np.where(rng.random((T, B, 1)) < 0.4, 1.0, -1.0)


def test_fc_hinge_head_matches_central_differences():
    """ReLU layer per temporal slice + one output + hinge loss (Fig. 2, Eq. 6).  The loss is
    piecewise linear in the head's output; the seed avoids samples within the difference
    step of a kink, which the test checks before differencing."""
    rng = np.random.default_rng(404)
    L, T, B, I, H, F = 2, 4, 3, 5, 4, 6
    p, shapes = _fc_params(rng, L, I, H, F)
    x = rng.standard_normal((T, B, I)); y = _pm_targets(rng, T, B)
    S = 10.0                                                 # the paper's static multiplier
    loss, cache = orc.forward(p, L, x, y, orc.HEAD_FC_HINGE)
    assert np.abs(cache["fc_pre"]).min() > 1e-4 and np.abs(1.0 - y[..., 0] * cache["z"]).min() > 1e-4
    assert (cache["fc_pre"] > 0).any() and (cache["fc_pre"] < 0).any()
    assert ((1.0 - y[..., 0] * cache["z"]) > 0).any()
    g = orc.backward(p, L, cache, S)
    eps = 1e-6
    for name, _ in shapes:
        flat = p[name].reshape(-1)
        for k in rng.choice(flat.size, size=min(flat.size, 10), replace=False):
            old = flat[k]
            flat[k] = old + eps; lp, _ = orc.forward(p, L, x, y, orc.HEAD_FC_HINGE)
            flat[k] = old - eps; lm, _ = orc.forward(p, L, x, y, orc.HEAD_FC_HINGE)
            flat[k] = old
            fd = S * (lp - lm) / (2 * eps)
            an = g[name].reshape(-1)[k]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 2e-8, (name, k, fd, an)


def test_fc_hinge_head_matches_torch_autograd():
    rng = np.random.default_rng(405)
    L, T, B, I, H, F = 1, 6, 4, 3, 5, 7
    p, shapes = _fc_params(rng, L, I, H, F, scale=0.6)
    x = rng.standard_normal((T, B, I)); y = _pm_targets(rng, T, B)
    loss, cache = orc.forward(p, L, x, y, orc.HEAD_FC_HINGE)
    g = orc.backward(p, L, cache, 1.0)
    lstm = torch.nn.LSTM(I, H, num_layers=1, bias=True).double()
    fc = torch.nn.Linear(H, F).double(); out = torch.nn.Linear(F, 1).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(p["W0"])); lstm.weight_hh_l0.copy_(torch.from_numpy(p["U0"]))
        lstm.bias_ih_l0.copy_(torch.from_numpy(p["b0"])); lstm.bias_hh_l0.zero_()
        fc.weight.copy_(torch.from_numpy(p["W_fc"])); fc.bias.copy_(torch.from_numpy(p["b_fc"]))
        out.weight.copy_(torch.from_numpy(p["w_head"][None, :])); out.bias.copy_(torch.from_numpy(p["b_head"]))
    hseq, _ = lstm(torch.from_numpy(x))
    z = out(torch.relu(fc(hseq)))[..., 0]
    tl = torch.clamp(1.0 - torch.from_numpy(y[..., 0]) * z, min=0.0).mean()
    tl.backward()
    assert abs(loss - tl.item()) < 1e-13
    np.testing.assert_allclose(g["W_fc"], fc.weight.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(g["b_fc"], fc.bias.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(g["w_head"], out.weight.grad.numpy()[0], atol=1e-14)
    np.testing.assert_allclose(g["b_head"], out.bias.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(g["W0"], lstm.weight_ih_l0.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(g["U0"], lstm.weight_hh_l0.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(g["b0"], lstm.bias_ih_l0.grad.numpy(), atol=1e-14)


def test_fc_hinge_head_closed_forms():
    rng = np.random.default_rng(406)
    L, T, B, I, H, F = 1, 3, 2, 2, 3, 4
    p, shapes = _fc_params(rng, L, I, H, F)
    x = rng.standard_normal((T, B, I)); y = _pm_targets(rng, T, B)
    # zero output weights: y = 0 everywhere, loss = max(0, 1 - 0) = 1, and d loss / d b_head = -mean(t)
    p0 = {k: v.copy() for k, v in p.items()}
    p0["w_head"][:] = 0.0; p0["b_head"][:] = 0.0
    loss, cache = orc.forward(p0, L, x, y, orc.HEAD_FC_HINGE)
    assert loss == 1.0
    g = orc.backward(p0, L, cache, 1.0)
    np.testing.assert_allclose(g["b_head"][0], -y.mean(), rtol=1e-15)
    assert not g["W_fc"].any() and not g["W0"].any()      # nothing flows below a zero output weight
    # large correct margin: every sample satisfied, loss and every gradient exactly zero
    p1 = {k: v.copy() for k, v in p.items()}
    p1["w_head"][:] = 0.0
    yc = np.ones((T, B, 1)); p1["b_head"][:] = 5.0
    loss, cache = orc.forward(p1, L, x, yc, orc.HEAD_FC_HINGE)
    assert loss == 0.0
    assert all(not v.any() for v in orc.backward(p1, L, cache, 10.0).values())
    # one unit, one sample, by hand: h = o*tanh(c); a = relu(w h + b); y = v a + c0
    pp = {"W0": np.array([[0.5], [0.0], [1.0], [2.0]]), "U0": np.zeros((4, 1)), "b0": np.zeros(4),
          "W_fc": np.array([[2.0], [-1.0]]), "b_fc": np.array([0.1, 0.0]), "w_head": np.array([3.0, 7.0]), "b_head": np.array([-0.2])}
    xx = np.array([[[1.0]]]); tt = np.array([[[-1.0]]])  # wrong side: margin 1 + y > 0
    i = 1 / (1 + math.exp(-0.5)); gg = math.tanh(1.0); o = 1 / (1 + math.exp(-2.0))
    h = o * math.tanh(i * gg)
    a1 = 2.0 * h + 0.1                                    # positive; the second unit (-h) is cut by the ReLU
    yv = 3.0 * a1 - 0.2
    loss, cache = orc.forward(pp, 1, xx, tt, orc.HEAD_FC_HINGE)
    assert abs(loss - (1.0 + yv)) < 1e-15 and yv > 0
    g = orc.backward(pp, 1, cache, 10.0)
    np.testing.assert_allclose(g["w_head"], [10.0 * a1, 0.0], rtol=1e-14)
    np.testing.assert_allclose(g["b_head"], [10.0], rtol=1e-14)
    np.testing.assert_allclose(g["b_fc"], [30.0, 0.0], rtol=1e-14)
    np.testing.assert_allclose(g["W_fc"][:, 0], [30.0 * h, 0.0], rtol=1e-14)


def test_fc_head_parameter_count():
    # Fig. 2: 2 x LSTM(200) on 9 features, FC(200) + ReLU, 1 output
    n = orc.param_count(2, 9, 200, 0, 0, 200)
    assert n == 4 * 200 * (9 + 200) + 800 + 4 * 200 * 400 + 800 + 200 * 200 + 200 + 200 + 1


# ---------------------------------------------------------------- the intermediates the rounding bound is built from
@pytest.mark.parametrize("head,vocab", [(1, 0), (3, 0), (2, 7), (4, 0)])
def test_trace_terms_add_up_to_the_gradients(head, vocab):
    """backward(trace=...) hands out da per layer; the weight gradients are its sums over the T*B rows
    (dW = da^T x, dU = da^T h_prev, db = sum da), and the sums of absolute terms the parity tests derive
    their rounding bound from can never be smaller than the gradient itself."""
    import workloads as wl
    from tests import parity_util as pu
    rng = np.random.default_rng(90 + head)
    L, T, B, I, H, F = 2, 4, 3, 5, 4, 3
    shapes = orc.param_shapes(L, I, H, vocab, 6 if vocab else 0, F if head == 4 else 0)
    p = {n: rng.uniform(-0.5, 0.5, s) for n, s in shapes}
    x = rng.integers(0, vocab, (T, B)) if vocab else rng.standard_normal((T, B, I))
    y = np.where(rng.random((T, B, 1)) < 0.5, 1.0, -1.0) if head == 4 else _targets(rng, head, T, B)
    _, cache = orc.forward(p, L, x, y, head)
    trace = {}
    g = orc.backward(p, L, cache, 3.0, trace)
    g_plain = orc.backward(p, L, cache, 3.0)
    for k in g:
        np.testing.assert_array_equal(g[k], g_plain[k])         # tracing changes nothing
    for l in range(L):
        da = trace[f"da{l}"].reshape(T * B, 4 * H)
        lay = cache["layers"][l]
        np.testing.assert_allclose(da.T @ lay["inp"].reshape(T * B, -1), g[f"W{l}"], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(da.T @ lay["h"][:-1].reshape(T * B, -1), g[f"U{l}"], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(da.sum(axis=0), g[f"b{l}"], rtol=1e-12, atol=1e-14)
    w = wl.Workload("t", L, I, H, T, B, "bf16", head, vocab=vocab, embed_dim=6 if vocab else 0, fc_units=F if head == 4 else 0)
    A, X = pu.term_magnitudes(w, p, cache, trace)
    for name, _ in shapes:
        assert A[name].shape == g[name].shape
        assert np.all(A[name] >= np.abs(g[name]) - 1e-12), name
    bound = pu.rounding_bound(w, orc.flatten(A, shapes), orc.flatten({n: X.get(n, np.zeros(s)) for n, s in shapes}, shapes), 3.0, shapes)
    assert bound.shape == (sum(int(np.prod(s)) for _, s in shapes),) and np.all(bound >= 0)
