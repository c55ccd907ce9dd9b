"""Pins of the oracle's multi-window SGD driver (CPU only).

The paper describes repeating a compiled training function N times inside the runtime and
returning only the last result (its section on calling a function object repeatedly) and
names no update rule; plain stochastic gradient descent on consecutive truncated windows
with the state carried is the reading used.  The driver is pinned by: the per-window
functions (themselves pinned by finite differences) for a single step; a learning rate of
zero; the zero-weight closed form of the first update; and torch's SGD optimiser run on a
float64 autograd model written out with torch ops.
"""
import math

import numpy as np
import pytest

import oracle
import rnn_inputs as ri

PNAMES = ("Wx", "Wh", "b", "V", "c")


def small_stream(windows=5, seed=77, **kw):
    args = dict(in_dim=30, hidden=7, out_dim=30, seq_len=4, batch=1, windows=windows,
                wdist=("normal", 0.4), bias_std=0.2, tokens="zipf", seed=seed)
    args.update(kw)
    return ri.make_case(**args)


def test_one_window_is_one_gradient_step():
    p = small_stream(windows=1, with_h0=True)
    ids = ri.stream_ids(p)
    r = oracle.train_stream(p, ids, 1, 0.3, h0=p["h0"])
    g = oracle.fwd_bptt(p, h0=p["h0"])
    assert abs(r["losses"][0] - g["loss"]) < 1e-14
    for k in PNAMES:
        np.testing.assert_allclose(r[k], np.asarray(p[k], dtype=np.float64) - 0.3 * g["d" + k],
                                   rtol=0, atol=1e-15)
    np.testing.assert_array_equal(r["h_last"], g["h_all"][-1])
    # a token that does not occur keeps its input vector, bit for bit
    unseen = sorted(set(range(p["in_dim"])) - set(p["x"].reshape(-1).tolist()))
    np.testing.assert_array_equal(r["Wx"][unseen], np.asarray(p["Wx"], dtype=np.float64)[unseen])


def test_zero_learning_rate_only_carries_the_state():
    p = small_stream(windows=6)
    ids = ri.stream_ids(p)
    r = oracle.train_stream(p, ids, 6, 0.0)
    for k in PNAMES:
        np.testing.assert_array_equal(r[k], np.asarray(p[k], dtype=np.float64))
    h = None
    for w in range(6):
        pw = ri.window(p, w)
        h_all = oracle.forward(pw, h)
        assert abs(r["losses"][w] - oracle.loss(pw, h_all)) < 1e-14   # thread-order rounding
        h = h_all[-1]
    np.testing.assert_array_equal(r["h_last"], h)


def test_first_update_from_zero_weights_closed_form():
    # all parameters zero: h = 1/2, z = 0, loss = ln NV; only c and V move, by
    # dc[k] = 1/NV - count(y = k)/N and dV[i,k] = dc[k]/2
    p = small_stream(windows=1)
    for k in PNAMES:
        p[k] = np.zeros_like(p[k])
    NV, N, lr = p["out_dim"], p["seq_len"], 0.7
    r = oracle.train_stream(p, ri.stream_ids(p), 1, lr)
    assert abs(r["losses"][0] - math.log(NV)) < 1e-14
    counts = np.bincount(p["y"].reshape(-1), minlength=NV)
    dc = 1.0 / NV - counts / N
    np.testing.assert_allclose(r["c"], -lr * dc, atol=1e-15)
    np.testing.assert_allclose(r["V"], np.tile(-lr * 0.5 * dc, (p["hidden"], 1)), atol=1e-15)
    for k in ("Wx", "Wh", "b"):
        assert not r[k].any()


@pytest.mark.parametrize("act", [ri.ACT_SIGMOID, ri.ACT_TANH])
def test_against_torch_sgd_optimiser(act):
    import torch
    torch.set_num_threads(2)
    W, lr = 7, 0.25
    p = small_stream(windows=W, seed=78, act=act, with_h0=True, batch=2)
    ids = ri.stream_ids(p)
    T, O = p["seq_len"], p["out_dim"]
    tt = {k: torch.tensor(np.asarray(p[k], dtype=np.float64), requires_grad=True) for k in PNAMES}
    opt = torch.optim.SGD(list(tt.values()), lr=lr)
    h = torch.tensor(np.asarray(p["h0"], dtype=np.float64))
    losses = []
    for w in range(W):
        x = torch.tensor(ids[w * T:w * T + T], dtype=torch.long)
        y = torch.tensor(ids[w * T + 1:w * T + T + 1], dtype=torch.long)
        hs = []
        for t in range(T):
            a = tt["Wx"][x[t]] + h @ tt["Wh"].T + tt["b"]
            h = torch.sigmoid(a) if act == ri.ACT_SIGMOID else torch.tanh(a)
            hs.append(h)
        Z = torch.stack(hs) @ tt["V"] + tt["c"]
        L = torch.nn.functional.cross_entropy(Z.reshape(-1, O), y.reshape(-1))
        opt.zero_grad()
        L.backward()
        opt.step()
        losses.append(L.item())
        h = h.detach()          # truncation: no gradient flows into earlier windows
    r = oracle.train_stream(p, ids, W, lr, h0=p["h0"])
    np.testing.assert_allclose(r["losses"], losses, rtol=0, atol=1e-13)
    for k in PNAMES:
        np.testing.assert_allclose(r[k], tt[k].detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(r["h_last"], h.numpy(), rtol=0, atol=1e-14)


def test_repeated_pattern_is_learned():
    # a periodic stream is predictable: the loss must fall well below ln NV
    p = small_stream(windows=400, seed=79)
    T = p["seq_len"]
    ids = np.tile(np.array([3, 1, 4, 1, 5, 9, 2, 6], dtype=np.int32), 400 * T // 8 + 1)[:400 * T + 1]
    r = oracle.train_stream(p, ids.reshape(-1, 1), 400, 0.5)
    assert r["losses"][:5].mean() > 2.0
    assert r["losses"][-20:].mean() < 0.5 * r["losses"][:5].mean()
    assert np.all(np.isfinite(r["losses"]))
