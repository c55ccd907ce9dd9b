"""Pins of the CPU oracle against things other than itself (CPU only).

The paper prints no worked example and no equations for the recurrent benchmark
(its recurrent-network benchmark section only names "a simple recurrent network",
batch size 1, vocabulary-sized input and output layers; its Scan section names
backpropagation through time).  So every pin is mathematical: finite differences,
closed forms, invariants, special cases that reduce to a separately written textbook
routine, and a float64 autograd cross-check.
"""
import math
import os

import numpy as np
import pytest

import oracle
import rnn_inputs as ri

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def as64(case):
    p = dict(case)
    for k in ("Wx", "Wh", "b", "V", "c", "X", "Y", "h0", "dh_last"):
        if p.get(k) is not None:
            p[k] = np.array(p[k], dtype=np.float64)
    return p


def total_objective(p, h0=None, dh_last=None):
    """Window loss plus <dh_last, h_{T-1}>: the scalar whose gradient bptt() returns."""
    h_all = oracle.forward(p, h0)
    L = oracle.loss(p, h_all)
    if dh_last is not None:
        L += float(np.sum(dh_last * h_all[-1]))
    return L


def fd_check(p, names, h0=None, dh_last=None, eps=1e-5, rtol=1e-6):
    h_all = oracle.forward(p, h0)
    g = oracle.bptt(p, h_all, dh_last)
    for name in names:
        arr = h0 if name == "h0" else p[name]
        an = g["dh0"] if name == "h0" else g["d" + name]
        fd = np.zeros_like(arr)
        flat, fdf = arr.reshape(-1), fd.reshape(-1)
        for i in range(flat.size):
            old = flat[i]
            flat[i] = old + eps
            lp = total_objective(p, h0, dh_last)
            flat[i] = old - eps
            lm = total_objective(p, h0, dh_last)
            flat[i] = old
            fdf[i] = (lp - lm) / (2 * eps)
        err = np.max(np.abs(fd - an))
        scale = np.max(np.abs(an))
        assert err <= rtol * scale + 1e-10, (name, err, scale)


# ---- P1: central finite differences ------------------------------------------------
def test_fd_all_parameters_tiny_lm_config():
    """Every one of the 2384 parameters of the tiny LM configuration (vocab 64, hidden 16, T 32)."""
    p = as64(ri.make_config("C1"))
    assert sum(p[k].size for k in ("Wx", "Wh", "b", "V", "c")) == 2384
    oracle.set_num_threads(1)
    fd_check(p, ["Wx", "Wh", "b", "V", "c"])


def test_fd_tanh_mse_dense_with_state_and_incoming_gradient():
    p = as64(ri.make_case(3, 4, 3, 5, 2, input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH,
                          loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.5), bias_std=0.3,
                          with_h0=True, with_dh_last=True, seed=7))
    fd_check(p, ["Wx", "Wh", "b", "V", "c", "h0"], h0=p["h0"], dh_last=p["dh_last"])


def test_fd_sigmoid_ce_batched_with_state_and_incoming_gradient():
    p = as64(ri.make_case(7, 5, 7, 4, 3, tokens="uniform", wdist=("normal", 0.7), bias_std=0.4,
                          with_h0=True, with_dh_last=True, seed=11))
    fd_check(p, ["Wx", "Wh", "b", "V", "c", "h0"], h0=p["h0"], dh_last=p["dh_last"])


def test_fd_dense_input_ce_and_token_input_mse():
    p = as64(ri.make_case(3, 4, 5, 3, 2, input_kind=ri.INPUT_DENSE, act=ri.ACT_SIGMOID,
                          loss_kind=ri.LOSS_SOFTMAX_CE, wdist=("normal", 0.5), bias_std=0.2, seed=3))
    fd_check(p, ["Wx", "Wh", "b", "V", "c"])
    p = as64(ri.make_case(6, 4, 3, 3, 2, input_kind=ri.INPUT_TOKENS, act=ri.ACT_TANH,
                          loss_kind=ri.LOSS_LINEAR_MSE, tokens="uniform", wdist=("normal", 0.5),
                          bias_std=0.2, seed=4))
    fd_check(p, ["Wx", "Wh", "b", "V", "c"])


# ---- P2: closed forms at zero weights ----------------------------------------------
def test_zero_weight_loss_is_log_vocab_and_gradients_closed_form():
    with open(os.path.join(GOLDEN, "zero_weight_loss.txt")) as f:
        golden = {int(a): float(b) for a, b in
                  (ln.split() for ln in f if ln.strip() and not ln.startswith("#"))}
    for nv, H, T, B in ((64, 16, 32, 1), (10000, 8, 6, 2)):
        p = as64(ri.make_case(nv, H, nv, T, B, tokens="zipf" if nv > 64 else "uniform", seed=5))
        for k in ("Wx", "Wh", "b", "V", "c"):
            p[k][...] = 0.0
        r = oracle.fwd_bptt(p)
        assert np.all(r["h_all"][1:] == 0.5)
        assert abs(r["loss"] - math.log(nv)) < 1e-12
        assert abs(r["loss"] - golden[nv]) < 1e-6
        N = T * B
        counts = np.bincount(p["y"].reshape(-1), minlength=nv)
        dc = 1.0 / nv - counts / N
        np.testing.assert_allclose(r["dc"], dc, atol=1e-15)
        np.testing.assert_allclose(r["dV"], 0.5 * np.broadcast_to(dc, (H, nv)), atol=1e-15)
        assert np.all(r["dWx"] == 0) and np.all(r["dWh"] == 0) and np.all(r["db"] == 0)
        assert np.all(r["dh0"] == 0)


def test_zero_weight_tanh_mse_closed_form():
    p = as64(ri.make_case(4, 6, 4, 5, 3, input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH,
                          loss_kind=ri.LOSS_LINEAR_MSE, seed=9))
    for k in ("Wx", "Wh", "b", "V", "c"):
        p[k][...] = 0.0
    r = oracle.fwd_bptt(p)
    N, O = 15, 4
    assert np.all(r["h_all"] == 0.0)
    assert abs(r["loss"] - np.sum(p["Y"] ** 2) / (N * O)) < 1e-14
    np.testing.assert_allclose(r["dc"], -2.0 * p["Y"].reshape(N, O).sum(0) / (N * O), atol=1e-15)
    for k in ("dWx", "dWh", "db", "dV", "dh0"):
        assert np.all(r[k] == 0)


# ---- P3/P4/P5: invariants -------------------------------------------------------------
def test_softmax_rows_sum_to_one_and_column_sum_invariants():
    p = as64(ri.make_case(50, 12, 50, 9, 3, wdist=("normal", 0.8), bias_std=0.5, seed=21))
    h_all = oracle.forward(p)
    L, lse, Z = oracle.loss(p, h_all, want_lse=True, want_Z=True)
    np.testing.assert_allclose(np.exp(Z - lse[:, None]).sum(1), 1.0, atol=1e-12)
    # lse against the unshifted definition (values are small enough not to overflow)
    np.testing.assert_allclose(lse, np.log(np.exp(Z).sum(1)), atol=1e-12)
    g = oracle.bptt(p, h_all, want_internals=True)
    assert abs(g["dc"].sum()) < 1e-15
    assert np.max(np.abs(g["dV"].sum(1))) < 1e-15
    assert np.max(np.abs(g["dZ"].sum(1))) < 1e-16
    # scatter invariant: summing the per-token rows of dWx gives db; unseen rows are exactly 0
    np.testing.assert_allclose(g["dWx"].sum(0), g["db"], atol=1e-15)
    unseen = np.setdiff1d(np.arange(50), np.unique(p["x"]))
    assert unseen.size > 0 and np.all(g["dWx"][unseen] == 0.0)


def test_large_logits_do_not_overflow():
    p = as64(ri.make_case(9, 4, 9, 3, 1, tokens="uniform", seed=2))
    p["c"] = np.linspace(-900.0, 900.0, 9)
    L = oracle.loss(p, oracle.forward(p))
    assert np.isfinite(L)


# ---- P6/P7: no recurrence reduces to a one-hidden-layer softmax network ------------------
def mlp_softmax_grads(Wx, b, V, c, x, y, hprev_rows):
    """Textbook one-hidden-layer softmax classifier, mean CE over the rows; written
    independently of the oracle (numpy matrix form)."""
    N = x.size
    h = 1.0 / (1.0 + np.exp(-(Wx[x] + b)))
    Z = h @ V + c
    Z = Z - Z.max(1, keepdims=True)
    P = np.exp(Z)
    P /= P.sum(1, keepdims=True)
    loss = -np.mean(np.log(P[np.arange(N), y]))
    dZ = P.copy()
    dZ[np.arange(N), y] -= 1.0
    dZ /= N
    dV, dc = h.T @ dZ, dZ.sum(0)
    da = (dZ @ V.T) * h * (1 - h)
    dWx = np.zeros_like(Wx)
    np.add.at(dWx, x, da)
    return dict(loss=loss, dV=dV, dc=dc, db=da.sum(0), dWx=dWx, dWh=da.T @ hprev_rows, h=h)


def test_zero_recurrent_matrix_equals_independent_mlp_steps():
    p = as64(ri.make_case(30, 6, 30, 8, 2, wdist=("normal", 0.6), bias_std=0.3, with_h0=True, seed=33))
    p["Wh"][...] = 0.0
    r = oracle.fwd_bptt(p, h0=p["h0"])
    x, y = p["x"].reshape(-1), p["y"].reshape(-1)
    hprev = r["h_all"][:-1].reshape(-1, 6)
    m = mlp_softmax_grads(p["Wx"], p["b"], p["V"], p["c"], x, y, hprev)
    assert abs(r["loss"] - m["loss"]) < 1e-13
    for k in ("dV", "dc", "db", "dWx", "dWh"):
        np.testing.assert_allclose(r[k], m[k], atol=1e-14)
    assert np.all(r["dh0"] == 0.0)


def test_single_step_sequence():
    p = as64(ri.make_case(12, 5, 12, 1, 3, tokens="uniform", wdist=("normal", 0.6), bias_std=0.3,
                          with_h0=True, seed=34))
    r = oracle.fwd_bptt(p, h0=p["h0"])
    # T=1: a = Wx[x] + Wh h0 + b is an MLP whose bias is shifted per row by Wh h0
    x, y = p["x"].reshape(-1), p["y"].reshape(-1)
    shift = p["h0"] @ p["Wh"].T
    h = 1 / (1 + np.exp(-(p["Wx"][x] + p["b"] + shift)))
    np.testing.assert_allclose(r["h_all"][1], h, atol=1e-15)
    Z = h @ p["V"] + p["c"]
    P = np.exp(Z) / np.exp(Z).sum(1, keepdims=True)
    dZ = P.copy(); dZ[np.arange(3), y] -= 1; dZ /= 3
    delta = (dZ @ p["V"].T) * h * (1 - h)
    np.testing.assert_allclose(r["dWh"], delta.T @ p["h0"], atol=1e-15)
    np.testing.assert_allclose(r["dh0"], delta @ p["Wh"], atol=1e-15)
    np.testing.assert_allclose(r["db"], delta.sum(0), atol=1e-15)


# ---- P8: batch averaging ------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["lm", "dense"])
def test_batch_result_is_mean_of_single_sequence_results(kind):
    if kind == "lm":
        p = as64(ri.make_case(20, 7, 20, 6, 4, wdist=("normal", 0.5), bias_std=0.2, seed=41))
    else:
        p = as64(ri.make_case(5, 7, 5, 6, 4, input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH,
                              loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.5), bias_std=0.2, seed=42))
    full = oracle.fwd_bptt(p)
    acc = None
    for b in range(4):
        q = dict(p); q["batch"] = 1
        for k in ("x", "y", "X", "Y"):
            if k in p:
                q[k] = np.ascontiguousarray(p[k][:, b:b + 1])
        r = oracle.fwd_bptt(q)
        np.testing.assert_allclose(r["h_all"][:, 0], full["h_all"][:, b], atol=1e-15)
        if acc is None:
            acc = {k: np.zeros_like(np.asarray(r[k], dtype=np.float64)) for k in ("loss", "dWx", "dWh", "db", "dV", "dc")}
        for k in acc:
            acc[k] = acc[k] + np.asarray(r[k]) / 4.0
    for k in acc:
        np.testing.assert_allclose(full[k], acc[k], atol=1e-14)


# ---- P9: window chaining --------------------------------------------------------------------
def test_two_chained_windows_reproduce_full_sequence():
    p = as64(ri.make_case(15, 6, 15, 10, 2, wdist=("normal", 0.6), bias_std=0.2, with_h0=True, seed=51))
    full = oracle.fwd_bptt(p, h0=p["h0"])
    halves = []
    for w in range(2):
        q = dict(p); q["seq_len"] = 5
        q["x"], q["y"] = p["x"][5 * w:5 * w + 5], p["y"][5 * w:5 * w + 5]
        halves.append(q)
    h_a = oracle.forward(halves[0], p["h0"])
    h_b = oracle.forward(halves[1], h_a[-1])
    np.testing.assert_allclose(np.concatenate([h_a, h_b[1:]]), full["h_all"], atol=1e-15)
    # each half's loss is a mean over half the rows: full = (La + Lb)/2, so the incoming
    # gradient for the first half is dh0 of the second half, both weighted 1/2
    g_b = oracle.bptt(halves[1], h_b)
    g_a = oracle.bptt(halves[0], h_a, dh_last=g_b["dh0"])
    for k in ("dWx", "dWh", "db", "dV", "dc"):
        np.testing.assert_allclose(0.5 * (g_a[k] + g_b[k]), full[k], atol=1e-14)
    np.testing.assert_allclose(0.5 * g_a["dh0"], full["dh0"], atol=1e-15)
    La, Lb = oracle.loss(halves[0], h_a), oracle.loss(halves[1], h_b)
    assert abs(0.5 * (La + Lb) - full["loss"]) < 1e-14


# ---- P10: float64 autograd cross-check (library routine, test only) --------------------------
@pytest.mark.parametrize("kind", ["lm_sigmoid_ce", "dense_tanh_mse"])
def test_against_torch_cpu_autograd(kind):
    import torch
    torch.set_num_threads(2)
    if kind == "lm_sigmoid_ce":
        p = as64(ri.make_case(40, 9, 40, 7, 3, wdist=("normal", 0.5), bias_std=0.3,
                              with_h0=True, with_dh_last=True, seed=61))
    else:
        p = as64(ri.make_case(6, 9, 6, 7, 3, input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH,
                              loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.5), bias_std=0.3,
                              with_h0=True, with_dh_last=True, seed=62))
    tt = {k: torch.tensor(p[k], dtype=torch.float64, requires_grad=True)
          for k in ("Wx", "Wh", "b", "V", "c", "h0")}
    h = tt["h0"]
    hs = []
    for t in range(p["seq_len"]):
        if p["input_kind"] == 0:
            inp = tt["Wx"][torch.tensor(p["x"][t], dtype=torch.long)]
        else:
            inp = torch.tensor(p["X"][t]) @ tt["Wx"].T
        a = inp + h @ tt["Wh"].T + tt["b"]
        h = torch.sigmoid(a) if p["act"] == 0 else torch.tanh(a)
        hs.append(h)
    Hs = torch.stack(hs)
    Z = Hs @ tt["V"] + tt["c"]
    if p["loss_kind"] == 0:
        L = torch.nn.functional.cross_entropy(Z.reshape(-1, p["out_dim"]),
                                              torch.tensor(p["y"].reshape(-1), dtype=torch.long))
    else:
        L = torch.nn.functional.mse_loss(Z, torch.tensor(p["Y"]))
    (L + (torch.tensor(p["dh_last"]) * hs[-1]).sum()).backward()
    r = oracle.fwd_bptt(p, h0=p["h0"], dh_last=p["dh_last"])
    assert abs(r["loss"] - L.item()) < 1e-13
    np.testing.assert_allclose(r["h_all"][1:], Hs.detach().numpy(), atol=1e-14)
    for k in ("Wx", "Wh", "b", "V", "c"):
        np.testing.assert_allclose(r["d" + k], tt[k].grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(r["dh0"], tt["h0"].grad.numpy(), atol=1e-14)


# ---- P11: scalar case worked by hand ------------------------------------------------------------
def test_scalar_two_class_two_step_hand_derivation():
    """H=1, two classes, T=2, B=1, zero initial state.  With m_t = h_t (V1-V0) + (c1-c0) and
    s_t = +1 if y_t is class 1 else -1, the per-step loss is softplus(-s_t m_t) and the total
    is their mean; every derivative below is the chain rule done by hand."""
    sig = lambda u: 1.0 / (1.0 + math.exp(-u))
    wx = np.array([[0.3], [-0.7]]); wh = np.array([[0.9]]); b = np.array([0.2])
    V = np.array([[0.5, -1.1]]); c = np.array([0.1, -0.4])
    x = np.array([[1], [0]], dtype=np.int32); y = np.array([[0], [1]], dtype=np.int32)
    p = dict(in_dim=2, hidden=1, out_dim=2, seq_len=2, batch=1, input_kind=0, act=0, loss_kind=0,
             Wx=wx, Wh=wh, b=b, V=V, c=c, x=x, y=y)
    r = oracle.fwd_bptt(p)
    h0 = sig(wx[1, 0] + b[0])
    h1 = sig(wx[0, 0] + wh[0, 0] * h0 + b[0])
    dVd, dcd = V[0, 1] - V[0, 0], c[1] - c[0]
    s = [-1.0, 1.0]
    m = [h0 * dVd + dcd, h1 * dVd + dcd]
    L = 0.5 * sum(math.log1p(math.exp(-s[t] * m[t])) for t in range(2))
    assert abs(r["loss"] - L) < 1e-15
    dm = [0.5 * (-s[t]) * sig(-s[t] * m[t]) for t in range(2)]        # dL/dm_t
    # output layer: m_t depends on V1 (+h_t), V0 (-h_t), c1 (+1), c0 (-1)
    np.testing.assert_allclose(r["dV"], [[-(dm[0] * h0 + dm[1] * h1), dm[0] * h0 + dm[1] * h1]], atol=1e-15)
    np.testing.assert_allclose(r["dc"], [-(dm[0] + dm[1]), dm[0] + dm[1]], atol=1e-15)
    da1 = dm[1] * dVd * h1 * (1 - h1)
    da0 = (dm[0] * dVd + da1 * wh[0, 0]) * h0 * (1 - h0)
    np.testing.assert_allclose(r["dWh"], [[da1 * h0]], atol=1e-15)     # a_0 sees h_{-1} = 0
    np.testing.assert_allclose(r["db"], [da0 + da1], atol=1e-15)
    np.testing.assert_allclose(r["dWx"], [[da1], [da0]], atol=1e-15)   # x_0 = token 1, x_1 = token 0
    np.testing.assert_allclose(r["dh0"], [[da0 * wh[0, 0]]], atol=1e-15)


# ---- orientation pins: a transposed operand must fail ---------------------------------------------
def test_matrix_orientations():
    """One recurrent step and one output row against explicit index sums."""
    p = as64(ri.make_case(5, 3, 4, 2, 1, input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH,
                          loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.8), bias_std=0.3,
                          with_h0=True, seed=71))
    h_all = oracle.forward(p, p["h0"])
    for j in range(3):
        a = p["b"][j] + sum(p["Wx"][j, k] * p["X"][0, 0, k] for k in range(5)) \
            + sum(p["Wh"][j, i] * p["h0"][0, i] for i in range(3))
        assert abs(h_all[1, 0, j] - math.tanh(a)) < 1e-15
    _, Z = oracle.loss(p, h_all, want_Z=True)
    for k in range(4):
        z = p["c"][k] + sum(h_all[2, 0, i] * p["V"][i, k] for i in range(3))
        assert abs(Z[1, k] - z) < 1e-15
