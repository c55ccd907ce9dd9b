"""Pins of the oracle's Gauss-Newton-vector product (CPU only).

The paper's section on the R-operator defines R{f} as the Jacobian-vector product (forward mode)
and names, for a recurrent network, the Gauss-Newton approximation of the Hessian times a vector,
computed as the vector-Jacobian product of the Jacobian-vector product.  It prints no formulas for
the network, so the pins are mathematical: central differences of the outputs along the direction
(the definition of a directional derivative), the explicit matrix J^T M J assembled from a
finite-difference Jacobian on a tiny case, symmetry and positive semi-definiteness of that
matrix, and torch's forward-over-reverse autograd in float64.
"""
import numpy as np
import pytest

import oracle
import rnn_inputs as ri

PNAMES = ("Wx", "Wh", "b", "V", "c")


def as64(case):
    p = dict(case)
    for k in PNAMES + ("X", "Y", "h0"):
        if p.get(k) is not None:
            p[k] = np.array(p[k], dtype=np.float64)
    return p


def tiny(kind, **kw):
    if kind == "lm":
        args = dict(in_dim=5, hidden=3, out_dim=5, seq_len=3, batch=2, wdist=("normal", 0.7),
                    bias_std=0.3, with_h0=True, seed=31, tokens="uniform")
    else:
        args = dict(in_dim=4, hidden=3, out_dim=4, seq_len=3, batch=2, input_kind=ri.INPUT_DENSE,
                    act=ri.ACT_TANH, loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.7),
                    bias_std=0.3, with_h0=True, seed=32)
    args.update(kw)
    return as64(ri.make_case(**args))


def outputs(p):
    h_all = oracle.forward(p, p.get("h0"))
    if p["loss_kind"] == 0:
        _, Z = oracle.loss(p, h_all, want_Z=True)
        return Z
    N, O = p["seq_len"] * p["batch"], p["out_dim"]
    return (h_all[1:].reshape(N, -1) @ p["V"] + p["c"]).reshape(N, O)   # linear outputs, written out


def shifted(p, gamma, eps):
    q = dict(p)
    for k in PNAMES:
        q[k] = p[k] + eps * np.asarray(gamma[k], dtype=np.float64)
    return q


@pytest.mark.parametrize("kind", ["lm", "dense"])
def test_r_operator_is_the_directional_derivative_of_the_outputs(kind):
    p = tiny(kind, hidden=6, seq_len=5)
    gamma = ri.make_direction(p, 1)
    r = oracle.gauss_newton_vec(p, gamma, want_Rz=True)
    eps = 1e-6
    fd = (outputs(shifted(p, gamma, eps)) - outputs(shifted(p, gamma, -eps))) / (2 * eps)
    np.testing.assert_allclose(r["Rz"], fd, rtol=0, atol=1e-8)


def explicit_matrix(p, metric):
    """G = J^T M J with J from central differences of the outputs, one parameter at a time."""
    flat = np.concatenate([p[k].reshape(-1) for k in PNAMES])
    shapes = [p[k].shape for k in PNAMES]

    def unflat(v):
        q, o = dict(p), 0
        for k, sh in zip(PNAMES, shapes):
            n = int(np.prod(sh))
            q[k] = v[o:o + n].reshape(sh)
            o += n
        return q
    Z0 = outputs(p)
    N, O = Z0.shape
    J = np.zeros((N * O, flat.size))
    eps = 1e-6
    for i in range(flat.size):
        vp, vm = flat.copy(), flat.copy()
        vp[i] += eps
        vm[i] -= eps
        J[:, i] = ((outputs(unflat(vp)) - outputs(unflat(vm))) / (2 * eps)).reshape(-1)
    M = np.zeros((N * O, N * O))
    for n in range(N):
        blk = slice(n * O, (n + 1) * O)
        if metric == 1:
            M[blk, blk] = np.eye(O)
        elif p["loss_kind"] == 0:
            e = np.exp(Z0[n] - Z0[n].max())
            pr = e / e.sum()
            M[blk, blk] = (np.diag(pr) - np.outer(pr, pr)) / N     # Hessian of the mean cross-entropy
        else:
            M[blk, blk] = 2.0 * np.eye(O) / (N * O)                # Hessian of the mean squared error
    return J.T @ M @ J


@pytest.mark.parametrize("kind,metric", [("lm", 0), ("lm", 1), ("dense", 0), ("dense", 1)])
def test_against_the_explicit_gauss_newton_matrix(kind, metric):
    p = tiny(kind)
    G = explicit_matrix(p, metric)
    assert np.allclose(G, G.T, atol=1e-9)
    assert np.linalg.eigvalsh(G).min() > -1e-9
    for seed in (2, 3):
        gamma = ri.make_direction(p, seed)
        r = oracle.gauss_newton_vec(p, gamma, metric=metric)
        got = np.concatenate([r["G" + k].reshape(-1) for k in PNAMES])
        want = G @ np.concatenate([np.asarray(gamma[k], np.float64).reshape(-1) for k in PNAMES])
        np.testing.assert_allclose(got, want, rtol=0, atol=2e-7 * max(1.0, np.abs(want).max()))


def test_symmetric_and_positive_semidefinite_on_a_larger_case():
    p = as64(ri.make_case(40, 9, 40, 7, 3, wdist=("normal", 0.5), bias_std=0.3, with_h0=True, seed=33))
    g1, g2 = ri.make_direction(p, 4), ri.make_direction(p, 5)
    r1, r2 = oracle.gauss_newton_vec(p, g1), oracle.gauss_newton_vec(p, g2)
    dot = lambda a, b: sum(float(np.sum(np.asarray(a[k], np.float64) * b["G" + k])) for k in PNAMES)
    assert abs(dot(g1, r2) - dot(g2, r1)) <= 1e-12 * max(1.0, abs(dot(g1, r2)))
    assert dot(g1, r1) >= 0.0 and dot(g2, r2) >= 0.0
    # a direction along the output bias only: J gamma = gamma_c in every row, so G_c = sum_n M_n gamma_c
    gc = {k: np.zeros_like(np.asarray(p[k])) for k in PNAMES}
    gc["c"] = np.asarray(g1["c"], np.float64)
    r = oracle.gauss_newton_vec(p, gc, want_Rz=True)
    np.testing.assert_allclose(r["Rz"], np.tile(gc["c"], (r["Rz"].shape[0], 1)), atol=1e-15)
    Z = outputs(p)
    want = np.zeros(p["out_dim"])
    for n in range(Z.shape[0]):
        e = np.exp(Z[n] - Z[n].max())
        pr = e / e.sum()
        want += (pr * gc["c"] - pr * (pr @ gc["c"])) / Z.shape[0]
    np.testing.assert_allclose(r["Gc"], want, atol=1e-14)


@pytest.mark.parametrize("kind", ["lm_sigmoid_ce", "dense_tanh_mse"])
def test_against_torch_forward_over_reverse(kind):
    import torch
    from torch.autograd.functional import jvp, vjp
    torch.set_num_threads(2)
    if kind == "lm_sigmoid_ce":
        p = as64(ri.make_case(12, 5, 12, 4, 2, wdist=("normal", 0.5), bias_std=0.3, with_h0=True, seed=34))
    else:
        p = as64(ri.make_case(6, 5, 6, 4, 2, input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH,
                              loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.5), bias_std=0.3,
                              with_h0=True, seed=35))
    gamma = ri.make_direction(p, 6)
    theta = tuple(torch.tensor(p[k]) for k in PNAMES)
    gam = tuple(torch.tensor(np.asarray(gamma[k], np.float64)) for k in PNAMES)
    h0 = torch.tensor(p["h0"])

    def net(Wx, Wh, b, V, c):
        h, hs = h0, []
        for t in range(p["seq_len"]):
            inp = Wx[torch.tensor(p["x"][t], dtype=torch.long)] if p["input_kind"] == 0 else torch.tensor(p["X"][t]) @ Wx.T
            a = inp + h @ Wh.T + b
            h = torch.sigmoid(a) if p["act"] == 0 else torch.tanh(a)
            hs.append(h)
        return (torch.stack(hs) @ V + c).reshape(-1, p["out_dim"])

    Z, Rz = jvp(net, theta, gam)
    N, O = Z.shape
    if p["loss_kind"] == 0:
        pr = torch.softmax(Z, dim=1)
        u = (pr * Rz - pr * (pr * Rz).sum(dim=1, keepdim=True)) / N
    else:
        u = 2.0 * Rz / (N * O)
    _, G = vjp(net, theta, u)
    r = oracle.gauss_newton_vec(p, gamma, want_Rz=True)
    np.testing.assert_allclose(r["Rz"], Rz.numpy(), atol=1e-13)
    for k, gk in zip(PNAMES, G):
        np.testing.assert_allclose(r["G" + k], gk.numpy(), atol=1e-13)
