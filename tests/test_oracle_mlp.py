"""Pins of the feed-forward classifier oracle (CPU only).  The paper gives the benchmark's
architectures and batch sizes (its neural-network training benchmark) but no equations, so the
pins are mathematical: central finite differences of the loss for every parameter of a small
network, the zero-weight closed form, logistic regression written out independently, torch's
autograd + SGD optimiser in float64 over several batches, a zero learning rate, and a problem
the update rule must learn."""
import numpy as np
import pytest
import torch

import rnn_inputs as ri
from oracle import mlp


def small(**kw):
    args = dict(in_dim=5, hidden=4, n_hidden=2, out_dim=3, batch=3, n_batches=4, bias_std=0.3, wscale=1.5, seed=5)
    args.update(kw)
    return ri.make_mlp_case(**args)


def loss_of(W, b, case, rows):
    acts, z = mlp.forward(W, b, case["X"][rows], case["act"])
    y = case["y"][rows]
    return float(np.mean(np.log(np.exp(z).sum(1)) - z[np.arange(len(y)), y]))   # unshifted, by the definition


@pytest.mark.parametrize("act", [ri.ACT_SIGMOID, ri.ACT_TANH])
@pytest.mark.parametrize("n_hidden", [0, 1, 3])
def test_gradients_match_central_differences(n_hidden, act):
    case = small(n_hidden=n_hidden, act=act)
    rows = slice(0, case["batch"])
    W = [w.astype(np.float64) for w in case["W"]]
    b = [v.astype(np.float64) for v in case["b"]]
    loss, dW, db = mlp.loss_and_grads(W, b, case["X"][rows], case["y"][rows], act)
    assert abs(loss - loss_of(W, b, case, rows)) < 1e-12
    eps = 1e-6
    for group, grads in ((W, dW), (b, db)):
        for l, arr in enumerate(group):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                keep = arr[idx]
                arr[idx] = keep + eps; lp = loss_of(W, b, case, rows)
                arr[idx] = keep - eps; lm = loss_of(W, b, case, rows)
                arr[idx] = keep
                assert abs((lp - lm) / (2 * eps) - grads[l][idx]) < 1e-8, (l, idx)


def test_zero_weights_closed_form():
    case = small(n_hidden=2, bias_std=0.0)
    case["W"] = [np.zeros_like(w) for w in case["W"]]
    B, O = case["batch"], case["out_dim"]
    out = mlp.train(case, lr=0.5, n_batches=1)
    assert abs(out["losses"][0] - np.log(O)) < 1e-12
    counts = np.bincount(case["y"][:B], minlength=O)
    np.testing.assert_allclose(out["b"][-1], -0.5 * (1.0 / O - counts / B), atol=1e-14)
    # tanh(0) = 0: the last layer's input is zero, so no weight moves; zero output weights send no gradient down
    for w in out["W"]:
        assert not w.any()
    for v in out["b"][:-1]:
        assert not v.any()


def test_no_hidden_layer_is_logistic_regression():
    case = small(n_hidden=0, in_dim=7, out_dim=4, batch=6)
    X, y = case["X"][:6].astype(np.float64), case["y"][:6]
    W, b = case["W"][0].astype(np.float64), case["b"][0].astype(np.float64)
    z = X @ W.T + b
    p = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-14)
    onehot = np.eye(4)[y]
    loss, dW, db = mlp.loss_and_grads([W], [b], X, y, case["act"])
    np.testing.assert_allclose(dW[0], (p - onehot).T @ X / 6, atol=1e-14)
    np.testing.assert_allclose(db[0], (p - onehot).mean(0), atol=1e-14)
    assert abs(loss + np.mean(np.log(p[np.arange(6), y]))) < 1e-13


@pytest.mark.parametrize("act", [ri.ACT_SIGMOID, ri.ACT_TANH])
def test_training_matches_torch_sgd_in_float64(act):
    case = small(n_hidden=2, in_dim=9, hidden=6, out_dim=5, batch=4, n_batches=5, act=act)
    lr = 0.3
    ref = mlp.train(case, lr)
    Ws = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in case["W"]]
    bs = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in case["b"]]
    opt = torch.optim.SGD(Ws + bs, lr=lr)
    X = torch.tensor(case["X"], dtype=torch.float64)
    y = torch.tensor(case["y"], dtype=torch.long)
    B = case["batch"]
    for i in range(case["n_batches"]):
        a = X[i * B:(i + 1) * B]
        for l in range(len(Ws) - 1):
            a = torch.nn.functional.linear(a, Ws[l], bs[l])
            a = torch.sigmoid(a) if act == ri.ACT_SIGMOID else torch.tanh(a)
        loss = torch.nn.functional.cross_entropy(torch.nn.functional.linear(a, Ws[-1], bs[-1]), y[i * B:(i + 1) * B])
        assert abs(loss.item() - ref["losses"][i]) < 1e-12
        opt.zero_grad()
        loss.backward()
        opt.step()
    for l in range(len(Ws)):
        np.testing.assert_allclose(ref["W"][l], Ws[l].detach().numpy(), atol=1e-13)
        np.testing.assert_allclose(ref["b"][l], bs[l].detach().numpy(), atol=1e-13)


def test_zero_learning_rate_changes_nothing_and_losses_are_per_batch():
    case = small()
    out = mlp.train(case, lr=0.0)
    B = case["batch"]
    for l, w in enumerate(case["W"]):
        np.testing.assert_array_equal(out["W"][l], w.astype(np.float64))
    for i in range(case["n_batches"]):
        rows = slice(i * B, (i + 1) * B)
        loss, _, _ = mlp.loss_and_grads(case["W"], case["b"], case["X"][rows], case["y"][rows], case["act"])
        assert out["losses"][i] == loss


def test_repeating_one_batch_is_learned():
    case = small(n_hidden=1, hidden=16, n_batches=1)
    rep = dict(case, X=np.tile(case["X"], (200, 1)), y=np.tile(case["y"], 200), n_batches=200)
    out = mlp.train(rep, lr=0.5)
    assert out["losses"][-1] < 0.05 * out["losses"][0]
