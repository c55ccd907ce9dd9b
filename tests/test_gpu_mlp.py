"""GPU parity of the feed-forward classifier training step (rnn_mlp_train through the C ABI)
against the float64 numpy oracle: every batch's loss and every parameter after several SGD
steps, on ragged small shapes (tiles of 16 with tails, batches that are multiples of nothing)
and on the paper's three benchmark architectures at its three batch sizes."""
import numpy as np
import pytest
import torch

import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import dev, grad_close
from oracle import mlp

pytestmark = pytest.mark.gpu


def run_gpu(case, lr, n_batches=None, want_losses=True):
    n = case["n_batches"] if n_batches is None else n_batches
    dims = rnn.MlpDims.of(case)
    W = [dev(w) for w in case["W"]]
    b = [dev(v) for v in case["b"]]
    X, y = dev(case["X"]), dev(case["y"])
    losses = torch.full((max(n, 1),), float("nan"), device="cuda") if want_losses else None
    ws = torch.full((rnn.rnn_mlp_workspace_bytes(dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    rnn.rnn_mlp_train(dims, W, b, X, y, n, lr, losses, ws)
    torch.cuda.synchronize()
    return dict(W=[w.cpu().numpy() for w in W], b=[v.cpu().numpy() for v in b],
                losses=None if losses is None else losses.cpu().numpy()[:n])


def check(got, ref, case):
    if got["losses"] is not None:
        np.testing.assert_allclose(got["losses"], ref["losses"], rtol=1e-4)
    for l in range(case["n_hidden"] + 1):
        # parameters after the updates, and the accumulated update itself, at the gradient tolerance
        grad_close(f"W[{l}]", got["W"][l], ref["W"][l])
        grad_close(f"b[{l}]", got["b"][l], ref["b"][l])
        grad_close(f"dW[{l}]", got["W"][l].astype(np.float64) - case["W"][l], ref["W"][l] - case["W"][l], rtol=2e-3)
        if np.abs(ref["b"][l] - case["b"][l]).max() > 0:
            grad_close(f"db[{l}]", got["b"][l].astype(np.float64) - case["b"][l], ref["b"][l] - case["b"][l], rtol=2e-3)


SMALL = {
    "logistic_ragged": dict(in_dim=37, hidden=0, n_hidden=0, out_dim=7, batch=5, n_batches=3),
    "one_hidden_ragged": dict(in_dim=50, hidden=45, n_hidden=1, out_dim=10, batch=13, n_batches=4),
    "three_hidden_sigmoid": dict(in_dim=70, hidden=130, n_hidden=3, out_dim=11, batch=20, n_batches=3, act=ri.ACT_SIGMOID),
    "batch_one": dict(in_dim=33, hidden=64, n_hidden=2, out_dim=5, batch=1, n_batches=6),
    "wide_batch_and_tiles": dict(in_dim=300, hidden=272, n_hidden=2, out_dim=40, batch=70, n_batches=2),
    "many_classes": dict(in_dim=20, hidden=24, n_hidden=1, out_dim=200, batch=9, n_batches=2),
    # 16 classes: the widest output layer whose launch also forms the loss; 37 rows = 3 row groups, the last ragged
    "sixteen_classes_three_row_groups": dict(in_dim=45, hidden=40, n_hidden=1, out_dim=16, batch=37, n_batches=3),
    "seventeen_classes": dict(in_dim=45, hidden=40, n_hidden=1, out_dim=17, batch=37, n_batches=3),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_networks_match_oracle(name):
    case = ri.make_mlp_case(**SMALL[name], bias_std=0.2, seed=300 + len(name))
    lr = 0.2
    check(run_gpu(case, lr), mlp.train(case, lr), case)


@pytest.mark.parametrize("batch", [1, 10, 60])
@pytest.mark.parametrize("name", ["MLP0", "MLP1", "MLP3"])
def test_benchmark_architectures_match_oracle(name, batch):
    case = ri.make_mlp_config(name, batch, n_batches=3)
    lr = 0.05
    check(run_gpu(case, lr), mlp.train(case, lr), case)


def test_run_to_run_identical_and_no_losses_wanted():
    case = ri.make_mlp_config("MLP1", 10, n_batches=5)
    a = run_gpu(case, 0.1)
    b = run_gpu(case, 0.1, want_losses=False)
    for l in range(2):
        assert np.array_equal(a["W"][l], b["W"][l]) and np.array_equal(a["b"][l], b["b"][l])


def test_split_calls_equal_one_call():
    case = ri.make_mlp_config("MLP1", 10, n_batches=4)
    whole = run_gpu(case, 0.1)
    dims = rnn.MlpDims.of(case)
    W = [dev(w) for w in case["W"]]
    b = [dev(v) for v in case["b"]]
    X, y = dev(case["X"]), dev(case["y"])
    ws = torch.zeros(rnn.rnn_mlp_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
    losses = torch.zeros(4, device="cuda")
    rnn.rnn_mlp_train(dims, W, b, X, y, 1, 0.1, losses, ws)
    rnn.rnn_mlp_train(dims, W, b, X[10:], y[10:], 3, 0.1, losses[1:], ws)
    torch.cuda.synchronize()
    assert np.array_equal(losses.cpu().numpy(), whole["losses"])
    for l in range(2):
        assert np.array_equal(W[l].cpu().numpy(), whole["W"][l])

