"""GPU parity of the persistent multi-window SGD driver against the oracle's driver."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import dev

pytestmark = pytest.mark.gpu
PNAMES = ("Wx", "Wh", "b", "V", "c")


def run_gpu_stream(case, ids, n_windows, lr, h0=None):
    dims = rnn.Dims.of(case)
    params = {k: dev(case[k]) for k in PNAMES}
    d_ids = dev(ids.reshape(-1))
    h_last = torch.full((case["hidden"],), float("nan"), device="cuda")
    losses = torch.full((max(n_windows, 1),), float("nan"), device="cuda")
    ws = torch.full((rnn.rnn_train_stream_workspace_bytes(dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    rnn.rnn_train_stream(dims, params, d_ids, n_windows, lr, dev(h0), h_last, losses, ws)
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    out = {k: v.cpu().numpy() for k, v in params.items()}
    out["h_last"] = h_last.cpu().numpy()
    out["losses"] = losses.cpu().numpy()[:n_windows]
    return out


def close(name, got, ref, rtol):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert np.all(np.isfinite(got)), name
    mx, scale = np.abs(got - ref).max(), np.abs(ref).max()
    print(f"  {name}: max|diff| {mx:.3e} scale {scale:.3e}", flush=True)
    assert mx <= rtol * scale + 1e-30, f"{name}: max|diff| {mx:.3e} > {rtol} * {scale:.3e}"


def compare_stream(got, ref, n_windows, param_rtol=1e-3):
    np.testing.assert_allclose(got["losses"], ref["losses"], rtol=1e-4, atol=0)
    for k in PNAMES:
        close(k, got[k], ref[k], param_rtol)
    assert np.max(np.abs(got["h_last"] - ref["h_last"].reshape(-1))) <= 1e-4


CASES = {
    "tiny": dict(in_dim=64, hidden=16, out_dim=64, seq_len=8, windows=6, lr=0.3),
    "ragged": dict(in_dim=300, hidden=37, out_dim=300, seq_len=5, windows=9, lr=0.2, act=ri.ACT_TANH, with_h0=True),
    "one_step": dict(in_dim=260, hidden=100, out_dim=260, seq_len=1, windows=7, lr=0.2),
    "wide": dict(in_dim=1000, hidden=128, out_dim=1000, seq_len=32, windows=4, lr=0.1),
}


@pytest.mark.parametrize("name", list(CASES))
def test_stream_matches_oracle(name):
    kw = dict(CASES[name])
    lr = kw.pop("lr")
    W = kw["windows"]
    print(f"case {name}: {kw}", flush=True)
    case = ri.make_case(batch=1, wdist=("normal", 0.3), bias_std=0.1, seed=4242, **kw)
    ids = ri.stream_ids(case)
    ref = oracle.train_stream(case, ids, W, lr, h0=case.get("h0"))
    got = run_gpu_stream(case, ids, W, lr, h0=case.get("h0"))
    compare_stream(got, ref, W)


def test_rnnlm_shape_300_windows():
    W, lr = 300, 0.1
    print("case C2 x 300 windows", flush=True)
    case = ri.make_config("C2", windows=W)
    ids = ri.stream_ids(case)
    ref = oracle.train_stream(case, ids, W, lr)
    got = run_gpu_stream(case, ids, W, lr)
    compare_stream(got, ref, W)
    # rows of Wx whose token never occurs are untouched, bit for bit
    unseen = np.setdiff1d(np.arange(case["in_dim"]), ids[:W * case["seq_len"]].reshape(-1))
    np.testing.assert_array_equal(got["Wx"][unseen], case["Wx"][unseen])


def test_rnnlm_shape_2000_windows_and_run_to_run_identical():
    # long enough for rounding differences of the float32 trajectory to show if they grew
    W, lr = 2000, 0.1
    print("case C2 x 2000 windows", flush=True)
    case = ri.make_config("C2", windows=W)
    ids = ri.stream_ids(case)
    ref = oracle.train_stream(case, ids, W, lr)
    got = run_gpu_stream(case, ids, W, lr)
    compare_stream(got, ref, W)
    assert got["losses"][-200:].mean() < got["losses"][:20].mean() - 1.0     # it learns the unigram statistics
    again = run_gpu_stream(case, ids, W, lr)
    for k in PNAMES + ("losses", "h_last"):
        np.testing.assert_array_equal(got[k], again[k])


def test_windows_can_be_split_over_calls():
    # two calls of 3 windows with the state carried equal one call of 6 windows, bit for bit
    case = ri.make_case(batch=1, wdist=("normal", 0.3), bias_std=0.1, seed=99, in_dim=500, hidden=64,
                        out_dim=500, seq_len=7, windows=6)
    ids = ri.stream_ids(case)
    T, lr = case["seq_len"], 0.2
    one = run_gpu_stream(case, ids, 6, lr)
    first = run_gpu_stream(case, ids[:3 * T + 1], 3, lr)
    mid = dict(case)
    mid.update({k: first[k] for k in PNAMES})
    second = run_gpu_stream(mid, ids[3 * T:], 3, lr, h0=first["h_last"])
    for k in PNAMES + ("h_last",):
        np.testing.assert_array_equal(one[k], second[k])
    np.testing.assert_array_equal(one["losses"], np.concatenate([first["losses"], second["losses"]]))


def test_zero_windows_and_unsupported_shapes():
    case = ri.make_config("C1", seq_len=8, windows=2)
    dims = rnn.Dims.of(case)
    params = {k: dev(case[k]) for k in PNAMES}
    before = {k: v.clone() for k, v in params.items()}
    ws = torch.zeros(rnn.rnn_train_stream_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
    rnn.rnn_train_stream(dims, params, dev(ri.stream_ids(case).reshape(-1)), 0, 0.1, None, None, None, ws)
    torch.cuda.synchronize()
    for k in PNAMES:
        assert torch.equal(params[k], before[k])


def test_expired_wait_sets_the_status_word_and_the_grid_drains():
    # failure handling forced from the host: with a spin limit of one poll the waits between the
    # workgroups expire at once; every workgroup must leave, and the status word must say so
    rnn.rnn_set_wait_limit(1)
    case = ri.make_config("C2", windows=4)
    dims = rnn.Dims.of(case)
    params = {k: dev(case[k]) for k in PNAMES}
    ws = torch.zeros(rnn.rnn_train_stream_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
    try:
        rnn.rnn_train_stream(dims, params, dev(ri.stream_ids(case).reshape(-1)), 4, 0.1, None, None, None, ws)
        torch.cuda.synchronize()
    finally:
        rnn.rnn_set_wait_limit(0)
    assert rnn.rnn_train_stream_status(ws) == 1
    params = {k: dev(case[k]) for k in PNAMES}     # and the next call on the same workspace is fine
    losses = torch.zeros(4, device="cuda")
    rnn.rnn_train_stream(dims, params, dev(ri.stream_ids(case).reshape(-1)), 4, 0.1, None, None, losses, ws)
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    ref = oracle.train_stream(case, ri.stream_ids(case), 4, 0.1)
    np.testing.assert_allclose(losses.cpu().numpy(), ref["losses"], rtol=1e-4)
