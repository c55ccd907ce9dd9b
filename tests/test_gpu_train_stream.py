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
