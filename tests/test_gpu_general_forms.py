"""rnn_window and rnn_train_stream on shapes outside their one-launch kernels (hidden > 128, long
windows, batches, wide vocabularies): the same entry points then enqueue the launches of
rnn_forward -> rnn_loss -> rnn_bptt (and one update launch per window).  Parity with the oracle,
through the C ABI, with the same tolerances as everywhere else."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import GRAD_NAMES, compare, dev, grad_close

pytestmark = pytest.mark.gpu
PNAMES = ("Wx", "Wh", "b", "V", "c")


def run_window(case, flags=0, keep_history=True, start=None):
    dims = rnn.Dims.of(case, flags)
    T, B, H = case["seq_len"], case["batch"], case["hidden"]
    params = {k: dev(case[k]) for k in PNAMES}
    h_all = torch.full((T + 1, B, H), float("nan"), device="cuda") if keep_history else None
    h_last = torch.full((B, H), float("nan"), device="cuda")
    loss = torch.full((1,), float("nan"), device="cuda")
    grads = {"d" + k: (torch.full_like(v, float("nan")) if start is None else dev(start["d" + k])) for k, v in params.items()}
    dh0 = torch.full((B, H), float("nan"), device="cuda")
    ws = torch.full((rnn.rnn_window_workspace_bytes(dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    rnn.rnn_window_workspace_init(dims, ws)
    rnn.rnn_window(dims, params, dev(case["x"]), dev(case["y"]), dev(case.get("h0")), dev(case.get("dh_last")),
                   h_all, h_last, loss, grads, dh0, ws)
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    out = {k: v.cpu().numpy() for k, v in grads.items()}
    out.update(loss=float(loss.item()), h_last=h_last.cpu().numpy(), dh0=dh0.cpu().numpy())
    if keep_history:
        out["h_all"] = h_all.cpu().numpy()
    return out


WINDOWS = {
    "hidden_200": dict(in_dim=300, hidden=200, out_dim=300, seq_len=12, batch=1, with_h0=True),
    "long_window": dict(in_dim=120, hidden=64, out_dim=120, seq_len=45, batch=1, act=ri.ACT_TANH, with_dh_last=True),
    "batch_of_three": dict(in_dim=90, hidden=40, out_dim=70, seq_len=5, batch=3, with_h0=True, with_dh_last=True),
    "wide_batched": dict(in_dim=260, hidden=600, out_dim=260, seq_len=22, batch=13),
}


@pytest.mark.parametrize("name", list(WINDOWS))
def test_window_outside_the_one_launch_kernel(name):
    print(f"case {name}", flush=True)
    case = ri.make_case(wdist=("normal", 0.2), bias_std=0.1, seed=909, **WINDOWS[name])
    ref = oracle.fwd_bptt(case, h0=case.get("h0"), dh_last=case.get("dh_last"))
    compare(run_window(case), ref)


def test_window_at_the_hidden_500_configuration_without_history_and_accumulating():
    case = ri.make_config("C3")
    ref = oracle.fwd_bptt(case)
    compare(run_window(case), ref)
    got = run_window(case, keep_history=False)                    # h_all not wanted: kept in the workspace
    assert abs(got["loss"] - ref["loss"]) <= 1e-4 * abs(ref["loss"])
    np.testing.assert_allclose(got["h_last"], ref["h_all"][-1], rtol=0, atol=2e-5)
    start = {k: np.ones_like(ref[k], dtype=np.float32) for k in GRAD_NAMES}
    acc = run_window(case, flags=rnn.FLAG_ACCUMULATE, start=start)
    for k in GRAD_NAMES:
        grad_close(k, acc[k] - 1.0, ref[k], rtol=2e-3)             # rounding of 1 + g, as in the other accumulate cases


STREAMS = {
    "hidden_200": dict(in_dim=300, hidden=200, out_dim=300, seq_len=6, batch=1, windows=5, lr=0.2),
    "batch_of_two_tanh": dict(in_dim=150, hidden=48, out_dim=150, seq_len=4, batch=2, windows=6, lr=0.3,
                              act=ri.ACT_TANH, with_h0=True),
    "long_windows": dict(in_dim=64, hidden=32, out_dim=64, seq_len=40, batch=1, windows=3, lr=0.1),
}


@pytest.mark.parametrize("name", list(STREAMS))
def test_stream_outside_the_one_launch_kernel(name):
    kw = dict(STREAMS[name])
    lr, W = kw.pop("lr"), kw["windows"]
    print(f"case {name}: {kw}", flush=True)
    case = ri.make_case(wdist=("normal", 0.3), bias_std=0.1, seed=515, **kw)
    ids = ri.stream_ids(case)
    ref = oracle.train_stream(case, ids, W, lr, h0=case.get("h0"))
    dims = rnn.Dims.of(case)
    params = {k: dev(case[k]) for k in PNAMES}
    B, H = case["batch"], case["hidden"]
    h_last = torch.full((B, H), float("nan"), device="cuda")
    losses = torch.full((W,), float("nan"), device="cuda")
    ws = torch.full((rnn.rnn_train_stream_workspace_bytes(dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    rnn.rnn_train_stream(dims, params, dev(ids.reshape(-1)), W, lr, dev(case.get("h0")), h_last, losses, ws)
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    np.testing.assert_allclose(losses.cpu().numpy(), ref["losses"], rtol=1e-4, atol=0)
    for k in PNAMES:
        grad_close(k, params[k].cpu().numpy().astype(np.float64) - case[k], ref[k] - case[k], rtol=2e-3)   # the updates
        grad_close(k, params[k].cpu().numpy(), ref[k])                                                     # the parameters
    assert np.max(np.abs(h_last.cpu().numpy() - ref["h_last"])) <= 1e-4
