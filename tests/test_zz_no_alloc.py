"""The one-window call for callers that cannot allocate (rnn_window_static: exchange boxes in a
fixed array of the library instead of a caller's workspace) against rnn_window, through the C ABI:
two calls in a row on the shared array, the second on a smaller problem, every output compared
with the workspace form's (same kernels, fixed summation order: identical bits)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import GRAD_NAMES, compare, dev

pytestmark = pytest.mark.gpu
PNAMES = ("Wx", "Wh", "b", "V", "c")


def run_both(case):
    dims = rnn.Dims.of(case)
    T, H = case["seq_len"], case["hidden"]
    params = {k: dev(case[k]) for k in PNAMES}
    x, y = dev(case["x"]), dev(case["y"])
    h0, dh_last = dev(case.get("h0")), dev(case.get("dh_last"))

    def buffers():
        out = {"d" + k: torch.full_like(v, float("nan")) for k, v in params.items()}
        out.update(h_all=torch.full((T + 1, 1, H), float("nan"), device="cuda"),
                   h_last=torch.full((1, H), float("nan"), device="cuda"),
                   loss=torch.full((1,), float("nan"), device="cuda"),
                   dh0=torch.full((1, H), float("nan"), device="cuda"))
        return out

    a, b = buffers(), buffers()
    ws = torch.full((rnn.rnn_window_workspace_bytes(dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    rnn.rnn_window_workspace_init(dims, ws)
    rnn.rnn_window(dims, params, x, y, h0, dh_last, a["h_all"], a["h_last"], a["loss"],
                   {k: a[k] for k in GRAD_NAMES}, a["dh0"], ws)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    rnn.rnn_window_static(dims, params, x, y, h0, dh_last, b["h_all"], b["h_last"], b["loss"],
                          {k: b[k] for k in GRAD_NAMES}, b["dh0"], status)
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    assert int(status.item()) == 0
    return ({k: v.cpu().numpy() for k, v in a.items()}, {k: v.cpu().numpy() for k, v in b.items()})


def test_static_scratch_form_matches_the_workspace_form_twice_in_a_row():
    big = ri.make_config("C2", windows=1)                       # 0.67 MB of boxes
    small = ri.make_case(in_dim=300, hidden=37, out_dim=300, seq_len=5, batch=1, act=ri.ACT_TANH,
                         with_h0=True, with_dh_last=True, wdist=("normal", 0.3), bias_std=0.1, seed=777)
    for name, case in (("rnnlm_window", big), ("smaller_ragged_tanh", small)):
        print(f"case {name}", flush=True)
        want, got = run_both(case)
        for k in want:
            assert np.all(np.isfinite(got[k])), k
            np.testing.assert_array_equal(got[k], want[k], err_msg=f"{name}: {k}")
        # and both agree with the oracle
        ref = oracle.fwd_bptt(case, h0=case.get("h0"), dh_last=case.get("dh_last"))
        got["loss"] = float(got["loss"][0])
        compare(got, ref)


def test_static_scratch_form_rejects_what_does_not_fit():
    case = ri.make_case(in_dim=8192, hidden=128, out_dim=8192, seq_len=32, batch=1,
                        wdist=("normal", 0.1), seed=3)     # 64 strips x 32 steps x 128 units of boxes
    dims = rnn.Dims.of(case)
    assert rnn.rnn_window_workspace_bytes(dims) > rnn.WINDOW_STATIC_BYTES
    params = {k: dev(case[k]) for k in PNAMES}
    grads = {"d" + k: torch.zeros_like(v) for k, v in params.items()}
    loss = torch.zeros(1, device="cuda")
    rc = rnn.rnn_window_static(dims, params, dev(case["x"]), dev(case["y"]), None, None, None, None, loss,
                               grads, None, None, check=False)
    assert rc == -5
    assert "rnn_window_static" in rnn.rnn_strerror(rc)
