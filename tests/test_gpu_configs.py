"""GPU parity on the five benchmark configurations, in the launch configuration bench.py times.

Every configuration is compared element by element at full size.  C4 costs the double-precision
oracle about a teraflop (run once, shared by both output-layer modes); C2 is the whole stream of
10000 dependent windows, through the three calls and through the one-launch call bench.py times.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import GRAD_NAMES, H_ATOL, LOSS_RTOL, Runner, compare, dev, grad_close, run_gpu

pytestmark = pytest.mark.gpu


def test_c1_tiny_full():
    case = ri.make_config("C1")
    compare(run_gpu(case), oracle.fwd_bptt(case))


def test_c3_larger_hidden_full():
    case = ri.make_config("C3")
    print("C3 oracle ...", flush=True)
    ref = oracle.fwd_bptt(case)
    got = run_gpu(case)
    compare(got, ref)
    unseen = np.setdiff1d(np.arange(10000), np.unique(case["x"]))
    assert np.all(got["dWx"][unseen] == 0.0)


def test_c2_stream_of_dependent_windows():
    """All 10000 windows on the GPU with the state carried; the oracle runs the whole stream
    forward (cheap), every sampled window's loss and a few windows' full gradients."""
    stream = ri.make_config("C2")
    T, W = stream["seq_len"], stream["windows"]
    whole = dict(stream); whole["seq_len"] = T * W; whole["windows"] = 1
    print("C2 oracle forward over the stream ...", flush=True)
    h_ref = oracle.forward(whole)                                   # [T*W+1, 1, H]

    r = Runner(ri.window(stream, 0))
    x_all, y_all = dev(stream["x"]), dev(stream["y"])
    losses = torch.zeros(W, device="cuda")
    carry = [torch.zeros_like(r.h_last), torch.zeros_like(r.h_last)]
    grad_windows = [0, 1, 4999, W - 1]
    kept = {}
    for w in range(W):
        r.x, r.y = x_all[w * T:(w + 1) * T], y_all[w * T:(w + 1) * T]
        r.h0 = None if w == 0 else carry[(w - 1) & 1]
        r.h_last = carry[w & 1]
        r.loss = losses[w:w + 1]
        r.forward(); r.loss_(); r.bptt()
        if w in grad_windows:
            kept[w] = r.results()
    torch.cuda.synchronize()
    losses = losses.cpu().numpy()
    assert np.max(np.abs(carry[(W - 1) & 1].cpu().numpy() - h_ref[-1])) <= H_ATOL
    rng = np.random.default_rng(7)
    for w in sorted(set(rng.integers(0, W, 60).tolist() + grad_windows)):
        win = ri.window(stream, w)
        ref = oracle.fwd_bptt(win, h0=h_ref[w * T]) if w in grad_windows else None
        h_w = h_ref[w * T:(w + 1) * T + 1]
        L = ref["loss"] if ref else oracle.loss(win, h_w)
        assert abs(losses[w] - L) <= LOSS_RTOL * abs(L), (w, losses[w], L)
        if ref:
            compare(kept[w], ref, check_dh0=False)


def test_c2_whole_stream_through_the_one_launch_call():
    """The path bench.py times on C2: rnn_window, 10000 dependent windows, the state carried on
    the GPU from window to window.  Every window's loss against the oracle; all gradients of
    windows spread over the stream; the accumulate-mode sum over the first 500 windows."""
    stream = ri.make_config("C2")
    T, W, H = stream["seq_len"], stream["windows"], stream["hidden"]
    whole = dict(stream); whole["seq_len"] = T * W; whole["windows"] = 1
    print("C2 oracle forward over the stream ...", flush=True)
    h_ref = oracle.forward(whole)                                   # [T*W+1, 1, H]
    wide = dict(stream)                                             # float64 once, not once per oracle call
    for k in ("Wx", "Wh", "b", "V", "c"):
        wide[k] = stream[k].astype(np.float64)

    dims = rnn.Dims.of(ri.window(stream, 0))
    names = ("Wx", "Wh", "b", "V", "c")
    params = {k: dev(stream[k]) for k in names}
    x_all, y_all = dev(stream["x"]), dev(stream["y"])
    ws = torch.full((rnn.rnn_window_workspace_bytes(dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    rnn.rnn_window_workspace_init(dims, ws)
    grads = {"d" + k: torch.full_like(v, float("nan")) for k, v in params.items()}
    h_all = torch.full((T + 1, 1, H), float("nan"), device="cuda")
    dh0 = torch.full((1, H), float("nan"), device="cuda")
    carry = [torch.zeros(1, H, device="cuda"), torch.zeros(1, H, device="cuda")]
    losses = torch.zeros(W, device="cuda")
    grad_windows = [0, 1, 2, 777, 2500, 4999, 7321, W - 2, W - 1]
    kept = {}
    print("C2 GPU: 10000 windows through rnn_window ...", flush=True)
    for w in range(W):
        rnn.rnn_window(dims, params, x_all[w * T:(w + 1) * T], y_all[w * T:(w + 1) * T],
                       None if w == 0 else carry[(w - 1) & 1], None, h_all, carry[w & 1],
                       losses[w:w + 1], grads, dh0, ws)
        if w in grad_windows:
            torch.cuda.synchronize()
            kept[w] = {k: v.cpu().numpy() for k, v in grads.items()}
            kept[w].update(h_all=h_all.cpu().numpy(), h_last=carry[w & 1].cpu().numpy(), dh0=dh0.cpu().numpy())
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    losses = losses.cpu().numpy()
    assert np.max(np.abs(carry[(W - 1) & 1].cpu().numpy() - h_ref[-1])) <= H_ATOL
    print("C2 oracle: loss of every window ...", flush=True)
    for w in range(W):
        L = oracle.loss(ri.window(wide, w), h_ref[w * T:(w + 1) * T + 1])
        assert abs(losses[w] - L) <= LOSS_RTOL * abs(L), (w, losses[w], L)
    for w in grad_windows:
        ref = oracle.fwd_bptt(ri.window(wide, w), h0=h_ref[w * T])
        kept[w]["loss"] = float(losses[w])
        compare(kept[w], ref)

    # accumulate mode: the first 500 windows summed into one set of buffers
    n_acc = 500
    print(f"C2 GPU + oracle: accumulate mode over {n_acc} windows ...", flush=True)
    adims = rnn.Dims.of(ri.window(stream, 0), rnn.FLAG_ACCUMULATE)
    for g in grads.values():
        g.zero_()
    loss1 = torch.zeros(1, device="cuda")
    for w in range(n_acc):
        rnn.rnn_window(adims, params, x_all[w * T:(w + 1) * T], y_all[w * T:(w + 1) * T],
                       None if w == 0 else carry[(w - 1) & 1], None, None, carry[w & 1], loss1, grads, None, ws)
    torch.cuda.synchronize()
    assert rnn.rnn_train_stream_status(ws) == 0
    total = {k: 0.0 for k in GRAD_NAMES}
    for w in range(n_acc):
        ref = oracle.fwd_bptt(ri.window(wide, w), h0=h_ref[w * T])
        for k in GRAD_NAMES:
            total[k] = total[k] + ref[k]
    for k in GRAD_NAMES:
        grad_close(k, grads[k].cpu().numpy(), total[k])


OUTPUT_MODES = pytest.mark.parametrize("flags", [0, rnn.FLAG_BF16X3_OUTPUT], ids=["f32", "bf16x3"])
_c4_cache = {}


def c4_reference(key, make):
    """The oracle's C4 results, computed once for both output-layer modes."""
    if key not in _c4_cache:
        _c4_cache[key] = make()
    return _c4_cache[key]


@OUTPUT_MODES
def test_c4_reduced_length_full_parity(flags):
    case = ri.make_config("C4", seq_len=6)
    print("C4 (T=6) oracle ...", flush=True)
    ref = c4_reference("short", lambda: oracle.fwd_bptt(case))
    compare(run_gpu(case, flags), ref)


@OUTPUT_MODES
def test_c4_full_size_every_tensor(flags):
    """T = 256, B = 64: the launch plans bench.py times (K cut of dV and dWh at K = 16384, the
    grouped token scatter over 16384 rows, 511 step launches)."""
    case = ri.make_config("C4")
    T, B, H, O = case["seq_len"], case["batch"], case["hidden"], case["out_dim"]
    print("C4 GPU ...", flush=True)
    got = run_gpu(case, flags)

    def reference():
        print("C4 oracle forward, loss and backpropagation (about 1.1 TFLOP in double) ...", flush=True)
        return oracle.fwd_bptt(case)
    ref = c4_reference("full", reference)
    compare(got, ref)
    # invariants that hold at any size
    assert abs(got["dc"].sum()) < 1e-4
    assert np.max(np.abs(got["dV"].sum(1))) < 1e-4
    np.testing.assert_allclose(got["dWx"].sum(0), got["db"], rtol=1e-3, atol=1e-6)
    unseen = np.setdiff1d(np.arange(O), np.unique(case["x"]))
    assert np.all(got["dWx"][unseen] == 0.0)


@OUTPUT_MODES
def test_c5_long_dense_sequence_full(flags):
    case = ri.make_config("C5")
    print("C5 GPU ...", flush=True)
    got = run_gpu(case, flags)
    print("C5 oracle (about 0.4 TFLOP in double) ...", flush=True)
    ref = c4_reference("c5", lambda: oracle.fwd_bptt(case))
    compare(got, ref)
