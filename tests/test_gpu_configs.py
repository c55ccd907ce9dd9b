"""GPU parity on the five benchmark configurations, in the launch configuration bench.py times.

Where the oracle finishes in seconds the comparison is element by element at full size (C1, C3,
C5 and every sampled window of C2).  C4 at full size costs the double-precision oracle about a
teraflop, so there the forward states, the loss and all row statistics are compared in full,
gradients of the output layer on sampled columns computed from the oracle's states and
log-sum-exps by the definition, and the rest through invariants that hold at any size; a
reduced-length C4 (same widths and batch) is compared element by element.
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
def test_c4_full_size_sampled(flags):
    case = ri.make_config("C4")
    T, B, H, O = case["seq_len"], case["batch"], case["hidden"], case["out_dim"]
    N = T * B
    print("C4 GPU ...", flush=True)
    got = run_gpu(case, flags)

    def reference():
        print("C4 oracle forward ...", flush=True)
        h = oracle.forward(case)
        print("C4 oracle loss and row statistics (335 GFLOP in double) ...", flush=True)
        return (h,) + tuple(oracle.loss(case, h, want_lse=True))
    h_ref, L, lse = c4_reference("full", reference)
    assert np.max(np.abs(got["h_all"] - h_ref)) <= H_ATOL
    assert abs(got["loss"] - L) <= LOSS_RTOL * abs(L)
    # output-layer gradients on sampled columns, from the oracle's states and log-sum-exps
    Hs = h_ref[1:].reshape(N, H)
    y = case["y"].reshape(-1)
    cols = np.array([0, 1, 7, 999, 5000, 9999])
    Zc = Hs @ case["V"][:, cols].astype(np.float64) + case["c"][cols]
    dZc = (np.exp(Zc - lse[:, None]) - (y[:, None] == cols[None, :])) / N
    grad_close("dc[cols]", got["dc"][cols], dZc.sum(0))
    grad_close("dV[:,cols]", got["dV"][:, cols], Hs.T @ dZc)
    # invariants that hold at any size
    assert abs(got["dc"].sum()) < 1e-4
    assert np.max(np.abs(got["dV"].sum(1))) < 1e-4
    np.testing.assert_allclose(got["dWx"].sum(0), got["db"], rtol=1e-3, atol=1e-6)
    unseen = np.setdiff1d(np.arange(O), np.unique(case["x"]))
    assert np.all(got["dWx"][unseen] == 0.0)
    for k in GRAD_NAMES:
        assert np.all(np.isfinite(got[k]))


@OUTPUT_MODES
def test_c5_long_dense_sequence_full(flags):
    case = ri.make_config("C5")
    print("C5 GPU ...", flush=True)
    got = run_gpu(case, flags)
    print("C5 oracle (about 0.4 TFLOP in double) ...", flush=True)
    ref = c4_reference("c5", lambda: oracle.fwd_bptt(case))
    compare(got, ref)
