"""GPU parity of the fused one-window call (forward, loss and BPTT in one launch) against the
oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import GRAD_NAMES, compare, dev

pytestmark = pytest.mark.gpu
PNAMES = ("Wx", "Wh", "b", "V", "c")


class WindowRunner:
    def __init__(self, case, flags=0):
        self.case = case
        self.dims = rnn.Dims.of(case, flags)
        T, H = case["seq_len"], case["hidden"]
        self.params = {k: dev(case[k]) for k in PNAMES}
        self.h0, self.dh_last = dev(case.get("h0")), dev(case.get("dh_last"))
        self.h_all = torch.full((T + 1, 1, H), float("nan"), device="cuda")
        self.h_last = torch.full((1, H), float("nan"), device="cuda")
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.grads = {"d" + k: torch.full_like(v, float("nan")) for k, v in self.params.items()}
        self.dh0 = torch.full((1, H), float("nan"), device="cuda")
        nbytes = rnn.rnn_window_workspace_bytes(self.dims)
        self.ws = torch.full((nbytes + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        rnn.rnn_window_workspace_init(self.dims, self.ws)

    def run(self, x, y):
        rnn.rnn_window(self.dims, self.params, x, y, self.h0, self.dh_last, self.h_all, self.h_last,
                       self.loss, self.grads, self.dh0, self.ws)
        torch.cuda.synchronize()
        assert rnn.rnn_train_stream_status(self.ws) == 0
        out = {k: v.cpu().numpy() for k, v in self.grads.items()}
        out.update(loss=float(self.loss.item()), h_all=self.h_all.cpu().numpy(),
                   h_last=self.h_last.cpu().numpy(), dh0=self.dh0.cpu().numpy())
        return out


CASES = {
    "tiny_lm_config": dict(name="C1"),
    "rnnlm_window": dict(name="C2", windows=1),
    "ragged_tanh_state": dict(in_dim=300, hidden=37, out_dim=300, seq_len=5, act=ri.ACT_TANH,
                              with_h0=True, with_dh_last=True),
    "one_step": dict(in_dim=260, hidden=100, out_dim=260, seq_len=1, with_h0=True),
    "widest_longest": dict(in_dim=1000, hidden=128, out_dim=1000, seq_len=32, with_dh_last=True),
    "two_vocabularies": dict(in_dim=150, hidden=50, out_dim=420, seq_len=9),
    "repeated_tokens": dict(in_dim=3, hidden=20, out_dim=200, seq_len=24),
}


def make(spec):
    spec = dict(spec)
    if "name" in spec:
        return ri.make_config(spec.pop("name"), **spec)
    return ri.make_case(batch=1, wdist=("normal", 0.3), bias_std=0.1, seed=777, **spec)


@pytest.mark.parametrize("name", list(CASES))
def test_window_matches_oracle(name):
    print(f"case {name}", flush=True)
    case = make(CASES[name])
    ref = oracle.fwd_bptt(case, h0=case.get("h0"), dh_last=case.get("dh_last"))
    r = WindowRunner(case)
    got = r.run(dev(case["x"]), dev(case["y"]))
    compare(got, ref)
    # rows of dWx whose token does not occur are exactly zero
    unseen = np.setdiff1d(np.arange(case["in_dim"]), case["x"].reshape(-1))
    assert not got["dWx"][unseen].any()


def test_consecutive_windows_on_one_workspace_and_accumulate_mode():
    stream = ri.make_config("C2", windows=6)
    T = stream["seq_len"]
    r = WindowRunner(ri.window(stream, 0))
    x, y = dev(stream["x"]), dev(stream["y"])
    h = None
    total = {k: 0.0 for k in GRAD_NAMES}
    for w in range(6):
        case = ri.window(stream, w)
        ref = oracle.fwd_bptt(case, h0=h)
        r.h0 = dev(h.astype(np.float32)) if h is not None else None
        got = r.run(x[w * T:(w + 1) * T], y[w * T:(w + 1) * T])    # windows start anywhere in the stream
        compare(got, ref)
        h = ref["h_all"][-1]
        for k in GRAD_NAMES:
            total[k] = total[k] + ref[k]
    # accumulate mode: the same six windows summed into one set of buffers
    acc = WindowRunner(ri.window(stream, 0), flags=rnn.FLAG_ACCUMULATE)
    for g in acc.grads.values():
        g.zero_()
    h = None
    for w in range(6):
        acc.h0 = dev(h.astype(np.float32)) if h is not None else None
        got = acc.run(x[w * T:(w + 1) * T], y[w * T:(w + 1) * T])
        h = got["h_last"]
    from gpu_harness import grad_close
    for k in GRAD_NAMES:
        grad_close(k, got[k], total[k])


def test_window_agrees_with_the_three_calls():
    from gpu_harness import run_gpu
    case = ri.make_config("C2", windows=1)
    three = run_gpu(case)
    one = WindowRunner(case).run(dev(case["x"]), dev(case["y"]))
    assert abs(one["loss"] - three["loss"]) <= 2e-6 * abs(three["loss"])
    for k in GRAD_NAMES:
        np.testing.assert_allclose(one[k], three[k], rtol=0, atol=2e-5 * np.abs(three[k]).max())
