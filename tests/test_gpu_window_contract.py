"""Launch contract of the one-launch kernels and of the short-sequence kernels whose workgroups
exchange tagged words: replays of a captured HIP graph (the tag is device state, so a replay never
meets its own tag in the words the previous replay left), the cooperative and the plain launch
form, and a GPU that is shared with another stream's long kernel while the call runs (bounded
waits: every kernel ends, and the status word tells whether the results are valid)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import GRAD_NAMES, Runner, compare, dev

pytestmark = pytest.mark.gpu
PNAMES = ("Wx", "Wh", "b", "V", "c")


class Buffers:
    def __init__(self, case, flags=0):
        self.dims = rnn.Dims.of(case, flags)
        T, H = case["seq_len"], case["hidden"]
        self.T = T
        self.params = {k: dev(case[k]) for k in PNAMES}
        self.x = torch.zeros(T, dtype=torch.int32, device="cuda")
        self.y = torch.zeros(T, dtype=torch.int32, device="cuda")
        self.h0 = torch.zeros(1, H, device="cuda")
        self.h_all = torch.full((T + 1, 1, H), float("nan"), device="cuda")
        self.h_last = torch.full((1, H), float("nan"), device="cuda")
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.grads = {"d" + k: torch.full_like(v, float("nan")) for k, v in self.params.items()}
        self.dh0 = torch.full((1, H), float("nan"), device="cuda")
        self.ws = torch.full((rnn.rnn_window_workspace_bytes(self.dims) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        rnn.rnn_window_workspace_init(self.dims, self.ws)

    def set_inputs(self, x, y, h0):
        self.x.copy_(x); self.y.copy_(y); self.h0.copy_(h0)

    def window(self):
        rnn.rnn_window(self.dims, self.params, self.x, self.y, self.h0, None, self.h_all, self.h_last,
                       self.loss, self.grads, self.dh0, self.ws)

    def results(self):
        torch.cuda.synchronize()
        out = {k: v.cpu().numpy().copy() for k, v in self.grads.items()}
        out.update(loss=float(self.loss.item()), h_all=self.h_all.cpu().numpy().copy(),
                   h_last=self.h_last.cpu().numpy().copy(), dh0=self.dh0.cpu().numpy().copy())
        return out


def assert_same_bits(a, b, what):
    for k in a:
        np.testing.assert_array_equal(np.asarray(a[k]), np.asarray(b[k]), err_msg=f"{what}: {k}")


def test_replays_of_a_captured_window_see_new_inputs():
    stream = ri.make_config("C2", windows=5)
    T = stream["seq_len"]
    x_all, y_all = dev(stream["x"]).reshape(-1), dev(stream["y"]).reshape(-1)
    cap, eager = Buffers(ri.window(stream, 0)), Buffers(ri.window(stream, 0))
    h = torch.zeros_like(cap.h0)
    cap.set_inputs(x_all[:T], y_all[:T], h)
    cap.window()                                  # warm-up outside the capture (one-time attribute calls)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cap.window()
    for w in range(5):                            # every replay: new tokens, new initial state
        print(f"replay {w}", flush=True)
        xs, ys = x_all[w * T:(w + 1) * T], y_all[w * T:(w + 1) * T]
        cap.set_inputs(xs, ys, h)
        for g in cap.grads.values():
            g.fill_(float("nan"))
        graph.replay()
        got = cap.results()
        eager.set_inputs(xs, ys, h)
        eager.window()
        want = eager.results()
        assert rnn.rnn_train_stream_status(cap.ws) == 0
        assert_same_bits(got, want, f"replay {w}")
        ref = oracle.fwd_bptt(ri.window(stream, w), h0=h.cpu().numpy())
        compare(got, ref)
        h = torch.from_numpy(got["h_last"]).cuda()


def test_replays_of_the_three_captured_calls_on_a_short_sequence():
    """rnn_forward -> rnn_loss -> rnn_bptt of one short window (column-strip kernels that exchange
    tagged words) captured once and replayed on new inputs."""
    stream = ri.make_config("C2", windows=4)
    T = stream["seq_len"]
    r = Runner(ri.window(stream, 0))
    e = Runner(ri.window(stream, 0))
    x_all, y_all = dev(stream["x"]), dev(stream["y"])
    for run in (r, e):
        run.x, run.y = torch.zeros_like(x_all[:T]), torch.zeros_like(y_all[:T])
        run.h0 = torch.zeros_like(run.h_last)
    r.x.copy_(x_all[:T]); r.y.copy_(y_all[:T])
    r.forward(); r.loss_(); r.bptt()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        r.forward(); r.loss_(); r.bptt()
    h = torch.zeros_like(r.h_last)
    for w in range(4):
        print(f"replay {w}", flush=True)
        for run in (r, e):
            run.x.copy_(x_all[w * T:(w + 1) * T]); run.y.copy_(y_all[w * T:(w + 1) * T]); run.h0.copy_(h)
        graph.replay()
        got = r.results()
        e.step()
        want = e.results()
        assert rnn.rnn_workspace_status(r.dims, r.ws) == 0
        assert_same_bits({k: got[k] for k in GRAD_NAMES + ("loss", "h_all", "dh0")},
                         {k: want[k] for k in GRAD_NAMES + ("loss", "h_all", "dh0")}, f"replay {w}")
        compare(got, oracle.fwd_bptt(ri.window(stream, w), h0=h.cpu().numpy()))
        h = torch.from_numpy(got["h_last"]).cuda()


def test_window_after_a_stream_on_the_same_workspace():
    """rnn_train_stream leaves words with its own tags in the boxes; a later rnn_window on the same
    memory continues above them."""
    case = ri.make_config("C1", seq_len=8, windows=6)
    ids = ri.stream_ids(case)
    dims = rnn.Dims.of(case)
    params = {k: dev(case[k]) for k in PNAMES}
    nbytes = max(rnn.rnn_train_stream_workspace_bytes(dims), rnn.rnn_window_workspace_bytes(dims))
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    rnn.rnn_train_stream(dims, params, dev(ids.reshape(-1)), 6, 0.0, None, None, None, ws)   # lr 0: parameters stay
    b = Buffers(ri.window(case, 0))
    b.ws = ws
    for w in (0, 1, 2):
        win = ri.window(case, w)
        b.set_inputs(dev(win["x"]).reshape(-1), dev(win["y"]).reshape(-1), torch.zeros_like(b.h0))
        b.window()
        got = b.results()
        assert rnn.rnn_train_stream_status(ws) == 0
        compare(got, oracle.fwd_bptt(win, h0=np.zeros((1, case["hidden"]))))


def test_cooperative_and_plain_launch_give_the_same_bits():
    case = ri.make_config("C2", windows=1)
    x, y = dev(case["x"]).reshape(-1), dev(case["y"]).reshape(-1)
    plain, coop = Buffers(case), Buffers(case, rnn.FLAG_COOPERATIVE)
    for b in (plain, coop):
        b.set_inputs(x, y, torch.zeros_like(b.h0))
        b.window()
    a, c = plain.results(), coop.results()
    assert rnn.rnn_train_stream_status(plain.ws) == 0 and rnn.rnn_train_stream_status(coop.ws) == 0
    assert_same_bits(a, c, "cooperative vs plain")


def test_window_beside_a_long_kernel_on_another_stream():
    """The plain launch relies on the GPU not being occupied by other work.  With a long product
    resident on a second stream the call either still fits (status 0, results as the oracle's) or
    its bounded waits expire (status 1, results invalid): never a hang, and after a new set-up of
    the workspace the next call is good."""
    case = ri.make_config("C2", windows=1)
    ref = oracle.fwd_bptt(case)
    x, y = dev(case["x"]).reshape(-1), dev(case["y"]).reshape(-1)
    b = Buffers(case)
    b.set_inputs(x, y, torch.zeros_like(b.h0))
    b.window()
    torch.cuda.synchronize()
    other = torch.cuda.Stream()
    A = torch.randn(8192, 8192, device="cuda")
    C = torch.empty_like(A)
    torch.mm(A, A, out=C)                          # warm-up of the product
    torch.cuda.synchronize()
    rnn.rnn_set_wait_limit(20000)                  # a few milliseconds of polling at most
    try:
        with torch.cuda.stream(other):
            for _ in range(4):
                torch.mm(A, A, out=C)              # about 7 ms each: the chip stays full
        b.window()                                  # on the current stream, beside the products
        torch.cuda.synchronize()
    finally:
        rnn.rnn_set_wait_limit(0)
    status = rnn.rnn_train_stream_status(b.ws)
    print(f"status beside a resident product: {status}", flush=True)
    assert status in (0, 1)
    if status == 0:
        compare(b.results(), ref)
    # a workspace that saw an expired wait is set up again before its next use
    rnn.rnn_window_workspace_init(b.dims, b.ws)
    b.window()
    got = b.results()
    assert rnn.rnn_train_stream_status(b.ws) == 0
    compare(got, ref)


@pytest.mark.parametrize("shape", ["wide_batched_loop", "batch_1_loop_of_several_workgroups"])
def test_smallest_wait_limit_on_the_multi_workgroup_loops_never_hangs(shape):
    """The time loops whose workgroups hand the state to each other wait with a bound.  With the
    bound set to a single poll from the host a wait may expire (status 1, results invalid) or not
    (status 0, results as the oracle's); either way every kernel ends, and after a new set-up of
    the workspace with the normal bound the next call is good."""
    from gpu_harness import Runner
    spec = (dict(in_dim=260, hidden=600, out_dim=260, seq_len=22, batch=13) if shape == "wide_batched_loop"
            else dict(in_dim=200, hidden=300, out_dim=200, seq_len=9, batch=1))
    case = ri.make_case(wdist=("normal", 0.2), bias_std=0.1, seed=31, **spec)
    ref = oracle.fwd_bptt(case)
    r = Runner(case)
    print("variant", rnn.rnn_recurrence_variant(r.dims), flush=True)
    rnn.rnn_set_wait_limit(1)
    try:
        for rep in range(3):
            rnn.rnn_workspace_init(r.dims, r.ws)
            r.step()
            status = rnn.rnn_workspace_status(r.dims, r.ws)
            print(f"rep {rep}: status {status}", flush=True)
            assert status in (0, 1)
            if status == 0:
                compare(r.results(), ref)
    finally:
        rnn.rnn_set_wait_limit(0)
    rnn.rnn_workspace_init(r.dims, r.ws)
    r.step()
    assert rnn.rnn_workspace_status(r.dims, r.ws) == 0
    compare(r.results(), ref)


@pytest.mark.parametrize("shape", ["wide_batched_loop", "batch_1_loop_of_several_workgroups"])
def test_replays_of_the_three_captured_calls_with_a_multi_workgroup_loop(shape):
    """The cooperative launches of the multi-workgroup time loops inside a captured graph: every
    replay (with the program's own eager work between replays) gives the oracle's results."""
    from gpu_harness import Runner
    spec = (dict(in_dim=260, hidden=600, out_dim=260, seq_len=22, batch=13) if shape == "wide_batched_loop"
            else dict(in_dim=200, hidden=300, out_dim=200, seq_len=9, batch=1))
    case = ri.make_case(wdist=("normal", 0.2), bias_std=0.1, seed=31, **spec)
    ref = oracle.fwd_bptt(case)
    r = Runner(case)
    r.step()                                      # warm-up outside the capture (one-time attribute calls)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        r.forward(); r.loss_(); r.bptt()
    for rep in range(3):
        print(f"replay {rep}", flush=True)
        for g in r.grads.values():
            g.fill_(float("nan"))
        r.h_all.fill_(float("nan"))
        graph.replay()
        got = r.results()
        assert rnn.rnn_workspace_status(r.dims, r.ws) == 0
        compare(got, ref)
