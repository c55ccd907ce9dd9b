"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the
same seeded inputs.  Sizes span several tiles and ragged tails; edge cases cover T=1, B=1,
sizes that are multiples of nothing, carried state, incoming gradients, accumulate mode,
history-free forward and both kernel families (tuned and shape-agnostic)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import GRAD_NAMES, Runner, compare, grad_close, run_gpu

pytestmark = pytest.mark.gpu

LM = dict(input_kind=ri.INPUT_TOKENS, act=ri.ACT_SIGMOID, loss_kind=ri.LOSS_SOFTMAX_CE)
DENSE = dict(input_kind=ri.INPUT_DENSE, act=ri.ACT_TANH, loss_kind=ri.LOSS_LINEAR_MSE)

SMALL_CASES = {
    # name: (in_dim, hidden, out_dim, T, B, extra)
    "lm_tiny_config": (64, 16, 64, 32, 1, dict(LM, tokens="uniform")),
    "lm_ragged": (301, 37, 301, 7, 3, dict(LM, wdist=("normal", 0.5), bias_std=0.3)),
    "lm_T1": (50, 20, 50, 1, 5, dict(LM, wdist=("normal", 0.5), bias_std=0.3, with_h0=True)),
    "lm_state_and_incoming_grad": (130, 100, 130, 10, 1,
                                   dict(LM, wdist=("normal", 0.3), bias_std=0.2, with_h0=True, with_dh_last=True)),
    "lm_window_rnnlm_shape": (10000, 100, 10000, 10, 1, dict(LM, wdist=("normal", 0.1), with_h0=True)),
    "lm_short_ragged_single": (301, 37, 301, 7, 1, dict(LM, wdist=("normal", 0.5), bias_std=0.3,
                                                       with_h0=True, with_dh_last=True)),
    "lm_short_two_passes": (700, 60, 700, 29, 1, dict(LM, wdist=("normal", 0.3), bias_std=0.2)),
    "lm_small_batch_resident": (300, 132, 300, 9, 4, dict(LM, wdist=("normal", 0.2), bias_std=0.1, with_h0=True)),
    "lm_lanes16": (120, 24, 120, 11, 2, dict(LM, wdist=("normal", 0.4), bias_std=0.2, with_h0=True, with_dh_last=True)),
    "lm_hidden_300_two_groups": (400, 300, 400, 9, 1, dict(LM, wdist=("uniform", 0.08), bias_std=0.1, with_dh_last=True)),
    "lm_batch5_stepwise": (200, 70, 200, 6, 5, dict(LM, wdist=("normal", 0.3), bias_std=0.2, with_h0=True, with_dh_last=True)),
    "dense_batched_stepwise": (48, 160, 40, 12, 40, dict(DENSE, wdist=("normal_fan", None), bias_std=0.1, with_h0=True)),
    "lm_batched_wide_stepwise": (300, 320, 300, 5, 24, dict(LM, wdist=("normal_fan", None), bias_std=0.1, with_h0=True, with_dh_last=True)),
    # the per-XCD persistent loop (10 steps and more): ragged batch groups and column slices, both K widths,
    # the shortest sequence it takes, dense/tanh; and the same widths below 10 steps (one launch per step)
    "lm_xcd_ragged_groups": (260, 600, 260, 23, 13, dict(LM, wdist=("normal_fan", None), bias_std=0.1, with_h0=True, with_dh_last=True)),
    "dense_xcd_tanh": (48, 388, 40, 21, 61, dict(DENSE, wdist=("normal_fan", None), bias_std=0.1, with_h0=True, with_dh_last=True)),
    "lm_xcd_shortest": (120, 1024, 120, 10, 9, dict(LM, wdist=("normal_fan", None), with_h0=True)),
    "lm_wide_one_step": (120, 1024, 120, 1, 9, dict(LM, wdist=("normal_fan", None), with_h0=True)),
    "lm_wide_9_steps": (260, 600, 260, 9, 13, dict(LM, wdist=("normal_fan", None), bias_std=0.1, with_h0=True, with_dh_last=True)),
    "lm_batched_ragged_mfma": (150, 100, 150, 7, 21, dict(LM, wdist=("normal", 0.2), bias_std=0.2, with_h0=True, with_dh_last=True)),
    "lm_long_id_list_chunked_scatter": (500, 64, 500, 128, 20, dict(LM, wdist=("normal", 0.2), bias_std=0.1)),
    "lm_multi_tile": (1000, 132, 1000, 40, 4, dict(LM, wdist=("normal", 0.2), bias_std=0.1)),
    "lm_hidden_500": (700, 500, 700, 12, 1, dict(LM, wdist=("uniform", 0.05))),
    "lm_batched_mfma_shape": (512, 256, 512, 6, 32, dict(LM, wdist=("normal_fan", None), with_h0=True)),
    "dense_tanh_mse": (24, 64, 24, 9, 16, dict(DENSE, wdist=("normal_fan", None), bias_std=0.2,
                                                with_h0=True, with_dh_last=True)),
    "dense_ragged": (13, 29, 7, 5, 3, dict(DENSE, wdist=("normal", 0.4), bias_std=0.2)),
    "dense_T1_B1": (8, 12, 8, 1, 1, dict(DENSE, wdist=("normal", 0.4))),
    "dense_input_ce": (10, 33, 45, 6, 4, dict(input_kind=ri.INPUT_DENSE, act=ri.ACT_SIGMOID,
                                               loss_kind=ri.LOSS_SOFTMAX_CE, wdist=("normal", 0.4), bias_std=0.2)),
    "tokens_tanh_mse": (40, 18, 5, 6, 2, dict(input_kind=ri.INPUT_TOKENS, act=ri.ACT_TANH,
                                               loss_kind=ri.LOSS_LINEAR_MSE, wdist=("normal", 0.4), bias_std=0.2)),
}


def make(name, seed=100):
    i, h, o, T, B, extra = SMALL_CASES[name]
    return ri.make_case(i, h, o, T, B, seed=seed + len(name), **extra)


@pytest.mark.parametrize("flags", [0, rnn.FLAG_REFERENCE_KERNELS], ids=["tuned", "reference"])
@pytest.mark.parametrize("name", list(SMALL_CASES))
def test_small_cases_match_oracle(name, flags):
    case = make(name)
    print(f"case={name} flags={flags}", flush=True)
    ref = oracle.fwd_bptt(case)
    got = run_gpu(case, flags)
    compare(got, ref)
    if case["input_kind"] == 0:
        unseen = np.setdiff1d(np.arange(case["in_dim"]), np.unique(case["x"]))
        assert np.all(got["dWx"][unseen] == 0.0)          # exact zeros for tokens that do not occur


def test_softmax_rows_sum_to_one_and_zero_weight_closed_form():
    case = ri.make_case(10000, 20, 10000, 4, 2, seed=5, **LM)
    for k in ("Wx", "Wh", "b", "V", "c"):
        case[k][...] = 0
    got = run_gpu(case)
    assert abs(got["loss"] - np.log(10000.0)) <= 1e-4 * np.log(10000.0)
    counts = np.bincount(case["y"].reshape(-1), minlength=10000)
    dc = 1.0 / 10000 - counts / 8.0
    grad_close("dc", got["dc"], dc)
    grad_close("dV", got["dV"], 0.5 * np.broadcast_to(dc, (20, 10000)))
    assert np.all(got["dWx"] == 0) and np.all(got["dWh"] == 0) and np.all(got["db"] == 0)
    # rows of softmax sum to one  <=>  rows of dZ sum to zero  <=>  sum_k dc[k] = 0 (float32 noise)
    case = make("lm_multi_tile")
    got = run_gpu(case)
    assert abs(got["dc"].sum()) < 1e-5
    assert np.max(np.abs(got["dV"].sum(1))) < 1e-5
    np.testing.assert_allclose(got["dWx"].sum(0), got["db"], atol=1e-5)


def test_accumulate_mode_adds_and_leaves_unseen_rows_alone():
    case = make("lm_ragged")
    ref = oracle.fwd_bptt(case)
    r = Runner(case, rnn.FLAG_ACCUMULATE)
    for k, g in r.grads.items():
        g.fill_(1.0)
    r.step()
    got = r.results()
    for k in GRAD_NAMES:
        grad_close(k, got[k] - 1.0, ref[k], rtol=2e-3)
    unseen = np.setdiff1d(np.arange(case["in_dim"]), np.unique(case["x"]))
    assert np.all(got["dWx"][unseen] == 1.0)


def test_bptt_recompute_flag_needs_no_prior_loss_call():
    case = make("lm_multi_tile")
    ref = oracle.fwd_bptt(case)
    r = Runner(case, rnn.FLAG_BPTT_RECOMPUTE)
    r.forward()
    r.bptt()
    got = r.results()
    for k in GRAD_NAMES:
        grad_close(k, got[k], ref[k])


@pytest.mark.parametrize("name", ["lm_state_and_incoming_grad", "dense_tanh_mse", "lm_hidden_500"])
def test_history_free_forward_returns_last_state(name):
    case = make(name)
    ref = oracle.forward(case)
    r = Runner(case, keep_history=False)
    r.forward()
    torch.cuda.synchronize()
    assert np.max(np.abs(r.h_last.cpu().numpy() - ref[-1])) <= 2e-5


def test_results_are_bit_identical_run_to_run():
    case = make("lm_multi_tile")
    r = Runner(case)
    r.step()
    first = r.results()
    for _ in range(5):
        r.step()
        again = r.results()
        for k in GRAD_NAMES + ("h_all", "dh0"):
            assert np.array_equal(first[k], again[k]), k
        assert first["loss"] == again["loss"]


@pytest.mark.parametrize("name", ["lm_hidden_500", "lm_hidden_300_two_groups", "lm_batched_wide_stepwise", "lm_xcd_ragged_groups",
                                  "lm_batched_mfma_shape"])
def test_multi_workgroup_loops_repeat_exactly_100_times(name):
    """A broken exchange or barrier between the workgroups of a time loop shows up as run-to-run
    noise: 100 repetitions of forward + BPTT must give the same bits every time."""
    case = make(name)
    r = Runner(case)
    r.step()
    first = {k: v.clone() for k, v in r.grads.items()}
    h_first, dh0_first = r.h_all.clone(), r.dh0.clone()
    for _ in range(100):
        r.forward(); r.loss_(); r.bptt()
        assert torch.equal(r.h_all, h_first)
        assert torch.equal(r.dh0, dh0_first)
        for k, v in r.grads.items():
            assert torch.equal(v, first[k]), k
    assert rnn.rnn_workspace_status(r.dims, r.ws) == 0


def test_two_windows_chain_state_forward_and_gradient_backward():
    full = ri.make_case(200, 48, 200, 12, 2, seed=77, wdist=("normal", 0.3), bias_std=0.1, **LM)
    ref = oracle.fwd_bptt(full)
    halves = []
    for w in range(2):
        q = dict(full); q["seq_len"] = 6
        q["x"], q["y"] = full["x"][6 * w:6 * w + 6], full["y"][6 * w:6 * w + 6]
        halves.append(q)
    ra, rb = Runner(halves[0]), Runner(halves[1])
    ra.forward(); ra.loss_()
    rb.h0 = ra.h_last
    rb.forward(); rb.loss_(); rb.bptt()
    ra.dh_last = rb.dh0
    ra.bptt()
    ga, gb = ra.results(), rb.results()
    assert np.max(np.abs(np.concatenate([ga["h_all"], gb["h_all"][1:]]) - ref["h_all"])) <= 2e-5
    for k in GRAD_NAMES:
        grad_close(k, 0.5 * (ga[k] + gb[k]), ref[k])
    assert abs(0.5 * (ga["loss"] + gb["loss"]) - ref["loss"]) <= 1e-4 * ref["loss"]


def test_variant_names_and_clean_status_word():
    expect = {"lm_window_rnnlm_shape": "wg_resident", "lm_hidden_500": "grid_resident",
              "lm_batched_mfma_shape": "batch_mfma"}
    for name, want in expect.items():
        case = make(name)
        r = Runner(case)
        assert rnn.rnn_recurrence_variant(r.dims) == want
        rnn.rnn_workspace_init(r.dims, r.ws)
        r.step()
        assert rnn.rnn_workspace_status(r.dims, r.ws) == 0


def test_accumulate_mode_on_the_short_sequence_path():
    case = make("lm_short_ragged_single")
    ref = oracle.fwd_bptt(case)
    r = Runner(case, rnn.FLAG_ACCUMULATE)
    for k, g in r.grads.items():
        g.fill_(1.0)
    r.step()
    got = r.results()
    for k in GRAD_NAMES:
        grad_close(k, got[k] - 1.0, ref[k], rtol=2e-3)
    unseen = np.setdiff1d(np.arange(case["in_dim"]), np.unique(case["x"]))
    assert np.all(got["dWx"][unseen] == 1.0)


def test_check_tokens_counts_out_of_range_ids():
    ids = torch.tensor([0, 5, 9, 10, -1, 3, 99], dtype=torch.int32, device="cuda")
    bad = torch.full((1,), 123, dtype=torch.int32, device="cuda")
    rnn.rnn_check_tokens(ids, ids.numel(), 10, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 3


def test_calls_are_asynchronous_on_a_side_stream():
    case = make("lm_multi_tile")
    ref = oracle.fwd_bptt(case)
    r = Runner(case)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r.forward(); r.loss_(); r.bptt()
    side.synchronize()
    compare(r.results(), ref)
