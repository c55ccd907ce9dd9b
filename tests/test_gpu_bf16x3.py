"""GPU parity of the opt-in bf16 hi/lo split output layer (RNN_FLAG_BF16X3_OUTPUT) against the CPU
oracle, at the float32 path's tolerances: the shapes of the ordinary parity tests (ragged tiles,
T = 1, sizes that are multiples of nothing; the flag is ignored where the column-strip kernels
serve a short single sequence), plus shapes that span several 128x128 tiles and cut K."""
import numpy as np
import pytest

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import Runner, compare, grad_close, run_gpu
from test_gpu_parity import DENSE, LM, SMALL_CASES, make

pytestmark = pytest.mark.gpu

BF3 = rnn.FLAG_BF16X3_OUTPUT


@pytest.mark.parametrize("name", list(SMALL_CASES))
def test_small_cases_match_oracle_with_split_products(name):
    case = make(name)
    compare(run_gpu(case, BF3), oracle.fwd_bptt(case))


BIG_CASES = {
    # several tiles in every product; K of dV = N = 2560 rows is cut in two
    "lm_split_k": (600, 96, 600, 64, 40, dict(LM, wdist=("normal", 0.2), bias_std=0.1, with_h0=True)),
    # ragged everywhere: 333 = 2 tiles + 77, K pads 333 -> 352, 130 -> 160
    "lm_ragged_tiles": (333, 130, 333, 19, 17, dict(LM, wdist=("normal", 0.2), bias_std=0.1, with_dh_last=True)),
    "dense_mse_wide": (40, 200, 300, 33, 24, dict(DENSE, wdist=("normal_fan", None), bias_std=0.1)),
}


@pytest.mark.parametrize("name", list(BIG_CASES))
def test_multi_tile_cases_match_oracle(name):
    i, h, o, T, B, extra = BIG_CASES[name]
    case = ri.make_case(i, h, o, T, B, seed=900 + len(name), **extra)
    compare(run_gpu(case, BF3), oracle.fwd_bptt(case))


def test_accumulate_recompute_and_row_sums():
    """Accumulate mode through the bf16 products, logits recomputed inside rnn_bptt, and softmax
    rows that still sum to 1 within float32 rounding (dc sums to 0)."""
    i, h, o, T, B, extra = BIG_CASES["lm_ragged_tiles"]
    case = ri.make_case(i, h, o, T, B, seed=77, **extra)
    ref = oracle.fwd_bptt(case)
    r = Runner(case, BF3 | rnn.FLAG_BPTT_RECOMPUTE)
    r.forward()
    r.bptt()
    once = r.results()
    for k in ("dWx", "dWh", "db", "dV", "dc"):
        grad_close(k, once[k], ref[k])
    assert abs(once["dc"].sum()) < 1e-5
    r.set_flags(BF3 | rnn.FLAG_BPTT_RECOMPUTE | rnn.FLAG_ACCUMULATE)
    r.bptt()
    twice = r.results()
    for k in ("dWx", "dWh", "db", "dV", "dc"):
        grad_close("2x" + k, twice[k], 2.0 * ref[k])


def test_split_products_stay_close_to_the_float32_path_and_repeat_exactly():
    """The error bound the split rests on (each product term within 2^-16 relative): the split path
    must land far closer to the float32 path than the tolerance against the oracle asks, and give
    the same bits on every run (fixed summation order, no atomics)."""
    i, h, o, T, B, extra = BIG_CASES["lm_split_k"]
    case = ri.make_case(i, h, o, T, B, seed=901, **extra)
    f32 = run_gpu(case, 0)
    a = run_gpu(case, BF3)
    b = run_gpu(case, BF3)
    assert abs(a["loss"] - f32["loss"]) <= 2e-6 * abs(f32["loss"])
    for k in ("dV", "dc", "dWh", "dWx", "db"):
        assert np.array_equal(a[k], b[k]), k
        scale = np.abs(f32[k]).max()
        assert np.abs(a[k] - f32[k]).max() <= 5e-5 * scale, (k, np.abs(a[k] - f32[k]).max() / scale)
