"""Parity at the sizes where the dispatcher changes kernel family: hidden sizes just below and
above 128, 256, 512 and 1024 against batch sizes just below and above 4 and 64 (one workgroup,
several workgroups, batched matrix-core loop, the one-launch wide loop, one launch per step), with
short windows, both activations, token and dense inputs, initial states and incoming gradients."""
import numpy as np
import pytest

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import Runner, compare

pytestmark = pytest.mark.gpu

HIDDEN = (128, 129, 256, 257, 512, 516, 1020, 1024, 1028)
BATCH = (1, 4, 5, 64, 65)


@pytest.mark.parametrize("H", HIDDEN)
def test_every_batch_size_at_this_hidden_size(H):
    rng = np.random.default_rng(H)
    seen = set()
    for n, B in enumerate(BATCH):
        T = int(rng.choice([1, 2, 3, 5, 9]))
        NV = int(rng.choice([64, 130, 200]))
        dense = n == 3
        kw = dict(in_dim=24 if dense else NV, hidden=H, out_dim=20 if dense else NV, seq_len=T, batch=B,
                  act=int(rng.integers(0, 2)), with_h0=bool(n % 2), with_dh_last=n % 3 == 0,
                  wdist=("normal", 0.5 / np.sqrt(H)), bias_std=0.1, seed=1000 + 7 * H + n)
        if dense:
            kw.update(input_kind=ri.INPUT_DENSE, loss_kind=ri.LOSS_LINEAR_MSE)
        case = ri.make_case(**kw)
        r = Runner(case)
        variant = rnn.rnn_recurrence_variant(r.dims)
        seen.add(variant)
        print(f"H={H} B={B} T={T} NV={NV} dense={dense} variant={variant}", flush=True)
        r.step()
        assert rnn.rnn_workspace_status(r.dims, r.ws) == 0
        compare(r.results(), oracle.fwd_bptt(case, h0=case.get("h0"), dh_last=case.get("dh_last")))
    assert len(seen) >= 2, seen        # every hidden size crosses at least one family boundary over these batches


@pytest.mark.parametrize("H", (260, 512, 516, 1020, 1024))
def test_the_one_launch_wide_loop_at_its_edges(H):
    """Batch 5 and 64 (the smallest and the largest the one-launch wide loop takes), 10 steps (its
    shortest sequence) and 9 (one launch per step), batch 65 (beyond it)."""
    for n, (B, T, want) in enumerate(((5, 10, "xcd_mfma"), (64, 21, "xcd_mfma"), (64, 9, "step_mfma"),
                                      (65, 20, "step_mfma"))):
        case = ri.make_case(in_dim=90, hidden=H, out_dim=70, seq_len=T, batch=B, act=n % 2, with_h0=bool(n % 2),
                            with_dh_last=n >= 2, wdist=("normal", 0.5 / np.sqrt(H)), bias_std=0.1, seed=9000 + 11 * H + n)
        r = Runner(case)
        variant = rnn.rnn_recurrence_variant(r.dims)
        print(f"H={H} B={B} T={T} variant={variant}", flush=True)
        assert variant == want
        r.step()
        assert rnn.rnn_workspace_status(r.dims, r.ws) == 0
        compare(r.results(), oracle.fwd_bptt(case, h0=case.get("h0"), dh_last=case.get("dh_last")))
