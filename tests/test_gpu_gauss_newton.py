"""GPU parity of the Gauss-Newton-vector product (R-operator sweep + reverse sweep through the C
ABI) against the CPU oracle, on the shapes of the ordinary parity tests so that every family of
loop kernels runs the R-operator's forward sweep once."""
import numpy as np
import pytest
import torch

import oracle
import paper_1211_5590_amd as rnn
import rnn_inputs as ri
from gpu_harness import Runner, dev, grad_close
from test_gpu_parity import SMALL_CASES, make

pytestmark = pytest.mark.gpu

PNAMES = ("Wx", "Wh", "b", "V", "c")
GN_CASES = ["lm_tiny_config", "lm_ragged", "lm_T1", "lm_window_rnnlm_shape", "lm_small_batch_resident",
            "lm_hidden_300_two_groups", "lm_batch5_stepwise", "dense_batched_stepwise",
            "lm_batched_ragged_mfma", "lm_long_id_list_chunked_scatter", "lm_hidden_500",
            "lm_batched_mfma_shape", "dense_tanh_mse", "dense_ragged", "dense_T1_B1", "dense_input_ce",
            "tokens_tanh_mse"]


class GnRunner(Runner):
    def __init__(self, case, flags=0):
        super().__init__(case, flags)
        nbytes = rnn.rnn_gauss_newton_workspace_bytes(self.dims)
        self.gws = torch.full((nbytes + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        rnn.rnn_workspace_init(self.dims, self.gws)
        N = case["seq_len"] * case["batch"]
        self.Rz = torch.full((N, case["out_dim"]), float("nan"), device="cuda")
        self.out = {"d" + k: torch.full_like(v, float("nan")) for k, v in self.params.items()}

    def gauss_newton(self, gamma, metric, want_Rz=True):
        g = {k: dev(np.asarray(gamma[k], dtype=np.float32)) for k in PNAMES}
        rnn.rnn_gauss_newton_vec(self.dims, self.params, g, self.x, self.h_all, metric, self.out,
                                 self.Rz if want_Rz else None, self.gws)
        torch.cuda.synchronize()
        return {k: v.cpu().numpy() for k, v in self.out.items()}


def check(got, Rz, ref):
    grad_close("Rz", Rz, ref["Rz"])
    for k in PNAMES:
        grad_close("G" + k, got["d" + k], ref["G" + k])


@pytest.mark.parametrize("flags", [0, rnn.FLAG_REFERENCE_KERNELS], ids=["tuned", "reference"])
@pytest.mark.parametrize("name", GN_CASES)
def test_gauss_newton_vec_matches_oracle(name, flags):
    case = make(name)
    gamma = ri.make_direction(case, 7)
    r = GnRunner(case, flags)
    r.forward()
    got = r.gauss_newton(gamma, rnn.GN_METRIC_LOSS)
    ref = oracle.gauss_newton_vec(case, gamma, metric=0, want_Rz=True)
    check(got, r.Rz.cpu().numpy(), ref)
    if case["input_kind"] == ri.INPUT_TOKENS:   # rows of tokens that do not occur are exactly 0
        unseen = np.setdiff1d(np.arange(case["in_dim"]), np.unique(case["x"]))
        assert not got["dWx"][unseen].any()


@pytest.mark.parametrize("name", ["lm_ragged", "dense_tanh_mse", "lm_hidden_300_two_groups"])
def test_identity_metric_and_accumulate(name):
    case = make(name)
    gamma = ri.make_direction(case, 8)
    r = GnRunner(case)
    r.forward()
    got = r.gauss_newton(gamma, rnn.GN_METRIC_IDENTITY)
    ref = oracle.gauss_newton_vec(case, gamma, metric=1, want_Rz=True)
    check(got, r.Rz.cpu().numpy(), ref)
    # accumulate mode adds the same product a second time; Rz is not wanted this time
    r.set_flags(rnn.FLAG_ACCUMULATE)
    twice = r.gauss_newton(gamma, rnn.GN_METRIC_IDENTITY, want_Rz=False)
    for k in PNAMES:
        grad_close("2G" + k, twice["d" + k], 2.0 * got["d" + k].astype(np.float64))


def test_ordinary_calls_still_work_on_the_front_of_the_workspace():
    """forward -> loss -> gauss-newton -> loss -> bptt on the Gauss-Newton workspace."""
    case = make("lm_multi_tile")
    gamma = ri.make_direction(case, 9)
    r = GnRunner(case)
    r.ws = r.gws
    r.forward()
    r.loss_()
    got = r.gauss_newton(gamma, rnn.GN_METRIC_LOSS)
    check(got, r.Rz.cpu().numpy(), oracle.gauss_newton_vec(case, gamma, metric=0, want_Rz=True))
    r.loss_()
    r.bptt()
    from gpu_harness import compare
    compare(r.results(), oracle.fwd_bptt(case))


def test_symmetry_of_the_product_on_the_gpu():
    """<a, G b> = <b, G a> for the Gauss-Newton matrix (a property that holds at any size)."""
    case = make("lm_small_batch_resident")
    a, b = ri.make_direction(case, 10), ri.make_direction(case, 11)
    r = GnRunner(case)
    r.forward()
    Ga = r.gauss_newton(a, rnn.GN_METRIC_LOSS)
    Gb = r.gauss_newton(b, rnn.GN_METRIC_LOSS)
    ab = sum(float(np.vdot(np.asarray(a[k], np.float64), Gb["d" + k])) for k in PNAMES)
    ba = sum(float(np.vdot(np.asarray(b[k], np.float64), Ga["d" + k])) for k in PNAMES)
    assert abs(ab - ba) <= 1e-3 * max(abs(ab), abs(ba))
    aa = sum(float(np.vdot(np.asarray(a[k], np.float64), Ga["d" + k])) for k in PNAMES)
    assert aa >= 0.0


@pytest.mark.parametrize("name", ["lm_multi_tile", "lm_batched_wide_stepwise", "dense_tanh_mse", "lm_hidden_500",
                                  "lm_long_id_list_chunked_scatter"])
def test_gauss_newton_vec_with_the_split_products(name):
    """The same product with its five output-layer products on the bf16 matrix cores
    (RNN_FLAG_BF16X3_OUTPUT), at the same tolerances."""
    case = make(name)
    gamma = ri.make_direction(case, 12)
    r = GnRunner(case, rnn.FLAG_BF16X3_OUTPUT)
    r.forward()
    got = r.gauss_newton(gamma, rnn.GN_METRIC_LOSS)
    check(got, r.Rz.cpu().numpy(), oracle.gauss_newton_vec(case, gamma, metric=0, want_Rz=True))


_config_refs = {}


@pytest.mark.parametrize("flags", [0, rnn.FLAG_BF16X3_OUTPUT], ids=["f32", "bf16x3"])
@pytest.mark.parametrize("name,overrides", [("C3", {}), ("C4", dict(seq_len=6))], ids=["C3_full", "C4_T6"])
def test_gauss_newton_vec_at_configuration_size(name, overrides, flags):
    """The product at the widths bench.py times it on: the whole larger-hidden configuration
    (grid-resident loops, 64-row product tiles) and the minibatched one at reduced length
    (step-wise loops, batch 64, hidden 1024, vocabulary 10000; the oracle's product is one serial
    loop nest, about a minute for these 384 rows); the oracle runs once per shape."""
    case = ri.make_config(name, **overrides)
    gamma = ri.make_direction(case, 13)
    if name not in _config_refs:
        print(f"{name} oracle ...", flush=True)
        _config_refs[name] = oracle.gauss_newton_vec(case, gamma, metric=0, want_Rz=True)
    r = GnRunner(case, flags)
    r.forward()
    got = r.gauss_newton(gamma, rnn.GN_METRIC_LOSS)
    check(got, r.Rz.cpu().numpy(), _config_refs[name])
