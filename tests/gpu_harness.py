"""Helpers for the GPU parity tests: run one window through the C ABI and compare with the oracle.

Tolerances (float32 path against the float64 oracle): loss relative 1e-4; every gradient tensor
max|diff| <= 1e-3 * max|ref| and ||diff||_2 <= 1e-3 * ||ref||_2; hidden states absolute 2e-5
(they live in (-1,1)).
"""
from __future__ import annotations

import numpy as np
import torch

import paper_1211_5590_amd as rnn

LOSS_RTOL = 1e-4
GRAD_RTOL = 1e-3
H_ATOL = 2e-5
GRAD_NAMES = ("dWx", "dWh", "db", "dV", "dc")


def dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class Runner:
    """Device buffers of one problem; forward/loss/bptt through the C ABI."""

    def __init__(self, case, flags=0, keep_history=True):
        self.case = case
        self.dims = rnn.Dims.of(case, flags)
        T, B, H = case["seq_len"], case["batch"], case["hidden"]
        self.params = {k: dev(case[k]) for k in ("Wx", "Wh", "b", "V", "c")}
        self.x = dev(case["x"]) if case["input_kind"] == 0 else dev(case["X"])
        self.y = dev(case["y"]) if case["loss_kind"] == 0 else dev(case["Y"])
        self.h0 = dev(case.get("h0"))
        self.dh_last = dev(case.get("dh_last"))
        self.h_all = torch.full((T + 1, B, H), float("nan"), device="cuda") if keep_history else None
        self.h_last = torch.full((B, H), float("nan"), device="cuda")
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.grads = {"d" + k: torch.full_like(v, float("nan")) for k, v in self.params.items()}
        self.dh0 = torch.full((B, H), float("nan"), device="cuda")
        nbytes = rnn.rnn_workspace_bytes(self.dims)
        # 0xA5 fill: a workspace is arbitrary memory until rnn_workspace_init has run on it
        self.ws = torch.full((nbytes + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        rnn.rnn_workspace_init(self.dims, self.ws)

    def set_flags(self, flags):
        self.dims.flags = flags

    def forward(self):
        rnn.rnn_forward(self.dims, self.params, self.x, self.h0, self.h_all, self.h_last, self.ws)

    def loss_(self):
        rnn.rnn_loss(self.dims, self.params, self.h_all, self.y, self.loss, self.ws)

    def bptt(self, want_dh0=True):
        rnn.rnn_bptt(self.dims, self.params, self.x, self.y, self.h_all, self.dh_last, self.grads,
                     self.dh0 if want_dh0 else None, self.ws)

    def step(self):
        self.forward()
        self.loss_()
        self.bptt()
        torch.cuda.synchronize()

    def results(self):
        torch.cuda.synchronize()
        out = {k: v.cpu().numpy() for k, v in self.grads.items()}
        out["loss"] = float(self.loss.item())
        out["h_all"] = self.h_all.cpu().numpy() if self.h_all is not None else None
        out["h_last"] = self.h_last.cpu().numpy()
        out["dh0"] = self.dh0.cpu().numpy()
        return out


def run_gpu(case, flags=0):
    r = Runner(case, flags)
    r.step()
    return r.results()


def grad_close(name, got, ref, rtol=GRAD_RTOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    diff = np.abs(got - ref)
    mx, scale = diff.max(), np.abs(ref).max()
    assert mx <= rtol * scale + 1e-30, f"{name}: max|diff| {mx:.3e} > {rtol} * {scale:.3e}"
    l2, l2ref = np.linalg.norm(got - ref), np.linalg.norm(ref)
    assert l2 <= rtol * l2ref + 1e-30, f"{name}: l2 {l2:.3e} > {rtol} * {l2ref:.3e}"


def compare(got, ref, check_dh0=True):
    """got: Runner.results(); ref: oracle.fwd_bptt() dict."""
    assert abs(got["loss"] - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"]), (got["loss"], ref["loss"])
    if got.get("h_all") is not None:
        assert np.max(np.abs(got["h_all"] - ref["h_all"])) <= H_ATOL
    assert np.max(np.abs(got["h_last"] - ref["h_all"][-1])) <= H_ATOL
    for k in GRAD_NAMES:
        grad_close(k, got[k], ref[k])
    if check_dh0:
        grad_close("dh0", got["dh0"], ref["dh0"])
