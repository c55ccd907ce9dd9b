#!/usr/bin/env python3
"""Benchmark of the Elman-RNN training path (forward recurrence -> output layer + loss -> BPTT).

One "step" is one pass of the whole path (rnn_forward -> rnn_loss -> rnn_bptt) over one batch of
synthetic input.  The headline workload is C4, the largest configuration (hidden 1024, vocabulary
10000, 256 steps, batch 64: 16384 tokens per step); the others are reported under `per_config`
and, in short, under `summary`:
  C2 (the paper's benchmark shape: batch 1, vocabulary-sized input and output layers): the
     100000-token Zipf stream as 10000 dependent truncated-BPTT windows of 10 steps; every window
     is one rnn_window call (forward, loss and BPTT of the window in one launch; the same outputs
     as the three calls, whose timing is reported beside it) with the hidden state carried, in
     stream order, exactly as if an optimiser step sat between windows; plus the same stream in
     one rnn_train_stream launch with an SGD update per window.
  C1, C3, C5: one window of the named configuration.
Prints ONE JSON line.  Inputs are resident in HBM before the timed region starts.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
FP32_MFMA_PEAK_TFLOPS = 157.3
BF16_MFMA_PEAK_TFLOPS = 2500.0   # dense bf16 matrix rate
N_CU = 256
LDS_PEAK_GBS_PER_CU = 256 * 2.4   # 16-byte LDS reads: 256 B/clk per compute unit at 2.4 GHz


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--windows", type=int, default=None, help="override the number of C2 windows")
    ap.add_argument("--others", default="C1,C2,C3,C5",
                    help="comma list of further configurations reported under 'per_config' ('none' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--three-calls", action="store_true",
                    help="time rnn_forward -> rnn_loss -> rnn_bptt even where rnn_window serves the shape")
    ap.add_argument("--no-train-stream", action="store_true",
                    help="skip the single-launch SGD driver leg of the headline workload")
    ap.add_argument("--only-mlp", action="store_true",
                    help="run only the feed-forward classifier workloads and print their JSON line")
    ap.add_argument("--no-mlp", action="store_true",
                    help="skip the feed-forward classifier workloads (the paper's second benchmark)")
    ap.add_argument("--cpu-seconds", type=float, default=30.0,
                    help="CPU budget of the headline oracle sample (the other configurations get at most 15 s each)")
    ap.add_argument("--reference-kernels", action="store_true")
    ap.add_argument("--bf16x3", action="store_true",
                    help="opt-in output layer on the bf16 matrix cores (hi/lo split operands, three products)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run a plain 64 MiB device copy (known traffic) to scale profiler counters by")
    return ap.parse_args()


class Workload:
    """Device-resident buffers and pre-marshalled C calls of one configuration."""

    def __init__(self, name, flags=0, windows=None, three_calls=False):
        import numpy as np
        import torch
        import paper_1211_5590_amd as rnn
        import rnn_inputs as ri
        self.rnn, self.torch, self.name = rnn, torch, name
        over = {}
        if windows is not None and ri.CONFIGS[name]["windows"] > 1:
            over["windows"] = windows
        case = ri.make_config(name, **over)
        self.case = case
        self.T, self.B, self.H = case["seq_len"], case["batch"], case["hidden"]
        self.windows = case["windows"]
        self.dims = rnn.Dims.of(case, flags)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.p = {k: dev(case[k]) for k in ("Wx", "Wh", "b", "V", "c")}
        self.x = dev(case["x"] if case["input_kind"] == 0 else case["X"])
        self.y = dev(case["y"] if case["loss_kind"] == 0 else case["Y"])
        self.g = {"d" + k: torch.zeros_like(v) for k, v in self.p.items()}
        self.h_all = torch.zeros((self.T + 1, self.B, self.H), device="cuda")
        self.carry = torch.zeros((2, self.B, self.H), device="cuda")
        self.loss = torch.zeros((max(self.windows, 1),), device="cuda")
        self.ws = torch.empty(rnn.rnn_workspace_bytes(self.dims), dtype=torch.uint8, device="cuda")
        rnn.rnn_workspace_init(self.dims, self.ws)
        # one launch per window (rnn_window) where its one-launch kernel serves the shape, else the three calls
        self.fused = False
        if (not three_calls and not flags and case["input_kind"] == 0 and case["loss_kind"] == 0
                and rnn.rnn_window_one_launch(self.dims)):
            try:
                self.wws = torch.empty(rnn.rnn_window_workspace_bytes(self.dims), dtype=torch.uint8, device="cuda")
                rnn.rnn_window_workspace_init(self.dims, self.wws)
                self.fused = True
            except rnn.RnnError:
                pass
        # pre-marshalled arguments: plain ints and ctypes structs, no per-call Python objects
        self.L = rnn.lib()
        self.P = rnn.Params(*[self.p[k].data_ptr() for k in ("Wx", "Wh", "b", "V", "c")])
        self.G = rnn.Grads(*[self.g["d" + k].data_ptr() for k in ("Wx", "Wh", "b", "V", "c")])
        self.x_stride = self.x[0].numel() * self.x.element_size() * self.T
        self.y_stride = self.y[0].numel() * self.y.element_size() * self.T
        case["_bf16x3"] = bool(flags & rnn.FLAG_BF16X3_OUTPUT)
        case["_name"] = name + ("B" if case["_bf16x3"] else "")   # key of the counter-based traffic table
        case["_variant"] = rnn.rnn_recurrence_variant(self.dims)
        case["_workgroups"] = rnn.rnn_recurrence_workgroups(self.dims)
        self.tokens_per_step = self.T * self.B * self.windows
        self.timesteps_per_step = self.T * self.windows

    def step(self, stream):
        """All windows of the stream, in order, on `stream` (a raw hipStream_t as int)."""
        L, d, P, G = self.L, ctypes.byref(self.dims), ctypes.byref(self.P), ctypes.byref(self.G)
        ws, wb = self.ws.data_ptr(), self.ws.numel()
        h_all = self.h_all.data_ptr()
        xb, yb, lb = self.x.data_ptr(), self.y.data_ptr(), self.loss.data_ptr()
        c0, c1 = self.carry[0].data_ptr(), self.carry[1].data_ptr()
        fwd, loss, bptt = L.rnn_forward, L.rnn_loss, L.rnn_bptt
        if self.fused:
            win, wws, wwb = L.rnn_window, self.wws.data_ptr(), self.wws.numel()
            for w in range(self.windows):
                h0 = None if w == 0 else (c1 if w & 1 else c0)
                rc = win(d, P, xb + w * self.x_stride, yb + w * self.y_stride, h0, None, None,
                         c0 if w & 1 else c1, lb + 4 * w, G, None, wws, wwb, stream)
                if rc:
                    raise RuntimeError(f"rnn_window failed in window {w}: {rc}")
            return
        for w in range(self.windows):
            x, y = xb + w * self.x_stride, yb + w * self.y_stride
            h0 = None if w == 0 else (c1 if w & 1 else c0)
            hl = c0 if w & 1 else c1
            rc = fwd(d, P, x, h0, h_all, hl, ws, wb, stream)
            rc |= loss(d, P, h_all, y, lb + 4 * w, ws, wb, stream)
            rc |= bptt(d, P, x, y, h_all, None, G, None, ws, wb, stream)
            if rc:
                raise RuntimeError(f"rnn call failed in window {w}: {rc}")

    def time_steps(self, steps, warmup):
        torch = self.torch
        stream = torch.cuda.current_stream().cuda_stream
        for _ in range(warmup):
            self.step(stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            self.step(stream)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) / 1e3

    def profile(self, steps=1):
        """Per-kernel HIP-event timing of `steps` further steps (events perturb throughput a
        little, so this runs after the timed region, on the same stream)."""
        stream = self.torch.cuda.current_stream().cuda_stream
        self.torch.cuda.synchronize()
        self.rnn.rnn_profile_begin(1 << 20)
        for _ in range(steps):
            self.step(stream)
        prof = self.rnn.rnn_profile_end()
        self.case["_skinny"] = "skinny_logits" in prof   # short-sequence output layer in use
        # An event pair with nothing between it does not read zero: measure that bracket cost
        # on the same stream and take it off every kernel's average (raw value kept).
        torch = self.torch
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                 for _ in range(64)]
        for a, b in pairs:
            a.record(); b.record()
        torch.cuda.synchronize()
        gaps = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
        bracket_us = gaps[len(gaps) // 2]
        out = {}
        for k, (c, ms) in prof.items():
            raw = 1e3 * ms / c
            avg = max(raw - bracket_us, 0.05 * raw)
            out[k] = dict(launches=c, total_ms=avg * c / 1e3, avg_us=avg, avg_us_raw=raw)
        self.bracket_us = bracket_us
        return out


def algorithmic_work(kernel, c):
    """Algorithmic (bytes, flops) of ONE launch of `kernel` for configuration dict `c`: what the
    method must move/compute (operands read once, results written once), not what the
    implementation happens to move.  None for bookkeeping kernels."""
    N, H, O, I = c["seq_len"] * c["batch"], c["hidden"], c["out_dim"], c["in_dim"]
    T, B = c["seq_len"], c["batch"]
    f = 4
    tokens = c["input_kind"] == 0
    table = {
        # hoisted matrix-matrix products
        "gemm_logits": (f * (N * H + H * O + N * O), 2.0 * N * H * O),      # Z = Hs V + c
        "gemm_dV": (f * (N * H + N * O + H * O), 2.0 * N * H * O),          # dV = Hs^T dZ
        "gemm_G": (f * (N * O + H * O + N * H), 2.0 * N * H * O),           # G = dZ V^T
        "gemm_dWh": (f * (2 * N * H + H * H), 2.0 * N * H * H),             # dWh = Delta^T Hprev
        "gemm_U": (f * (N * I + H * I + N * H), 2.0 * N * H * I),           # U = X Wx^T + b
        "gemm_dWx": (f * (N * H + N * I + H * I), 2.0 * N * H * I),         # dWx = Delta^T X
        # element-wise / row-wise passes over the logits
        "ce_row_stats": (f * N * O, 3.0 * N * O),
        "mse_row_loss": (2 * f * N * O, 3.0 * N * O),
        "dz": ((3 if not c["loss_kind"] == 0 else 2) * f * N * O, 3.0 * N * O),
        "dwx_tokens": (f * (N * H + I * H), 1.0 * N * H),
        # float32 matrix in, bf16 hi/lo planes out (row-major and transposed: 4 bytes per element each);
        # per step: h, V and dZ
        "split_bf16": (f * 3 * (N * H + H * O + N * O) / 3.0, 6.0 * (N * H + H * O + N * O) / 3.0),
        # time loops: the recurrent matrix once per launch, one state row in and out per step
        "rec_fwd": None, "rec_bwd": None,
        # short-sequence output layer (column strips): V in, Z out, and the strips' shares of the
        # softmax part of G (a second contraction with the same strip of V)
        "skinny_logits": (f * (H * O + N * O + N * H), 4.0 * N * H * O),
        # whole window in one launch: V and Wh in, dV, dWh and the dense dWx out (logits and dZ
        # never leave the chip); logits, shares of G and dV are three contractions with V-sized
        # operands, the loops and dWh three with Wh-sized ones
        "window": (f * (2 * H * O + 2 * H * H + I * H + 3 * N * H + 2 * O), 6.0 * N * H * O + 6.0 * N * H * H),
    }
    variant = c.get("_variant", "")
    if variant == "step_mfma":      # one launch = one step: matrix + state in, state out
        table["rec_fwd"] = (f * (H * H + 3 * B * H), 2.0 * B * H * H)
        table["rec_bwd"] = (f * (H * H + 4 * B * H), 2.0 * B * H * H)
    else:                           # one launch = all T steps
        table["rec_fwd"] = (f * (H * H + 2 * N * H + (0 if tokens else N * H)), 2.0 * N * H * H)
        table["rec_bwd"] = (f * (H * H + 3 * N * H), 2.0 * N * H * H)
        if c.get("_skinny"):        # the same launch runs the backward strips and the small
            nb, nf = table["rec_bwd"]   # weight gradients: Z in, dV out, dWx zero fill, dWh out
            table["rec_bwd"] = (nb + f * (N * O + H * O + I * H + H * H), nf + 2.0 * N * H * O + 2.0 * N * H * H)
    return table.get(kernel)


RIDGE = FP32_MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # flop per byte


def on_chip_roofline(name, us, c):
    """The time loops keep the recurrent matrix on chip, so HBM says little about them: their
    own ceiling is the on-chip rate of the compute units they occupy (one workgroup per unit).
    Weights resident in LDS/registers and used once per step (batch rows do not share a
    workgroup): LDS read bandwidth of those units against T*B*H*H*4 bytes per launch.
    Matrix-core loops: the fp32 MFMA rate of those units against 2*rows*H*H flop per launch."""
    if name not in ("rec_fwd", "rec_bwd"):
        return None
    T, B, H = c["seq_len"], c["batch"], c["hidden"]
    variant, wgs = c.get("_variant", ""), c.get("_workgroups", 0)
    n_cu = min(N_CU, wgs)
    sec = us * 1e-6
    if n_cu <= 0 or variant == "reference":
        return None
    if variant in ("wg_resident", "grid_resident"):
        nbytes = 4.0 * T * B * H * H
        peak = n_cu * LDS_PEAK_GBS_PER_CU
        ach = nbytes / sec / 1e9
        return dict(bound="lds", n_cu=n_cu, achieved=ach, peak=peak, unit="GB/s", frac=ach / peak,
                    on_chip_bytes=nbytes)
    rows = B if variant == "step_mfma" else T * B      # one launch = one step, or all of them
    flops = 2.0 * rows * H * H
    peak = FP32_MFMA_PEAK_TFLOPS * n_cu / N_CU
    ach = flops / sec / 1e12
    return dict(bound="mfma", n_cu=n_cu, achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak,
                flops=flops)


MEASURED = {}   # filled by main(): the chip's measured ceilings (rnn_measure_ceilings)


def roofline_entry(name, prof, case):
    r = _roofline_entry(name, prof, case)
    if MEASURED and r.get("achieved") is not None:
        key = ("hbm_copy_GBps" if r["bound"] == "hbm" else
               "mfma_bf16_TFLOPs" if r.get("dtype", "").startswith("bf16") else "mfma_f32_TFLOPs")
        peak = max(MEASURED[key], MEASURED["hbm_read_GBps"]) if key == "hbm_copy_GBps" else MEASURED[key]
        r["peak_measured"] = peak
        r["frac_measured"] = (r.get("frac_executed", r["frac"]) * r["peak"]) / peak
    oc = on_chip_roofline(name, prof[name]["avg_us"], case)
    if oc:
        r["on_chip"] = oc
    return r


def _roofline_entry(name, prof, case):
    work = algorithmic_work(name, case)
    us = prof[name]["avg_us"]
    if work is None:
        return dict(kernel=name, bound=None, achieved=None, peak=None, unit=None, frac=None,
                    traffic=None, avg_us=us)
    nbytes, flops = work
    sec = us * 1e-6
    if case.get("_bf16x3") and name in ("gemm_logits", "gemm_dV", "gemm_G"):
        # hi/lo split operands: three bf16 matrix instructions per product term, so the matrix
        # cores execute 3x the algorithmic flops; both rates are stated against the bf16 peak
        ach = flops / sec / 1e12
        return dict(kernel=name, bound="mfma", achieved=ach, peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=ach / BF16_MFMA_PEAK_TFLOPS, traffic=None, avg_us=us, algorithmic_flops=flops,
                    dtype="bf16 hi/lo split, f32 accumulate", executed_flops=3.0 * flops,
                    frac_executed=3.0 * ach / BF16_MFMA_PEAK_TFLOPS)
    if flops / nbytes >= RIDGE:   # above the ridge point: arithmetic bound
        ach = flops / sec / 1e12
        # the batch-1..4 loops multiply on the vector ALUs (same fp32 peak as the matrix cores)
        valu = name in ("rec_fwd", "rec_bwd") and case.get("_variant") in ("wg_resident", "grid_resident")
        return dict(kernel=name, bound="alu" if valu else "mfma", achieved=ach, peak=FP32_MFMA_PEAK_TFLOPS,
                    unit="TFLOP/s", frac=ach / FP32_MFMA_PEAK_TFLOPS, traffic=None, avg_us=us,
                    algorithmic_flops=flops)
    ach = nbytes / sec / 1e9
    return dict(kernel=name, bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                frac=ach / HBM_PEAK_GBS, traffic=None, avg_us=us, algorithmic_bytes=nbytes)


def roofline_of(prof, case):
    """Roofline entry of the dominant kernel (largest total time in the profile pass), with the
    counter-measured HBM traffic per launch when profiles/hbm_traffic.json has it."""
    if not prof:
        return None
    name = max(prof, key=lambda k: prof[k]["total_ms"])
    r = roofline_entry(name, prof, case)
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
            t = json.load(fh).get(case.get("_name", ""), {}).get(name)
        if t:
            r["traffic"] = t["bytes_per_launch"]
            r["traffic_source"] = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                   "command, scaled by a 64 MiB copy; committed, not measured in this run")
    except (OSError, ValueError):
        pass
    return r


def all_rooflines(prof, case):
    return [roofline_entry(k, prof, case) for k in sorted(prof, key=lambda k: -prof[k]["total_ms"])
            if algorithmic_work(k, case) is not None]


def cpu_baseline(name, budget_s, one_thread_row=True):
    """The oracle as it stands, timed on the host cores (as many threads as it is set to use) over a
    bounded sample of the workload: the whole configuration when a short probe says that fits the
    budget, else the same widths at a shorter sequence, which the `sample` field states."""
    import oracle
    import rnn_inputs as ri
    cores = oracle.num_threads()
    cfg = ri.CONFIGS[name]
    if cfg["windows"] > 1:
        cap = min(cfg["windows"], 4096)
        case = ri.make_config(name, windows=cap)

        def run(limit_s):
            t0 = time.perf_counter()
            h, done = None, 0
            while done < cap and (done < 4 or time.perf_counter() - t0 < limit_s):
                r = oracle.fwd_bptt(ri.window(case, done), h0=h)
                h = r["h_all"][-1]
                done += 1
            return done, time.perf_counter() - t0
        done, dt = run(budget_s)
        tokens = done * cfg["seq_len"] * cfg["batch"]
        out = dict(value=tokens / dt, unit="tokens/s", cores=cores, kind="oracle", seconds=dt,
                   sample=f"first {done} windows of the stream (state carried), forward+loss+BPTT each")
        if one_thread_row and cores > 1:
            oracle.set_num_threads(1)
            try:
                done1, dt1 = run(min(3.0, budget_s))
            finally:
                oracle.set_num_threads(cores)
            out["one_thread"] = dict(value=done1 * cfg["seq_len"] * cfg["batch"] / dt1, unit="tokens/s", cores=1,
                                     sample=f"first {done1} windows", seconds=dt1)
        return out
    T, B = cfg["seq_len"], cfg["batch"]
    # probe: a few steps of the full batch give the oracle's seconds per row on these threads
    Tp = min(T, 2 if B >= 16 else 16)
    probe = ri.make_config(name, seq_len=Tp)
    t0 = time.perf_counter()
    oracle.fwd_bptt(probe)
    per_row = (time.perf_counter() - t0) / (Tp * B)
    rows = max(1.0, budget_s / per_row)
    while T * B > rows and T > 1:
        T = max(1, T // 2)
    case = probe if T == Tp else ri.make_config(name, seq_len=T)
    t0 = time.perf_counter()
    oracle.fwd_bptt(case)
    dt = time.perf_counter() - t0
    whole = T == cfg["seq_len"]
    sample = ("the whole configuration, once" if whole else
              f"one window with seq_len {T} instead of {cfg['seq_len']} (same widths and batch)") + ", forward+loss+BPTT"
    out = dict(value=T * B / dt, unit="tokens/s", cores=cores, kind="oracle", sample=sample, seconds=dt)
    if one_thread_row and cores > 1:
        oracle.set_num_threads(1)
        try:
            one = cpu_baseline(name, min(6.0, budget_s), one_thread_row=False)
        finally:
            oracle.set_num_threads(cores)
        out["one_thread"] = {k: one[k] for k in ("value", "unit", "cores", "sample", "seconds")}
    return out


def train_stream_leg(windows, reps=3, lr=0.1):
    """The whole C2 stream in ONE call of rnn_train_stream (persistent launch, SGD after every
    window): time of the launch from HIP events on its stream, tokens/s, and what the launch does
    per window against the matrix-core rate of the compute units it occupies."""
    import numpy as np
    import torch
    import paper_1211_5590_amd as rnn
    import rnn_inputs as ri
    case = ri.make_config("C2", **({"windows": windows} if windows else {}))
    W, T, H, NV = case["windows"], case["seq_len"], case["hidden"], case["out_dim"]
    dims = rnn.Dims.of(case)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    p0 = {k: dev(case[k]) for k in ("Wx", "Wh", "b", "V", "c")}
    ids = dev(ri.stream_ids(case).reshape(-1))
    losses = torch.zeros(W, device="cuda")
    h_last = torch.zeros(H, device="cuda")
    ws = torch.empty(rnn.rnn_train_stream_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
    times = []
    for rep in range(reps + 1):                      # first repetition is the warm-up
        p = {k: v.clone() for k, v in p0.items()}
        torch.cuda.synchronize()
        rnn.rnn_profile_begin(16)
        rnn.rnn_train_stream(dims, p, ids, W, lr, None, h_last, losses, ws)
        prof = rnn.rnn_profile_end()
        assert rnn.rnn_train_stream_status(ws) == 0, "a bounded wait expired"
        if rep:
            times.append(prof["train_stream"][1] / 1e3)
    sec = sorted(times)[len(times) // 2]
    strips = (NV + 127) // 128
    n_cu = 1 + strips
    # per window: logits, shares of G and the update of V (2 N H NV each), both time loops and both
    # copies of Wh (2 T H^2 each)
    flops = W * (6.0 * T * H * NV + 8.0 * T * H * H)
    peak = n_cu * 256 * 2.4e9 / 1e12                # fp32 matrix rate of the occupied units, TFLOP/s
    lo = losses.cpu().numpy()
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
            t = json.load(fh).get("C2", {}).get("train_stream")
        if t and t.get("windows"):
            traffic = t["bytes_per_launch"] / t["windows"] * W    # counters were taken on a shorter stream
    except (OSError, ValueError):
        pass
    measured = ({"peak_measured": MEASURED["mfma_f32_TFLOPs"] * n_cu / N_CU,
                 "frac_measured": flops / sec / 1e12 / (MEASURED["mfma_f32_TFLOPs"] * n_cu / N_CU)}
                if MEASURED else {})
    return {
        "entry_point": "rnn_train_stream", "windows": W, "lr": lr, "workgroups": n_cu,
        "tokens_per_s": W * T / sec, "us_per_window": 1e6 * sec / W, "ms_per_stream": 1e3 * sec,
        "loss_first_window": float(lo[0]), "loss_mean_last_100_windows": float(lo[-100:].mean()),
        "roofline": {"kernel": "train_stream", "bound": "mfma", "achieved": flops / sec / 1e12,
                     "peak": peak, "unit": "TFLOP/s", "frac": flops / sec / 1e12 / peak,
                     "traffic": traffic, "n_cu": n_cu, "avg_us": 1e6 * sec,
                     "algorithmic_flops": flops, **measured,
                     "note": "one launch per stream; the model stays on chip (memory sees the ids, "
                             "the touched rows of Wx, the losses and the tagged words the workgroups "
                             "exchange), so the ceiling stated is the matrix rate of the occupied "
                             "compute units; the launch is bound by the latency of its dependent steps "
                             "and exchanges"},
    }


def mlp_leg(n_batches=400, lr=0.01):
    """The paper's neural-network training benchmark shapes (784 inputs, 10 classes; logistic
    regression, 1 x 500 and 3 x 1000 hidden units; batches of 1, 10, 60) through rnn_mlp_train:
    examples per second of `n_batches` consecutive SGD steps in one call, HIP-event timed on the
    call's stream, plus the per-kernel times of one configuration."""
    import numpy as np
    import torch
    import paper_1211_5590_amd as rnn
    import rnn_inputs as ri
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    out = {}
    for name in ("MLP0", "MLP1", "MLP3"):
        for batch in (1, 10, 60):
            case = ri.make_mlp_config(name, batch, n_batches=n_batches)
            dims = rnn.MlpDims.of(case)
            W, b = [dev(w) for w in case["W"]], [dev(v) for v in case["b"]]
            X, y = dev(case["X"]), dev(case["y"])
            losses = torch.zeros(n_batches, device="cuda")
            ws = torch.empty(rnn.rnn_mlp_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
            pr = rnn.mlp_params(W, b)
            rnn.rnn_mlp_train(dims, pr, None, X, y, 20, lr, losses, ws)          # warm-up
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record()
            rnn.rnn_mlp_train(dims, pr, None, X, y, n_batches, lr, losses, ws)
            e1.record()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            n_params = sum(w.numel() + v.numel() for w, v in zip(W, b))
            entry = dict(examples_per_s=n_batches * batch / wall, us_per_batch=1e6 * wall / n_batches,
                         gpu_event_us_per_batch=1e3 * e0.elapsed_time(e1) / n_batches,
                         launches_per_batch=2 * case["n_hidden"] + 2, parameters=n_params,
                         loss_first=float(losses[0]), loss_last=float(losses[-1]))
            if name == "MLP3" and batch == 60:
                rnn.rnn_profile_begin(1 << 16)
                rnn.rnn_mlp_train(dims, pr, None, X, y, 50, lr, losses, ws)
                prof = rnn.rnn_profile_end()
                entry["kernels"] = {k: dict(launches=c, avg_us_raw=round(1e3 * ms / c, 3)) for k, (c, ms) in sorted(prof.items())}
                # the update pass reads and rewrites every weight once: 8 bytes per parameter
                upd = prof.get("mlp_update")
                if upd:
                    us = 1e3 * upd[1] / upd[0]
                    nbytes = 8.0 * n_params          # one launch updates every layer
                    entry["roofline"] = dict(kernel="mlp_update", bound="hbm", achieved=nbytes / (us * 1e-6) / 1e9,
                                             peak=HBM_PEAK_GBS, unit="GB/s", frac=nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                             traffic=None, avg_us=us, algorithmic_bytes=nbytes,
                                             **({"peak_measured": max(MEASURED["hbm_read_GBps"], MEASURED["hbm_copy_GBps"]),
                                                 "frac_measured": nbytes / (us * 1e-6) / 1e9
                                                 / max(MEASURED["hbm_read_GBps"], MEASURED["hbm_copy_GBps"])}
                                                if MEASURED else {}),
                                             note="one launch per batch updates all layers; event bracket not removed")
            out[f"{name}_batch{batch}"] = entry
    return out


def mlp_cpu_baseline(seconds=3.0):
    """The classifier oracle (float64 numpy) timed on the host cores: three hidden layers, batch 60."""
    import rnn_inputs as ri
    from oracle import mlp
    case = ri.make_mlp_config("MLP3", 60, n_batches=4)
    t0 = time.perf_counter()
    done = 0
    while done < 1 or time.perf_counter() - t0 < seconds:
        mlp.train(case, 0.01, n_batches=4)
        done += 4
    dt = time.perf_counter() - t0
    return dict(value=done * 60 / dt, unit="examples/s", kind="oracle", cores=os.cpu_count(),
                sample=f"{done} batches of 60, 784-1000-1000-1000-10, float64 numpy", seconds=dt)


def gauss_newton_leg(names=("C3", "C4", "C5"), reps=5, flags=0):
    """One Gauss-Newton-vector product (R-operator sweep, loss metric, reverse sweep) per call of
    rnn_gauss_newton_vec on the named configurations, with the states of one forward pass:
    HIP-event time per product and its per-kernel times."""
    import numpy as np
    import torch
    import paper_1211_5590_amd as rnn
    import rnn_inputs as ri
    out = {}
    for name in names:
        w = Workload(name, flags, None, three_calls=True)
        stream = torch.cuda.current_stream().cuda_stream
        rc = w.L.rnn_forward(ctypes.byref(w.dims), ctypes.byref(w.P), w.x.data_ptr(), None, w.h_all.data_ptr(),
                             w.carry[0].data_ptr(), w.ws.data_ptr(), w.ws.numel(), stream)
        assert rc == 0, rc
        gamma = ri.make_direction(w.case, 1)
        g = {k: torch.from_numpy(np.ascontiguousarray(gamma[k])).cuda() for k in ("Wx", "Wh", "b", "V", "c")}
        res = {"d" + k: torch.zeros_like(v) for k, v in w.p.items()}
        gws = torch.empty(rnn.rnn_gauss_newton_workspace_bytes(w.dims), dtype=torch.uint8, device="cuda")
        rnn.rnn_workspace_init(w.dims, gws)
        call = lambda: rnn.rnn_gauss_newton_vec(w.dims, w.p, g, w.x, w.h_all, rnn.GN_METRIC_LOSS, res, None, gws)
        call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rnn.rnn_profile_begin(1 << 16)
        call()
        prof = rnn.rnn_profile_end()
        top = sorted(prof.items(), key=lambda kv: -kv[1][1])[:6]
        out[name] = dict(ms_per_product=ms, tokens_per_s=w.tokens_per_step / (ms * 1e-3),
                         kernels={k: dict(launches=c, total_ms_raw=round(t, 4)) for k, (c, t) in top})
        del w, gws, res, g
        torch.cuda.empty_cache()
    return out


def describe(c):
    return dict(in_dim=c["in_dim"], hidden=c["hidden"], out_dim=c["out_dim"], seq_len=c["seq_len"],
                batch=c["batch"], windows=c["windows"],
                input="token ids" if c["input_kind"] == 0 else "dense",
                act="sigmoid" if c["act"] == 0 else "tanh",
                loss="softmax-CE" if c["loss_kind"] == 0 else "linear-MSE")


def device_facts(torch):
    """What the runtime reports about the GPU the numbers were taken on."""
    pr = torch.cuda.get_device_properties(0)
    return dict(name=pr.name, arch=getattr(pr, "gcnArchName", None), compute_units=pr.multi_processor_count,
                memory_bytes=pr.total_memory, l2_bytes=getattr(pr, "L2_cache_size", None))


def oracle_rows(names, budget_s):
    """The oracle on the host cores for each named configuration: a row on all cores and a row on
    one thread (cpu_baseline says what each was timed on)."""
    return {name: cpu_baseline(name, budget_s) for name in names}


def sig(x, digits=5):
    """Floats of the output line rounded to a few significant digits (keeps the line short)."""
    if isinstance(x, float):
        return float(f"{x:.{digits}g}") if x == x and abs(x) != float("inf") else None
    if isinstance(x, dict):
        return {k: sig(v, digits) for k, v in x.items()}
    if isinstance(x, (list, tuple)):
        return [sig(v, digits) for v in x]
    return x


def run_config(name, flags, windows=None, three_calls=False, steps=None, warm=None, all_kernels=False):
    """Time one configuration and profile one more step of it per kernel."""
    import torch
    import paper_1211_5590_amd as rnn
    w = Workload(name, flags, windows, three_calls)
    steps = steps if steps is not None else DEFAULT_STEPS[name]
    warm = warm if warm is not None else DEFAULT_WARM[name]
    wall, gpu_s = w.time_steps(steps, warm)
    prof = w.profile(1)
    if w.fused and rnn.rnn_train_stream_status(w.wws) != 0:
        print("bench.py: a bounded wait of rnn_window expired; results invalid", file=sys.stderr)
        sys.exit(4)
    res = dict(workload=name, steps=steps, warmup=warm, wall_s=wall, gpu_s=gpu_s,
               tokens_per_s=w.tokens_per_step * steps / wall,
               timesteps_per_s=w.timesteps_per_step * steps / wall,
               ms_per_step=1e3 * wall / steps, gpu_event_ms_per_step=1e3 * gpu_s / steps,
               entry_points="rnn_window" if w.fused else "rnn_forward,rnn_loss,rnn_bptt",
               recurrence_variant=rnn.rnn_recurrence_variant(w.dims),
               describe=describe(w.case), roofline=roofline_of(prof, w.case),
               kernels={k: dict(launches=v["launches"], avg_us=round(v["avg_us"], 3),
                                total_ms=round(v["total_ms"], 4)) for k, v in sorted(prof.items())},
               bracket_us=w.bracket_us)
    if all_kernels:
        res["rooflines_all_kernels"] = all_rooflines(prof, w.case)
    if name == "C2" and res["roofline"] and res["roofline"]["kernel"] == "window":
        # what the method must move per window: V in and dV out (8.0 MB); the dense token-gradient
        # buffer the overwrite convention fills adds 4 MB
        H, O, I = w.case["hidden"], w.case["out_dim"], w.case["in_dim"]
        us = res["roofline"]["avg_us"]
        core = 4.0 * 2 * H * O
        res["roofline"]["algorithmic_bytes_without_dWx_fill"] = core
        res["roofline"]["frac_without_dWx_fill"] = core / (us * 1e-6) / 1e9 / HBM_PEAK_GBS
    del w
    torch.cuda.empty_cache()
    return res


def per_config_entry(r):
    return dict(tokens_per_s=r["tokens_per_s"], timesteps_per_s=r["timesteps_per_s"], ms_per_step=r["ms_per_step"],
                entry_points=r["entry_points"], recurrence_variant=r["recurrence_variant"],
                roofline=r["roofline"], kernels=r["kernels"])


def summary_row(r):
    rf = r.get("roofline") or {}
    return [round(r["ms_per_step"], 4), round(r["tokens_per_s"], 1), rf.get("kernel"),
            None if rf.get("frac") is None else round(rf["frac"], 4)]


# at least 20 timed steps after at least 3 warm-ups, except the 10000-window stream (0.24 s per pass)
DEFAULT_STEPS = {"C1": 200, "C2": 3, "C3": 50, "C4": 20, "C5": 20}
DEFAULT_WARM = {"C1": 20, "C2": 1, "C3": 5, "C4": 3, "C5": 3}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              f"--gpus {a.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_1211_5590_amd as rnn
    scratch = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    MEASURED.update(rnn.rnn_measure_ceilings(scratch))
    del scratch
    torch.cuda.empty_cache()
    if a.only_mlp:
        print(json.dumps({"metric": "classifier training examples/sec", "unit": "examples/s", "n_gpus": 1,
                          "dtype": "f32", "data": "synthetic", "mlp_workloads": mlp_leg()}))
        return
    flags = rnn.FLAG_REFERENCE_KERNELS if a.reference_kernels else 0
    if a.bf16x3:
        flags |= rnn.FLAG_BF16X3_OUTPUT
    plain = not a.reference_kernels and not a.bf16x3

    if a.calibration_copy:
        src = torch.ones(16 << 20, device="cuda")          # 64 MiB read + 64 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head = run_config(a.workload, flags, a.windows, a.three_calls, a.steps, a.warmup, all_kernels=True)
    summary = {a.workload: summary_row(head)}

    per = {}
    others = [s for s in a.others.split(",") if s and s != "none" and s != a.workload]
    for name in others:
        r = run_config(name, flags, a.windows if name == "C2" else None)
        per[name] = per_config_entry(r)
        summary[name] = summary_row(r)
    extra = {}
    if "C2" in [a.workload] + others and plain:
        # the same stream through the three separate calls, and through the one-launch SGD driver
        if not a.three_calls:
            r3 = run_config("C2", flags, a.windows, three_calls=True, steps=1, warm=1)
            extra["C2_three_calls"] = per_config_entry(r3)
            summary["C2_three_calls"] = summary_row(r3)
        if not a.no_train_stream:
            ts = train_stream_leg(a.windows)
            extra["C2_train_stream"] = ts
            summary["C2_train_stream"] = [round(ts["ms_per_stream"], 4), round(ts["tokens_per_s"], 1),
                                          "train_stream", round(ts["roofline"]["frac"], 4)]
    if "C4" in [a.workload] + others and plain:
        # the same configuration with the opt-in bf16 hi/lo split output layer
        rb = run_config("C4", flags | rnn.FLAG_BF16X3_OUTPUT)
        e = per_config_entry(rb)
        e["flag"] = "RNN_FLAG_BF16X3_OUTPUT"
        extra["C4_bf16x3_output"] = e
        summary["C4_bf16x3_output"] = summary_row(rb)

    out = {
        "metric": "fwd+BPTT tokens/sec",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (output-layer products: bf16 hi/lo split, f32 accumulate)" if a.bf16x3 else "f32",
        "data": "synthetic",
        "config": dict(workload=a.workload, **head["describe"], entry_points=head["entry_points"],
                       recurrence_variant=head["recurrence_variant"]),
        # every configuration in one place: [ms per step, tokens/s, dominant kernel, its roofline fraction]
        "summary": summary,
        "timesteps_per_s": head["timesteps_per_s"],
        "gpu_event_ms_per_step": head["gpu_event_ms_per_step"],
        "roofline": head["roofline"],
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.workload, a.cpu_seconds)
    out["kernels"] = head["kernels"]
    out["rooflines_all_kernels"] = head["rooflines_all_kernels"]
    out["event_bracket_us"] = round(head["bracket_us"], 3)
    if per or extra:
        out["per_config"] = dict(per, **extra)
    if not a.no_cpu_baseline and others:
        out["oracle_timing"] = oracle_rows([n for n in others if n in ("C2", "C3", "C5")], min(a.cpu_seconds, 15.0))
    if plain and not a.no_mlp and others:
        out["mlp_workloads"] = mlp_leg()
        if not a.no_cpu_baseline:
            out["mlp_workloads"]["cpu_baseline"] = mlp_cpu_baseline()
    if plain and others:
        gn = [n for n in ("C3", "C4", "C5") if n in [a.workload] + others]
        out["gauss_newton_vec"] = gauss_newton_leg(gn)
        if "C4" in gn:
            out["gauss_newton_vec"]["C4_bf16x3_output"] = gauss_newton_leg(["C4"], flags=rnn.FLAG_BF16X3_OUTPUT)["C4"]
    out["device"] = device_facts(torch)
    out["measured_ceilings"] = dict(MEASURED, note="saturating kernels of the library itself on this GPU: "
                                    "device-memory copy (read + written bytes) and read (the larger is the HBM ceiling), 32x32x2 f32 and 32x32x16 bf16 "
                                    "matrix products, 16-byte LDS reads; frac_measured in the roofline entries "
                                    "is stated against these, frac against the published peaks")
    print(json.dumps(sig(out)))


if __name__ == "__main__":
    main()
