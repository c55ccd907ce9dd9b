"""Seeded synthetic inputs for the Elman-RNN training path.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no recurrence, no softmax, no gradients).  Both the CPU
oracle's tests and the GPU library's tests/bench import it so that the two sides
see identical arrays.

The paper's recurrent benchmark (its section on benchmarking recurrent networks)
trains a simple recurrent language model with batch size 1 and equal input/output
vocabulary; its corpus is not available, so token streams here are synthetic:
Zipf-distributed ids over a finite vocabulary reproduce the skewed token
frequencies that matter to the embedding gather/scatter.  Nothing else on the
path depends on token identity.

Layouts (all float32, row-major, time-major):
  token input : x int32[T,B], y int32[T,B] (next-token targets)
  dense input : X f32[T,B,D], Y f32[T,B,O]
  Wx f32[NV,H] (token input; row v is token v's input vector) or f32[H,D] (dense)
  Wh f32[H,H]  (pre-activation a[j] = sum_i Wh[j,i] * h_prev[i])
  b  f32[H],  V f32[H,OUT] (z[k] = sum_i h[i] * V[i,k] + c[k]),  c f32[OUT]
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 12115590

INPUT_TOKENS, INPUT_DENSE = 0, 1
ACT_SIGMOID, ACT_TANH = 0, 1
LOSS_SOFTMAX_CE, LOSS_LINEAR_MSE = 0, 1

# The five benchmark configurations.  "windows" > 1 means a token stream cut into
# consecutive truncated-BPTT windows of seq_len steps with the hidden state carried.
CONFIGS = {
    "C1": dict(in_dim=64, hidden=16, out_dim=64, seq_len=32, batch=1, windows=1,
               input_kind=INPUT_TOKENS, act=ACT_SIGMOID, loss_kind=LOSS_SOFTMAX_CE,
               tokens="uniform", wdist=("normal", 0.1), seed=BASE_SEED + 1000),
    "C2": dict(in_dim=10000, hidden=100, out_dim=10000, seq_len=10, batch=1, windows=10000,
               input_kind=INPUT_TOKENS, act=ACT_SIGMOID, loss_kind=LOSS_SOFTMAX_CE,
               tokens="zipf", wdist=("normal", 0.1), seed=BASE_SEED + 2000),
    "C3": dict(in_dim=10000, hidden=500, out_dim=10000, seq_len=100, batch=1, windows=1,
               input_kind=INPUT_TOKENS, act=ACT_SIGMOID, loss_kind=LOSS_SOFTMAX_CE,
               tokens="zipf", wdist=("uniform", 0.05), seed=BASE_SEED + 3000),
    "C4": dict(in_dim=10000, hidden=1024, out_dim=10000, seq_len=256, batch=64, windows=1,
               input_kind=INPUT_TOKENS, act=ACT_SIGMOID, loss_kind=LOSS_SOFTMAX_CE,
               tokens="zipf", wdist=("normal_fan", None), seed=BASE_SEED + 4000),
    "C5": dict(in_dim=128, hidden=256, out_dim=128, seq_len=4096, batch=128, windows=1,
               input_kind=INPUT_DENSE, act=ACT_TANH, loss_kind=LOSS_LINEAR_MSE,
               tokens=None, wdist=("normal_fan", None), seed=BASE_SEED + 5000),
}

ZIPF_S = 1.1


def zipf_cdf(nv: int, s: float = ZIPF_S) -> np.ndarray:
    """CDF of P(id = r) proportional to (r+1)^-s on r = 0..nv-1 (exact finite normalisation)."""
    w = np.arange(1, nv + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    return cdf / cdf[-1]


def draw_tokens(rng: np.random.Generator, n: int, nv: int, kind: str) -> np.ndarray:
    """n token ids in [0, nv): 'uniform', or 'zipf' by inverse CDF (id 0 most frequent)."""
    if kind == "uniform":
        return rng.integers(0, nv, size=n, dtype=np.int64).astype(np.int32)
    if kind == "zipf":
        u = rng.random(n)
        ids = np.searchsorted(zipf_cdf(nv), u, side="left")
        return np.minimum(ids, nv - 1).astype(np.int32)
    raise ValueError(f"unknown token distribution {kind!r}")


def _draw_weight(rng, shape, wdist, fan_in):
    kind, scale = wdist
    if kind == "normal":
        w = rng.normal(0.0, scale, size=shape)
    elif kind == "uniform":
        w = rng.uniform(-scale, scale, size=shape)
    elif kind == "normal_fan":  # standard deviation 1/sqrt(fan_in)
        w = rng.normal(0.0, 1.0 / np.sqrt(fan_in), size=shape)
    else:
        raise ValueError(f"unknown weight distribution {kind!r}")
    return np.ascontiguousarray(w, dtype=np.float32)


def make_case(in_dim, hidden, out_dim, seq_len, batch, *, input_kind=INPUT_TOKENS,
              act=ACT_SIGMOID, loss_kind=LOSS_SOFTMAX_CE, tokens="zipf",
              wdist=("normal", 0.1), seed=BASE_SEED, windows=1, bias_std=0.0,
              with_h0=False, with_dh_last=False, **_unused):
    """Draw one problem instance.  Returns a dict of numpy arrays plus the sizes.

    Token input: a stream of windows*seq_len+1 ids per batch row is drawn; x is the
    first windows*seq_len of them and y the same stream shifted by one (next token),
    both shaped [windows*seq_len, batch].  Window w of a stream uses rows
    [w*seq_len, (w+1)*seq_len).
    Dense input: X ~ N(0,1) of shape [T,B,D]; Y[0] = 0 and Y[t] = X[t-1] (needs O == D).
    Sub-streams are spawned in the fixed order (inputs, Wx, Wh, V, extras).
    """
    ss = np.random.SeedSequence(seed)
    s_in, s_wx, s_wh, s_v, s_extra = ss.spawn(5)
    T_total = seq_len * windows
    H = hidden
    out = dict(in_dim=in_dim, hidden=hidden, out_dim=out_dim, seq_len=seq_len, batch=batch,
               windows=windows, input_kind=input_kind, act=act, loss_kind=loss_kind)

    if input_kind == INPUT_TOKENS:
        rows = []
        for s_row in s_in.spawn(batch):
            rows.append(draw_tokens(np.random.default_rng(s_row), T_total + 1, in_dim, tokens))
        ids = np.stack(rows, axis=1)                      # [T_total+1, B]
        out["x"] = np.ascontiguousarray(ids[:-1])
        if loss_kind == LOSS_SOFTMAX_CE:
            if out_dim != in_dim:                         # targets must lie in [0, out_dim)
                out["y"] = np.ascontiguousarray(ids[1:] % out_dim).astype(np.int32)
            else:
                out["y"] = np.ascontiguousarray(ids[1:])
        wx_shape, wx_fan = (in_dim, H), in_dim
    else:
        rng = np.random.default_rng(s_in)
        X = rng.standard_normal(size=(T_total, batch, in_dim), dtype=np.float32)
        out["X"] = X
        if loss_kind == LOSS_SOFTMAX_CE:
            out["y"] = rng.integers(0, out_dim, size=(T_total, batch)).astype(np.int32)
        wx_shape, wx_fan = (H, in_dim), in_dim
    if loss_kind == LOSS_LINEAR_MSE:
        if input_kind == INPUT_DENSE and out_dim == in_dim:
            Y = np.zeros_like(out["X"])
            Y[1:] = out["X"][:-1]
        else:
            Y = np.random.default_rng(s_extra.spawn(1)[0]).standard_normal(
                size=(T_total, batch, out_dim), dtype=np.float32)
        out["Y"] = Y

    out["Wx"] = _draw_weight(np.random.default_rng(s_wx), wx_shape, wdist, wx_fan)
    out["Wh"] = _draw_weight(np.random.default_rng(s_wh), (H, H), wdist, H)
    out["V"] = _draw_weight(np.random.default_rng(s_v), (H, out_dim), wdist, H)
    rng_e = np.random.default_rng(s_extra)
    if bias_std > 0.0:
        out["b"] = rng_e.normal(0.0, bias_std, size=H).astype(np.float32)
        out["c"] = rng_e.normal(0.0, bias_std, size=out_dim).astype(np.float32)
    else:
        out["b"] = np.zeros(H, dtype=np.float32)
        out["c"] = np.zeros(out_dim, dtype=np.float32)
    lo, hi = (0.05, 0.95) if act == ACT_SIGMOID else (-0.9, 0.9)
    out["h0"] = rng_e.uniform(lo, hi, size=(batch, H)).astype(np.float32) if with_h0 else None
    out["dh_last"] = (rng_e.normal(0.0, 0.01, size=(batch, H)).astype(np.float32)
                      if with_dh_last else None)
    return out


def make_config(name: str, **overrides):
    """One of the five named configurations (C1..C5), optionally with sizes overridden."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    return make_case(**cfg)


def window(case: dict, w: int) -> dict:
    """View of truncated-BPTT window w of a multi-window token stream (no copies of weights)."""
    T = case["seq_len"]
    out = dict(case)
    out["windows"] = 1
    for k in ("x", "y", "X", "Y"):
        if k in case and case[k] is not None:
            out[k] = np.ascontiguousarray(case[k][w * T:(w + 1) * T])
    return out


def stream_ids(case: dict) -> np.ndarray:
    """The token stream of a multi-window token case as one array int32[windows*T + 1, B]:
    x followed by the last target (y is the same stream shifted by one step)."""
    return np.ascontiguousarray(np.concatenate([case["x"], case["y"][-1:]], axis=0), dtype=np.int32)


def make_direction(case: dict, seed: int, scale: float = 1.0) -> dict:
    """A random direction gamma of the parameters' shapes (for Jacobian-vector products)."""
    rng = np.random.default_rng(np.random.SeedSequence([BASE_SEED, seed]))
    return {k: (scale * rng.standard_normal(size=np.shape(case[k]))).astype(np.float32)
            for k in ("Wx", "Wh", "b", "V", "c")}


# ---------------------------------------------------------------------------------------
# Feed-forward classifier workloads (the paper's neural-network training benchmark: 10-class
# classification of a 784-dimensional input with 0, 1 x 500 or 3 x 1000 hidden units, batches of
# 1, 10 or 60).  Its data set is not available: inputs are uniform in [0,1) like pixel
# intensities, labels uniform over the classes.
MLP_CONFIGS = {
    "MLP0": dict(in_dim=784, hidden=0, n_hidden=0, out_dim=10),
    "MLP1": dict(in_dim=784, hidden=500, n_hidden=1, out_dim=10),
    "MLP3": dict(in_dim=784, hidden=1000, n_hidden=3, out_dim=10),
}


def mlp_layer_shapes(in_dim, hidden, n_hidden, out_dim):
    """[(fan_out, fan_in)] of the n_hidden + 1 layers, input side first."""
    widths = [in_dim] + [hidden] * n_hidden + [out_dim]
    return [(widths[l + 1], widths[l]) for l in range(n_hidden + 1)]


def make_mlp_case(in_dim, hidden, n_hidden, out_dim, batch, n_batches=1, *, act=ACT_TANH, seed=BASE_SEED + 77,
                  bias_std=0.0, wscale=1.0):
    """One feed-forward problem: X float32 [n_batches*batch, in_dim] ~ U[0,1), y int32 labels,
    W[l] float32 [fan_out, fan_in] ~ N(0, wscale/sqrt(fan_in)), b[l] float32 [fan_out]."""
    s_x, s_y, s_w, s_b = np.random.SeedSequence(seed).spawn(4)
    rows = batch * n_batches
    out = dict(in_dim=in_dim, hidden=hidden, n_hidden=n_hidden, out_dim=out_dim, batch=batch,
               n_batches=n_batches, act=act)
    out["X"] = np.random.default_rng(s_x).random(size=(rows, in_dim), dtype=np.float32)
    out["y"] = np.random.default_rng(s_y).integers(0, out_dim, size=rows).astype(np.int32)
    shapes = mlp_layer_shapes(in_dim, hidden, n_hidden, out_dim)
    out["W"] = [(np.random.default_rng(s).normal(0.0, wscale / np.sqrt(sh[1]), size=sh)).astype(np.float32)
                for s, sh in zip(s_w.spawn(len(shapes)), shapes)]
    rb = np.random.default_rng(s_b)
    out["b"] = [(rb.normal(0.0, bias_std, size=sh[0]) if bias_std > 0 else np.zeros(sh[0])).astype(np.float32)
                for sh in shapes]
    return out


def make_mlp_config(name: str, batch: int, n_batches: int = 1, **overrides):
    cfg = dict(MLP_CONFIGS[name])
    cfg.update(overrides)
    return make_mlp_case(batch=batch, n_batches=n_batches, **cfg)
