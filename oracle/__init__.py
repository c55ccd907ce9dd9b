"""Python front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's cpu_baseline leg may import this package;
the GPU library and its binding never do.  Everything is computed by the plain C loops
in rnn_oracle.c in double precision; this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rnn_oracle.c")
_LIB = os.path.join(_HERE, "librnn_oracle.so")


def build(force: bool = False) -> str:
    """Compile rnn_oracle.c with gcc (plain -O3, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("in_dim", "hidden", "out_dim", "seq_len", "batch", "input_kind", "act", "loss_kind")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(ctypes.c_int(n))


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dims(p):
    return _Dims(p["in_dim"], p["hidden"], p["out_dim"], p["seq_len"], p["batch"],
                 p["input_kind"], p["act"], p["loss_kind"])


def _inputs(p):
    if p["input_kind"] == 0:
        x = np.ascontiguousarray(p["x"], dtype=np.int32)
        assert x.shape == (p["seq_len"], p["batch"])
    else:
        x = _f64(p["X"])
        assert x.shape == (p["seq_len"], p["batch"], p["in_dim"])
    return x


def _targets(p):
    if p["loss_kind"] == 0:
        y = np.ascontiguousarray(p["y"], dtype=np.int32)
        assert y.shape == (p["seq_len"], p["batch"])
    else:
        y = _f64(p["Y"])
        assert y.shape == (p["seq_len"], p["batch"], p["out_dim"])
    return y


def forward(p, h0=None):
    """h_all float64[T+1,B,H]; h_all[0] is the initial state, h_all[t+1] = h_t."""
    lib = _load()
    T, B, H = p["seq_len"], p["batch"], p["hidden"]
    Wx, Wh, b = _f64(p["Wx"]), _f64(p["Wh"]), _f64(p["b"])
    x = _inputs(p)
    h0 = _f64(h0 if h0 is not None else p.get("h0"))
    h_all = np.empty((T + 1, B, H), dtype=np.float64)
    d = _dims(p)
    rc = lib.orc_forward(ctypes.byref(d), _ptr(Wx), _ptr(Wh), _ptr(b), _ptr(x), _ptr(h0), _ptr(h_all))
    if rc != 0:
        raise ValueError("orc_forward: bad argument")
    return h_all


def loss(p, h_all, want_lse=False, want_Z=False):
    """Scalar loss (and optionally lse[N], Z[N,O]) from stored hidden states."""
    lib = _load()
    N, O = p["seq_len"] * p["batch"], p["out_dim"]
    V, c = _f64(p["V"]), _f64(p["c"])
    y = _targets(p)
    h_all = _f64(h_all)
    out = ctypes.c_double(0.0)
    lse = np.empty(N, dtype=np.float64) if want_lse else None
    Z = np.empty((N, O), dtype=np.float64) if want_Z else None
    d = _dims(p)
    rc = lib.orc_loss(ctypes.byref(d), _ptr(V), _ptr(c), _ptr(h_all), _ptr(y),
                      ctypes.byref(out), _ptr(lse), _ptr(Z))
    if rc != 0:
        raise ValueError("orc_loss: bad argument")
    res = [float(out.value)]
    if want_lse:
        res.append(lse)
    if want_Z:
        res.append(Z)
    return res[0] if len(res) == 1 else tuple(res)


def bptt(p, h_all, dh_last=None, want_internals=False):
    """Gradients dict: dWx, dWh, db, dV, dc, dh0 (+ delta, g, dZ when want_internals)."""
    lib = _load()
    T, B, H, O = p["seq_len"], p["batch"], p["hidden"], p["out_dim"]
    N = T * B
    Wx, Wh, V, c = _f64(p["Wx"]), _f64(p["Wh"]), _f64(p["V"]), _f64(p["c"])
    x, y = _inputs(p), _targets(p)
    h_all = _f64(h_all)
    dh_last = _f64(dh_last if dh_last is not None else p.get("dh_last"))
    g = dict(dWx=np.empty_like(Wx), dWh=np.empty_like(Wh), db=np.empty(H), dV=np.empty_like(V),
             dc=np.empty(O), dh0=np.empty((B, H)))
    delta = np.empty((T, B, H)) if want_internals else None
    gg = np.empty((T, B, H)) if want_internals else None
    dZ = np.empty((N, O)) if want_internals else None
    d = _dims(p)
    rc = lib.orc_bptt(ctypes.byref(d), _ptr(Wx), _ptr(Wh), _ptr(V), _ptr(c), _ptr(x), _ptr(y),
                      _ptr(h_all), _ptr(dh_last), _ptr(g["dWx"]), _ptr(g["dWh"]), _ptr(g["db"]),
                      _ptr(g["dV"]), _ptr(g["dc"]), _ptr(g["dh0"]), _ptr(delta), _ptr(gg), _ptr(dZ))
    if rc != 0:
        raise ValueError("orc_bptt: bad argument")
    if want_internals:
        g.update(delta=delta, g=gg, dZ=dZ)
    return g


def fwd_bptt(p, h0=None, dh_last=None):
    """Convenience: forward, loss and gradients of one window."""
    h_all = forward(p, h0)
    L, lse = (loss(p, h_all, want_lse=True) if p["loss_kind"] == 0 else (loss(p, h_all), None))
    g = bptt(p, h_all, dh_last)
    g.update(loss=L, lse=lse, h_all=h_all)
    return g


def train_stream(p, ids, n_windows, lr, h0=None):
    """Plain SGD over n_windows consecutive windows of a token stream (token input, softmax-CE).

    ids int32[n_windows*T + 1, B].  Returns dict: Wx, Wh, b, V, c (after the last update),
    h_last [B,H] and losses [n_windows]; p's arrays are not modified.
    """
    lib = _load()
    T, B, H = p["seq_len"], p["batch"], p["hidden"]
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1, B)
    assert ids.shape[0] >= n_windows * T + 1
    out = {k: np.array(p[k], dtype=np.float64, order="C", copy=True) for k in ("Wx", "Wh", "b", "V", "c")}
    h = np.zeros((B, H)) if h0 is None else np.array(h0, dtype=np.float64, order="C", copy=True).reshape(B, H)
    losses = np.empty(n_windows, dtype=np.float64)
    d = _dims(p)
    rc = lib.orc_train_stream(ctypes.byref(d), _ptr(out["Wx"]), _ptr(out["Wh"]), _ptr(out["b"]),
                              _ptr(out["V"]), _ptr(out["c"]), _ptr(ids), ctypes.c_long(n_windows),
                              ctypes.c_double(lr), _ptr(h), _ptr(losses))
    if rc != 0:
        raise ValueError("orc_train_stream: bad argument")
    out.update(h_last=h, losses=losses)
    return out


def gauss_newton_vec(p, gamma, h_all=None, metric=0, want_Rz=False):
    """G gamma = J^T M J gamma by one R-operator sweep and one reverse sweep.

    gamma: dict with Wx, Wh, b, V, c (a direction of the parameters' shapes); metric 0 = the
    loss Hessian w.r.t. the outputs, 1 = identity.  Returns dict GWx, GWh, Gb, GV, Gc (+ Rz).
    """
    lib = _load()
    N, O = p["seq_len"] * p["batch"], p["out_dim"]
    Wx, Wh, V, c = _f64(p["Wx"]), _f64(p["Wh"]), _f64(p["V"]), _f64(p["c"])
    g = {k: _f64(gamma[k]) for k in ("Wx", "Wh", "b", "V", "c")}
    x = _inputs(p)
    h_all = _f64(h_all if h_all is not None else forward(p, p.get("h0")))
    out = dict(GWx=np.empty_like(Wx), GWh=np.empty_like(Wh), Gb=np.empty(p["hidden"]),
               GV=np.empty_like(V), Gc=np.empty(O))
    Rz = np.empty((N, O)) if want_Rz else None
    d = _dims(p)
    rc = lib.orc_gauss_newton_vec(ctypes.byref(d), ctypes.c_int(metric), _ptr(Wx), _ptr(Wh), _ptr(V),
                                  _ptr(c), _ptr(g["Wx"]), _ptr(g["Wh"]), _ptr(g["b"]), _ptr(g["V"]),
                                  _ptr(g["c"]), _ptr(x), _ptr(h_all), _ptr(out["GWx"]), _ptr(out["GWh"]),
                                  _ptr(out["Gb"]), _ptr(out["GV"]), _ptr(out["Gc"]), _ptr(Rz))
    if rc != 0:
        raise ValueError("orc_gauss_newton_vec: bad argument")
    if want_Rz:
        out["Rz"] = Rz
    return out
