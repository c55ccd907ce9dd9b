"""ctypes binding with the same names as the C ABI (argument marshalling only).

Tensors are torch CUDA tensors used purely as device memory; raw pointers and the current
torch stream are handed to the library.  Nothing here computes anything.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
# RNN_MI355X_LIB selects another build of the same library (e.g. an instrumented one)
_LIB_PATH = os.environ.get("RNN_MI355X_LIB") or os.path.join(_PKG, "librnn_mi355x.so")

INPUT_TOKENS, INPUT_DENSE = 0, 1
ACT_SIGMOID, ACT_TANH = 0, 1
LOSS_SOFTMAX_CE, LOSS_LINEAR_MSE = 0, 1
FLAG_ACCUMULATE, FLAG_SYNC, FLAG_BPTT_RECOMPUTE, FLAG_REFERENCE_KERNELS = 1, 2, 4, 8
FLAG_BF16X3_OUTPUT = 16
FLAG_COOPERATIVE = 32

EXPORTS = ("rnn_workspace_bytes", "rnn_forward", "rnn_loss", "rnn_bptt", "rnn_check_tokens",
           "rnn_strerror", "rnn_recurrence_variant", "rnn_recurrence_workgroups", "rnn_profile_begin", "rnn_profile_end",
           "rnn_profile_kernel_count", "rnn_profile_kernel_name", "rnn_workspace_init", "rnn_set_wait_limit",
           "rnn_workspace_status", "rnn_train_stream_workspace_bytes", "rnn_train_stream",
           "rnn_train_stream_status", "rnn_window_one_launch", "rnn_window_workspace_bytes", "rnn_window_workspace_init",
           "rnn_window", "rnn_window_static", "rnn_gauss_newton_workspace_bytes", "rnn_gauss_newton_vec",
           "rnn_mlp_workspace_bytes", "rnn_mlp_train", "rnn_measure_ceilings")
MLP_MAX_LAYERS = 16
GN_METRIC_LOSS, GN_METRIC_IDENTITY = 0, 1


class RnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"rnn error {code}: {msg}")
        self.code = code


class Dims(ctypes.Structure):
    _fields_ = [("in_dim", ctypes.c_int32), ("hidden", ctypes.c_int32), ("out_dim", ctypes.c_int32),
                ("seq_len", ctypes.c_int32), ("batch", ctypes.c_int32), ("input_kind", ctypes.c_int32),
                ("act", ctypes.c_int32), ("loss_kind", ctypes.c_int32), ("flags", ctypes.c_uint32)]

    @classmethod
    def of(cls, case: dict, flags: int = 0) -> "Dims":
        return cls(case["in_dim"], case["hidden"], case["out_dim"], case["seq_len"], case["batch"],
                   case["input_kind"], case["act"], case["loss_kind"], flags)


class Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("Wx", "Wh", "b", "V", "c")]


class Grads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("dWx", "dWh", "db", "dV", "dc")]


class MlpDims(ctypes.Structure):
    _fields_ = [("in_dim", ctypes.c_int32), ("hidden", ctypes.c_int32), ("n_hidden", ctypes.c_int32),
                ("out_dim", ctypes.c_int32), ("batch", ctypes.c_int32), ("act", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]

    @classmethod
    def of(cls, case: dict, flags: int = 0) -> "MlpDims":
        return cls(case["in_dim"], case["hidden"], case["n_hidden"], case["out_dim"], case["batch"],
                   case["act"], flags)


class MlpParams(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p * MLP_MAX_LAYERS), ("b", ctypes.c_void_p * MLP_MAX_LAYERS)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Load librnn_mi355x.so (building it first only if it has never been built)."""
    global _lib
    if _lib is None:
        # torch ships its own HIP runtime: it has to be in the process before this library is
        # loaded, so that both use the same one whatever the import order of the caller
        import torch  # noqa: F401
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.rnn_workspace_bytes.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(sz)]
        L.rnn_forward.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Params), vp, vp, vp, vp, vp, sz, vp]
        L.rnn_loss.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Params), vp, vp, vp, vp, sz, vp]
        L.rnn_bptt.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Params), vp, vp, vp, vp,
                               ctypes.POINTER(Grads), vp, vp, sz, vp]
        L.rnn_check_tokens.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, vp]
        L.rnn_strerror.argtypes = [ctypes.c_int]
        L.rnn_strerror.restype = ctypes.c_char_p
        L.rnn_recurrence_variant.argtypes = [ctypes.POINTER(Dims)]
        L.rnn_recurrence_variant.restype = ctypes.c_char_p
        L.rnn_recurrence_workgroups.argtypes = [ctypes.POINTER(Dims)]
        L.rnn_recurrence_workgroups.restype = ctypes.c_int
        L.rnn_workspace_init.argtypes = [ctypes.POINTER(Dims), vp, sz, vp]
        L.rnn_workspace_status.argtypes = [ctypes.POINTER(Dims), vp, sz, vp, ctypes.POINTER(ctypes.c_int32)]
        L.rnn_set_wait_limit.argtypes = [ctypes.c_int]
        L.rnn_set_wait_limit.restype = ctypes.c_int
        L.rnn_workspace_init.restype = ctypes.c_int
        L.rnn_workspace_status.restype = ctypes.c_int
        L.rnn_profile_begin.argtypes = [ctypes.c_int]
        L.rnn_profile_end.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)]
        L.rnn_profile_kernel_name.argtypes = [ctypes.c_int]
        L.rnn_profile_kernel_name.restype = ctypes.c_char_p
        for name in ("rnn_profile_begin", "rnn_profile_end", "rnn_profile_kernel_count"):
            getattr(L, name).restype = ctypes.c_int
        L.rnn_train_stream_workspace_bytes.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(sz)]
        L.rnn_train_stream.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Grads), vp, ctypes.c_int64,
                                       ctypes.c_float, vp, vp, vp, vp, sz, vp]
        L.rnn_train_stream_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32)]
        L.rnn_window_one_launch.argtypes = [ctypes.POINTER(Dims)]
        L.rnn_window_one_launch.restype = ctypes.c_int
        L.rnn_window_workspace_bytes.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(sz)]
        L.rnn_window_workspace_init.argtypes = [ctypes.POINTER(Dims), vp, sz, vp]
        L.rnn_window.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Params), vp, vp, vp, vp, vp, vp, vp,
                                 ctypes.POINTER(Grads), vp, vp, sz, vp]
        L.rnn_window_static.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Params), vp, vp, vp, vp, vp, vp, vp,
                                        ctypes.POINTER(Grads), vp, vp, vp]
        L.rnn_window_static.restype = ctypes.c_int
        L.rnn_gauss_newton_workspace_bytes.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(sz)]
        L.rnn_gauss_newton_vec.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(Params), ctypes.POINTER(Params),
                                           vp, vp, ctypes.c_int32, ctypes.POINTER(Grads), vp, vp, sz, vp]
        L.rnn_mlp_workspace_bytes.argtypes = [ctypes.POINTER(MlpDims), ctypes.POINTER(sz)]
        L.rnn_mlp_train.argtypes = [ctypes.POINTER(MlpDims), ctypes.POINTER(MlpParams), vp, vp, ctypes.c_int64,
                                    ctypes.c_float, vp, vp, sz, vp]
        L.rnn_measure_ceilings.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_double), vp]
        for name in ("rnn_mlp_workspace_bytes", "rnn_mlp_train", "rnn_measure_ceilings"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("rnn_gauss_newton_workspace_bytes", "rnn_gauss_newton_vec"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("rnn_train_stream_workspace_bytes", "rnn_train_stream", "rnn_train_stream_status",
                     "rnn_window_workspace_bytes", "rnn_window_workspace_init", "rnn_window"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("rnn_workspace_bytes", "rnn_forward", "rnn_loss", "rnn_bptt", "rnn_check_tokens"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def exported_symbols():
    L = lib()
    return [n for n in EXPORTS if hasattr(L, n)]


def _p(t):
    """Device (or host) address of a tensor-like, None -> NULL, int passes through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc):
    if rc != 0:
        raise RnnError(rc, rnn_strerror(rc))


def rnn_strerror(code: int) -> str:
    return lib().rnn_strerror(code).decode()


def rnn_recurrence_variant(dims: Dims) -> str:
    return lib().rnn_recurrence_variant(ctypes.byref(dims)).decode()


def rnn_recurrence_workgroups(dims: Dims) -> int:
    n = lib().rnn_recurrence_workgroups(ctypes.byref(dims))
    if n < 0:
        raise RnnError(n, rnn_strerror(n))
    return n


def rnn_workspace_bytes(dims: Dims) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().rnn_workspace_bytes(ctypes.byref(dims), ctypes.byref(out)))
    return int(out.value)


def _params(params) -> Params:
    if isinstance(params, Params):
        return params
    return Params(*[_p(params[k]) for k in ("Wx", "Wh", "b", "V", "c")])


def _grads(grads) -> Grads:
    if isinstance(grads, Grads):
        return grads
    return Grads(*[_p(grads[k]) for k in ("dWx", "dWh", "db", "dV", "dc")])


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def rnn_forward(dims, params, x, h0, h_all, h_last, workspace, stream=None, check=True):
    wp, wb = _ws(workspace)
    pr = _params(params)
    rc = lib().rnn_forward(ctypes.byref(dims), ctypes.byref(pr), _p(x), _p(h0), _p(h_all),
                           _p(h_last), wp, wb, _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_loss(dims, params, h_all, targets, loss, workspace, stream=None, check=True):
    wp, wb = _ws(workspace)
    pr = _params(params)
    rc = lib().rnn_loss(ctypes.byref(dims), ctypes.byref(pr), _p(h_all), _p(targets), _p(loss),
                        wp, wb, _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_bptt(dims, params, x, targets, h_all, dh_last, grads, dh0, workspace, stream=None, check=True):
    wp, wb = _ws(workspace)
    pr, gr = _params(params), _grads(grads)
    rc = lib().rnn_bptt(ctypes.byref(dims), ctypes.byref(pr), _p(x), _p(targets), _p(h_all),
                        _p(dh_last), ctypes.byref(gr), _p(dh0), wp, wb, _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_gauss_newton_workspace_bytes(dims: Dims) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().rnn_gauss_newton_workspace_bytes(ctypes.byref(dims), ctypes.byref(n)))
    return n.value


def rnn_gauss_newton_vec(dims, params, gamma, x, h_all, metric, out, Rz, workspace, stream=None, check=True):
    wp, wb = _ws(workspace)
    pr, ga, gr = _params(params), _params(gamma), _grads(out)
    rc = lib().rnn_gauss_newton_vec(ctypes.byref(dims), ctypes.byref(pr), ctypes.byref(ga), _p(x), _p(h_all),
                                    int(metric), ctypes.byref(gr), _p(Rz), wp, wb, _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_mlp_workspace_bytes(dims: MlpDims) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().rnn_mlp_workspace_bytes(ctypes.byref(dims), ctypes.byref(n)))
    return n.value


def mlp_params(W, b) -> MlpParams:
    """Pointer struct of the per-layer weight and bias tensors (lists, input side first)."""
    p = MlpParams()
    for l, (w, v) in enumerate(zip(W, b)):
        p.W[l], p.b[l] = _p(w), _p(v)
    return p


def rnn_mlp_train(dims, W, b, X, y, n_batches, lr, losses, workspace, stream=None, check=True):
    wp, wb = _ws(workspace)
    pr = W if isinstance(W, MlpParams) else mlp_params(W, b)
    rc = lib().rnn_mlp_train(ctypes.byref(dims), ctypes.byref(pr), _p(X), _p(y), int(n_batches), float(lr),
                             _p(losses), wp, wb, _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_check_tokens(ids, n, limit, bad_count, stream=None, check=True):
    rc = lib().rnn_check_tokens(_p(ids), int(n), int(limit), _p(bad_count), _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_measure_ceilings(scratch, stream=None) -> dict:
    """Measured device-memory, matrix-core and LDS rates of the current device (scratch: a device
    tensor of at least 128 MiB that may be overwritten)."""
    res = (ctypes.c_double * 5)()
    _check(lib().rnn_measure_ceilings(_p(scratch), scratch.numel() * scratch.element_size(), res, _stream(stream)))
    return {"hbm_copy_GBps": res[0], "mfma_f32_TFLOPs": res[1], "mfma_bf16_TFLOPs": res[2], "lds_read_GBps": res[3],
            "hbm_read_GBps": res[4]}


def rnn_profile_begin(max_launches: int = 1 << 16) -> None:
    _check(lib().rnn_profile_begin(int(max_launches)))


def rnn_profile_end() -> dict:
    """{kernel name: (launch count, total ms)} for the kernels launched since rnn_profile_begin."""
    L = lib()
    n = L.rnn_profile_kernel_count()
    counts = (ctypes.c_int64 * n)()
    ms = (ctypes.c_double * n)()
    _check(L.rnn_profile_end(n, counts, ms))
    return {L.rnn_profile_kernel_name(k).decode(): (int(counts[k]), float(ms[k]))
            for k in range(n) if counts[k] > 0}


def rnn_set_wait_limit(polls: int) -> None:
    _check(lib().rnn_set_wait_limit(int(polls)))


def rnn_workspace_init(dims, workspace, stream=None) -> None:
    wp, wb = _ws(workspace)
    _check(lib().rnn_workspace_init(ctypes.byref(dims), wp, wb, _stream(stream)))


def rnn_workspace_status(dims, workspace, stream=None) -> int:
    wp, wb = _ws(workspace)
    out = ctypes.c_int32(-1)
    _check(lib().rnn_workspace_status(ctypes.byref(dims), wp, wb, _stream(stream), ctypes.byref(out)))
    return int(out.value)


def rnn_train_stream_workspace_bytes(dims: Dims) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().rnn_train_stream_workspace_bytes(ctypes.byref(dims), ctypes.byref(out)))
    return int(out.value)


def rnn_train_stream(dims, params, ids, n_windows, lr, h0, h_last, losses, workspace, stream=None,
                     check=True):
    """params: dict of the five parameter tensors (updated in place) or a 5-pointer struct."""
    wp, wb = _ws(workspace)
    pr = params if isinstance(params, Grads) else Grads(*[_p(params[k]) for k in ("Wx", "Wh", "b", "V", "c")])
    rc = lib().rnn_train_stream(ctypes.byref(dims), ctypes.byref(pr), _p(ids), int(n_windows),
                                float(lr), _p(h0), _p(h_last), _p(losses), wp, wb, _stream(stream))
    if check:
        _check(rc)
    return rc


def rnn_train_stream_status(workspace, stream=None) -> int:
    out = ctypes.c_int32(-1)
    _check(lib().rnn_train_stream_status(_p(workspace), _stream(stream), ctypes.byref(out)))
    return int(out.value)


def rnn_window_one_launch(dims: Dims) -> bool:
    """True: rnn_window runs these sizes as one launch; False: as the launches of the three calls."""
    rc = lib().rnn_window_one_launch(ctypes.byref(dims))
    if rc < 0:
        _check(rc)
    return rc == 1


def rnn_window_workspace_bytes(dims: Dims) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().rnn_window_workspace_bytes(ctypes.byref(dims), ctypes.byref(out)))
    return int(out.value)


def rnn_window_workspace_init(dims, workspace, stream=None) -> None:
    wp, wb = _ws(workspace)
    _check(lib().rnn_window_workspace_init(ctypes.byref(dims), wp, wb, _stream(stream)))


def rnn_window(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0, workspace,
               stream=None, check=True):
    wp, wb = _ws(workspace)
    pr, gr = _params(params), _grads(grads)
    rc = lib().rnn_window(ctypes.byref(dims), ctypes.byref(pr), _p(x), _p(targets), _p(h0), _p(dh_last),
                          _p(h_all), _p(h_last), _p(loss), ctypes.byref(gr), _p(dh0), wp, wb,
                          _stream(stream))
    if check:
        _check(rc)
    return rc


WINDOW_STATIC_BYTES = 2 << 20


def rnn_window_static(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0, status=None,
                      stream=None, check=True):
    pr, gr = _params(params), _grads(grads)
    rc = lib().rnn_window_static(ctypes.byref(dims), ctypes.byref(pr), _p(x), _p(targets), _p(h0), _p(dh_last),
                                 _p(h_all), _p(h_last), _p(loss), ctypes.byref(gr), _p(dh0), _p(status),
                                 _stream(stream))
    if check:
        _check(rc)
    return rc
