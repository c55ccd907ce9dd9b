"""The C-ABI library loads without a GPU, exports everything include/rnn.h declares, and
rejects bad arguments before launching anything (CPU only)."""
import ctypes
import os
import re

import pytest

import paper_1211_5590_amd as rnn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "rnn.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(rnn_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"rnn_forward", "rnn_loss", "rnn_bptt", "rnn_workspace_bytes"} <= set(names)
    L = ctypes.CDLL(rnn.lib_path())
    for n in names:
        assert hasattr(L, n), n
    assert set(rnn.exported_symbols()) == set(names)


def good_dims(**kw):
    d = dict(in_dim=64, hidden=16, out_dim=64, seq_len=32, batch=1, input_kind=0, act=0, loss_kind=0)
    d.update(kw)
    return rnn.Dims.of(d, kw.get("flags", 0))


def test_workspace_bytes_grows_with_the_problem_and_rejects_bad_dims():
    small = rnn.rnn_workspace_bytes(good_dims())
    big = rnn.rnn_workspace_bytes(good_dims(seq_len=64))
    assert 0 < small < big
    for bad in (dict(hidden=0), dict(seq_len=-1), dict(act=2), dict(loss_kind=5), dict(input_kind=3),
                dict(flags=1 << 20), dict(seq_len=1 << 20, batch=1 << 12)):
        with pytest.raises(rnn.RnnError) as e:
            rnn.rnn_workspace_bytes(good_dims(**bad))
        assert e.value.code == -1


def test_hot_calls_reject_bad_arguments_without_a_gpu():
    d = good_dims()
    fake = 0x1000  # never dereferenced: every check below fails before any launch
    P = rnn.Params(fake, fake, fake, fake, fake)
    G = rnn.Grads(fake, fake, fake, fake, fake)
    L = rnn.lib()
    need = rnn.rnn_workspace_bytes(d)
    # NULL required pointers
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(P), None, None, fake, None, fake, need, None) == -1
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(P), fake, None, None, None, fake, need, None) == -1
    assert L.rnn_loss(ctypes.byref(d), ctypes.byref(P), fake, fake, None, fake, need, None) == -1
    assert L.rnn_bptt(ctypes.byref(d), ctypes.byref(P), fake, fake, fake, None, None, None, fake, need, None) == -1
    Gbad = rnn.Grads(fake, fake, None, fake, fake)
    assert L.rnn_bptt(ctypes.byref(d), ctypes.byref(P), fake, fake, fake, None, ctypes.byref(Gbad), None, fake, need, None) == -1
    Pbad = rnn.Params(fake, None, fake, fake, fake)
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(Pbad), fake, None, fake, None, fake, need, None) == -1
    # misaligned pointer
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(P), fake + 2, None, fake, None, fake, need, None) == -1
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(P), fake, fake + 4, fake, None, fake, need, None) == -1
    # workspace missing / too small / misaligned
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(P), fake, None, fake, None, None, need, None) == -2
    assert L.rnn_forward(ctypes.byref(d), ctypes.byref(P), fake, None, fake, None, fake, need - 1, None) == -2
    assert L.rnn_loss(ctypes.byref(d), ctypes.byref(P), fake, fake, fake, fake + 8, need, None) == -2
    assert L.rnn_bptt(ctypes.byref(d), ctypes.byref(P), fake, fake, fake, None, ctypes.byref(G), None, fake, 16, None) == -2
    # bad dims in a hot call
    dbad = good_dims(hidden=-3)
    assert L.rnn_forward(ctypes.byref(dbad), ctypes.byref(P), fake, None, fake, None, fake, need, None) == -1
    assert L.rnn_check_tokens(None, 4, 10, fake, None) == -1
    assert L.rnn_check_tokens(fake, 4, 0, fake, None) == -1


def test_strerror_and_variant_names():
    assert rnn.rnn_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(rnn.rnn_strerror(code)) > 0
    assert rnn.rnn_recurrence_variant(good_dims()) in ("wg_resident", "grid_resident", "batch_mfma", "xcd_mfma", "step_mfma", "reference")
    assert rnn.rnn_recurrence_workgroups(good_dims()) >= 1
    assert rnn.rnn_recurrence_workgroups(good_dims(hidden=256, batch=128)) == 32   # 4 rows each


def test_which_sizes_the_one_window_call_runs_as_one_launch():
    lm = good_dims(seq_len=10, hidden=100, in_dim=10000, out_dim=10000)
    assert rnn.rnn_window_one_launch(lm) is True
    for wider in (dict(batch=2), dict(hidden=129), dict(seq_len=33), dict(in_dim=40000, out_dim=40000)):
        assert rnn.rnn_window_one_launch(good_dims(**wider)) is False, wider
    with pytest.raises(rnn.RnnError) as e:
        rnn.rnn_window_one_launch(good_dims(loss_kind=1))
    assert e.value.code == -3


def test_train_stream_rejects_what_it_cannot_run_without_a_gpu():
    ok = good_dims(seq_len=10, hidden=100, in_dim=10000, out_dim=10000)
    need_of_ok = rnn.rnn_train_stream_workspace_bytes(ok)
    assert need_of_ok > 0
    # shapes beyond the one-launch kernel are served by the launches of the three calls
    for wider in (dict(batch=2), dict(hidden=129), dict(seq_len=33), dict(in_dim=40000, out_dim=40000)):
        assert rnn.rnn_train_stream_workspace_bytes(good_dims(**wider)) > 0, wider
    for bad, code in ((dict(out_dim=128), -3), (dict(input_kind=1), -3), (dict(loss_kind=1), -3),
                      (dict(hidden=0), -1), (dict(act=7), -1), (dict(flags=1), -1)):
        with pytest.raises(rnn.RnnError) as e:
            rnn.rnn_train_stream_workspace_bytes(good_dims(**bad))
        assert e.value.code == code, bad
    L = rnn.lib()
    fake = 0x1000
    P = rnn.Grads(fake, fake, fake, fake, fake)
    need = rnn.rnn_train_stream_workspace_bytes(ok)
    call = lambda params, ids, n, ws, nbytes: L.rnn_train_stream(
        ctypes.byref(ok), ctypes.byref(params) if params else None, ids, n, 0.1, None, None, None, ws, nbytes, None)
    assert call(None, fake, 1, fake, need) == -1
    assert call(rnn.Grads(fake, None, fake, fake, fake), fake, 1, fake, need) == -1
    assert call(P, None, 1, fake, need) == -1
    assert call(P, fake + 2, 1, fake, need) == -1
    assert call(P, fake, -1, fake, need) == -1
    assert call(P, fake, 1, None, need) == -2
    assert call(P, fake, 1, fake, need - 1) == -2
    assert call(P, fake, 0, fake, need) == 0          # nothing to do: nothing is launched


def test_gauss_newton_rejects_bad_arguments_without_a_gpu():
    d = good_dims()
    fake = 0x1000  # never dereferenced: every check below fails before any launch
    P = rnn.Params(fake, fake, fake, fake, fake)
    G = rnn.Grads(fake, fake, fake, fake, fake)
    L = rnn.lib()
    need = rnn.rnn_gauss_newton_workspace_bytes(d)
    assert need > rnn.rnn_workspace_bytes(d)

    def call(dims=d, params=P, gamma=P, x=fake, h_all=fake, metric=0, out=G, Rz=None, ws=fake, nbytes=need):
        return L.rnn_gauss_newton_vec(ctypes.byref(dims), ctypes.byref(params), ctypes.byref(gamma), x, h_all,
                                      metric, ctypes.byref(out), Rz, ws, nbytes, None)
    assert call(x=None) == -1
    assert call(h_all=None) == -1
    assert call(gamma=rnn.Params(fake, fake, None, fake, fake)) == -1
    assert call(out=rnn.Grads(fake, fake, fake, None, fake)) == -1
    assert call(metric=2) == -1
    assert call(Rz=fake + 4) == -1
    assert call(dims=good_dims(flags=rnn.FLAG_BPTT_RECOMPUTE)) == -1
    assert call(dims=good_dims(hidden=0)) == -1
    assert call(ws=None) == -2
    assert call(nbytes=rnn.rnn_workspace_bytes(d)) == -2
    with pytest.raises(rnn.RnnError):
        rnn.rnn_gauss_newton_workspace_bytes(good_dims(act=7))


def test_mlp_rejects_bad_arguments_without_a_gpu():
    d = rnn.MlpDims(784, 500, 1, 10, 60, 1, 0)
    need = rnn.rnn_mlp_workspace_bytes(d)
    assert need > 0
    fake = 0x1000
    L = rnn.lib()
    P = rnn.MlpParams()
    for l in range(2):
        P.W[l], P.b[l] = fake, fake

    def call(dims=d, params=P, X=fake, y=fake, n=1, ws=fake, nbytes=need):
        return L.rnn_mlp_train(ctypes.byref(dims), ctypes.byref(params), X, y, n, 0.1, None, ws, nbytes, None)
    assert call(X=None) == -1
    assert call(y=None) == -1
    assert call(n=-1) == -1
    assert call(X=fake + 4) == -1
    missing = rnn.MlpParams()
    missing.W[0], missing.b[0] = fake, fake
    assert call(params=missing) == -1
    assert call(dims=rnn.MlpDims(784, 0, 1, 10, 60, 1, 0)) == -1      # hidden layers need a width
    assert call(dims=rnn.MlpDims(784, 500, 16, 10, 60, 1, 0)) == -1    # too many layers
    assert call(dims=rnn.MlpDims(784, 500, 1, 10, 60, 1, 1)) == -1     # flag the call does not take
    assert call(dims=rnn.MlpDims(784, 500, 1, 10, 2000, 1, 0)) == -3   # batch beyond what the kernels serve
    assert call(ws=None) == -2
    assert call(nbytes=need - 1) == -2


def test_split_product_flag_is_taken_only_where_it_applies():
    d = good_dims(flags=rnn.FLAG_BF16X3_OUTPUT)
    assert rnn.rnn_workspace_bytes(d) > rnn.rnn_workspace_bytes(good_dims())   # room for the bf16 operands
    fake = 0x1000
    P = rnn.Params(fake, fake, fake, fake, fake)
    G = rnn.Grads(fake, fake, fake, fake, fake)
    L = rnn.lib()
    n = ctypes.c_size_t(0)
    # the one-launch kernels do not take the flag; the Gauss-Newton product does (and asks for more room)
    assert L.rnn_window_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == -1
    assert L.rnn_train_stream_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == -1
    assert rnn.rnn_gauss_newton_workspace_bytes(d) > rnn.rnn_gauss_newton_workspace_bytes(good_dims())


def test_measure_ceilings_rejects_bad_arguments_without_a_gpu():
    L = rnn.lib()
    res = (ctypes.c_double * 5)()
    fake = 0x100000
    assert L.rnn_measure_ceilings(None, 1 << 30, res, None) == -1
    assert L.rnn_measure_ceilings(fake, 1 << 30, None, None) == -1
    assert L.rnn_measure_ceilings(fake, (128 << 20) - 1, res, None) == -1     # scratch too short
    assert L.rnn_measure_ceilings(fake + 8, 1 << 30, res, None) == -1       # misaligned
