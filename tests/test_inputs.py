"""Host-side checks of the seeded synthetic input generators (CPU only)."""
import numpy as np

import rnn_inputs as ri


def test_zipf_finite_vocab_distribution():
    cdf = ri.zipf_cdf(10000)
    p = np.diff(np.concatenate([[0.0], cdf]))
    assert abs(p[0] - 0.1514) < 1e-3 and abs(p[1] - 0.0706) < 1e-3
    assert np.searchsorted(cdf, 0.5) + 1 == 24          # 24 most frequent ids cover half the mass
    ids = ri.draw_tokens(np.random.default_rng(1), 200000, 10000, "zipf")
    assert ids.min() >= 0 and ids.max() < 10000 and ids.dtype == np.int32
    assert abs(np.mean(ids == 0) - p[0]) < 5e-3


def test_cases_are_reproducible_and_shaped():
    a, b = ri.make_config("C1"), ri.make_config("C1")
    for k in ("x", "y", "Wx", "Wh", "V"):
        assert np.array_equal(a[k], b[k])
    assert a["x"].shape == (32, 1) and a["Wx"].shape == (64, 16) and a["V"].shape == (16, 64)
    assert np.array_equal(a["x"][1:], a["y"][:-1])      # targets are the next token
    assert abs(a["Wx"].std() - 0.1) < 0.01
    c3 = ri.make_config("C3", in_dim=200, out_dim=200, hidden=20, seq_len=5)
    assert np.abs(c3["Wh"]).max() <= 0.05
    c5 = ri.make_config("C5", seq_len=6, batch=3)
    assert c5["X"].shape == (6, 3, 128) and np.array_equal(c5["Y"][1:], c5["X"][:-1])
    assert np.all(c5["Y"][0] == 0) and abs(c5["Wh"].std() - 1 / 16) < 0.01


def test_window_views():
    s = ri.make_config("C2", windows=3, in_dim=50, out_dim=50, hidden=4)
    w1 = ri.window(s, 1)
    assert w1["x"].shape == (10, 1) and np.array_equal(w1["x"], s["x"][10:20])
    assert np.array_equal(w1["y"][:-1], w1["x"][1:])
