"""The synthetic input generators: shapes, determinism, value ranges, bf16 rounding."""
import numpy as np
import pytest
import torch

import workloads as wl


@pytest.mark.parametrize("name", ["tiny", "electricity", "traffic"])
def test_shapes_and_determinism(name):
    w = wl.WORKLOADS[name]
    x, info = wl.make_signals(w, seed=1)
    assert x.shape == (w.B, w.N, w.L) and x.dtype == np.float32
    x2, _ = wl.make_signals(w, seed=1)
    assert np.array_equal(x, x2)
    x3, _ = wl.make_signals(w, seed=2)
    assert not np.array_equal(x, x3)
    tok = wl.make_tokens(w, x, seed=1)
    assert tok.shape == (w.B, w.N, w.d)
    Wq, Wk, Wv, Wo = wl.make_weights(w, seed=1)
    assert Wq.shape == (w.d, w.d) and abs(float(Wq.std()) - w.d ** -0.5) < 0.1 * w.d ** -0.5
    assert info["redrawn"] == 0


def test_the_five_configurations():
    got = {n: (w.B, w.N, w.L, w.k, w.ratio, w.d, w.H, w.dtype, w.eps) for n, w in wl.WORKLOADS.items()}
    assert got == {
        "tiny": (4, 32, 96, 3, (1, 4), 64, 2, "fp32", 25),
        "electricity": (32, 321, 96, 3, (1, 5), 512, 8, "bf16", 25),
        "traffic": (32, 862, 96, 3, (1, 10), 512, 8, "bf16", 25),
        "long": (16, 2048, 336, 4, (1, 10), 512, 8, "bf16", 85),
        "stress": (8, 8192, 512, 5, (1, 20), 768, 12, "bf16", 129),
    }


def test_traffic_values_lie_near_the_unit_interval():
    w = wl.WORKLOADS["traffic"]
    x, _ = wl.make_signals(w, 0)
    assert -0.2 < x.min() and x.max() < 1.2 and 0.2 < x.mean() < 0.8


def test_accept_callback_redraws_only_rejected_variates():
    w = wl.WORKLOADS["tiny"]
    x0, _ = wl.make_signals(w, 0)
    calls = []

    def accept(x):
        calls.append(x.shape[1])
        ok = np.ones(x.shape[1], dtype=bool)
        if len(calls) == 1:
            ok[[3, 7]] = False
        return ok

    x1, info = wl.make_signals(w, 0, accept=accept)
    assert calls == [w.N, 2] and info["redrawn"] == 2 and info["unresolved"] == 0
    changed = [n for n in range(w.N) if not np.array_equal(x0[:, n], x1[:, n])]
    assert changed == [3, 7]


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(10000) * 10.0 ** rng.integers(-3, 4, size=10000)).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wl.round_bf16(a), want)
