"""Pins for oracle.router_logits / router_gate (the linear router in front of
the top-k gate, Section 2.1): a scalar-loop definition, structural cases that a
transposed weight, a dropped bias or a wrong axis would break, and agreement
with the generator's own logits recipe (which is written independently)."""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth


def test_matches_scalar_loops():
    rng = np.random.default_rng(0)
    T, d, E = 7, 5, 3
    x = rng.standard_normal((T, d)).astype(np.float32)
    w = rng.standard_normal((d, E)).astype(np.float32)
    b = rng.standard_normal(E)
    lg = O.router_logits(x, w, b)
    for t in range(T):
        for e in range(E):
            s = 0.0
            for i in range(d):
                s += float(x[t, i]) * float(w[i, e])
            assert lg[t, e] == pytest.approx(s + b[e], rel=1e-14, abs=1e-14)


def test_structure():
    rng = np.random.default_rng(1)
    T, d, E = 9, 6, 4
    x = rng.standard_normal((T, d))
    b = np.array([0.5, -1.0, 2.0, 0.0])
    np.testing.assert_array_equal(O.router_logits(np.zeros((T, d)), rng.standard_normal((d, E)), b), np.tile(b, (T, 1)))
    sel = np.zeros((d, E)); sel[2, 0] = 1; sel[5, 3] = -2            # one-hot columns pick input features
    lg = O.router_logits(x, sel, None)
    np.testing.assert_array_equal(lg[:, 0], x[:, 2])
    np.testing.assert_array_equal(lg[:, 3], -2 * x[:, 5])
    assert not lg[:, 1:3].any()
    w = rng.standard_normal((d, E))
    np.testing.assert_allclose(O.router_logits(2 * x, w, None), 2 * O.router_logits(x, w, None), rtol=1e-14)
    with pytest.raises(ValueError):
        O.router_logits(x, w.T, None)
    with pytest.raises(ValueError):
        O.router_logits(x, w, np.zeros(E + 1))


def test_bf16_inputs_and_the_generators_recipe():
    cfg = synth.config("c4").with_(T=64)
    x = synth.make_x(cfg)
    w_g, bias = synth.make_router(cfg)
    lg = O.router_logits(x, w_g, bias)
    np.testing.assert_array_equal(lg.astype(np.float32), synth.make_logits(cfg, x))
    assert lg.shape == (64, 64)


def test_router_gate_is_projection_then_topk():
    cfg = synth.config("c1b")
    x = synth.make_x(cfg)
    w_g, bias = synth.make_router(cfg)
    lg, idx, w = O.router_gate(x, w_g, bias, 2)
    idx2, w2 = O.topk_gate(lg, 2)
    np.testing.assert_array_equal(idx, idx2)
    np.testing.assert_array_equal(w, w2)
    for t in range(0, cfg.T, 17):                                   # definition, token by token
        order = sorted(range(cfg.E), key=lambda e: (-lg[t, e], e))
        assert idx[t].tolist() == order[:2]
