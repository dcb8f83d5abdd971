"""Pins for the LARC update oracle (``oracle/larc.py``): the defining property
(update size relative to the weights' norm), clipping, closed forms."""
import numpy as np

from oracle import larc as LO


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_update_size_is_a_fixed_fraction_of_the_weight_norm():
    # no decay, no momentum, clip not in effect (huge global rate): ||dw|| = trust * ||w|| whatever the gradient's scale
    for scale in (1e-6, 1.0, 1e4):
        w, g = _rand(1, 7, 3, 3, 5), _rand(2, 7, 3, 3, 5) * scale
        (w2,), _, (rate,) = LO.larc_sgd_step([w], [g], [None], lr=1e9, trust=0.02)
        assert abs(np.linalg.norm(w2 - w) / np.linalg.norm(w) - 0.02) < 1e-12
        assert abs(rate - 0.02 * np.linalg.norm(w) / np.linalg.norm(g)) < 1e-12 * rate


def test_clipping_caps_the_rate_at_the_global_one():
    w, g = _rand(3, 50), _rand(4, 50) * 1e-3            # tiny gradient: the local rate would be large
    (w2,), _, (rate,) = LO.larc_sgd_step([w], [g], [None], lr=0.1, trust=0.02, clip=True)
    assert rate == 0.1 and np.allclose(w2, w - 0.1 * g, rtol=0, atol=1e-15)
    (_,), _, (rate,) = LO.larc_sgd_step([w], [g * 1e6], [None], lr=0.1, trust=0.02, clip=True)
    assert rate < 0.1                                   # large gradient: the local rate rules
    (_,), _, (rate_s,) = LO.larc_sgd_step([w], [g], [None], lr=0.1, trust=0.02, clip=False)
    assert abs(rate_s - 0.1 * 0.02 * np.linalg.norm(w) / np.linalg.norm(g)) < 1e-12 * rate_s


def test_hand_example_with_decay_and_momentum():
    # w = (3, 4): ||w|| = 5; g = (0, 2): ||g|| = 2; wd = 0.1, trust = 0.5: local = 2.5 / (2 + 0.5) = 1
    w, g, v = np.array([3.0, 4.0]), np.array([0.0, 2.0]), np.array([1.0, -1.0])
    (w2,), (v2,), (rate,) = LO.larc_sgd_step([w], [g], [v], lr=10.0, trust=0.5, weight_decay=0.1, momentum=0.5)
    assert abs(rate - 1.0) < 1e-15
    # u = g + 0.1 w = (0.3, 2.4); v' = 0.5 v + u = (0.8, 1.9); w' = (2.2, 2.1)
    assert np.allclose(v2, [0.8, 1.9], rtol=0, atol=1e-15) and np.allclose(w2, [2.2, 2.1], rtol=0, atol=1e-15)


def test_layers_are_independent_and_degenerate_layers_fall_back():
    ws = [_rand(5, 10), _rand(6, 4, 4), np.zeros(6), _rand(7, 3)]
    gs = [_rand(8, 10), _rand(9, 4, 4) * 100, _rand(10, 6), np.zeros(3)]
    w2, _, rates = LO.larc_sgd_step(ws, gs, [None] * 4, lr=0.05, trust=0.01)
    for i in range(4):
        (wi,), _, (ri,) = LO.larc_sgd_step([ws[i]], [gs[i]], [None], lr=0.05, trust=0.01)
        assert np.array_equal(wi, w2[i]) and ri == rates[i]
    assert rates[2] == 0.05 and rates[3] == 0.05        # zero weights / zero gradient: the global rate
    assert np.array_equal(w2[3], ws[3])                 # zero gradient, no decay: nothing moves
