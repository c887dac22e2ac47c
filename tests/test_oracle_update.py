"""Pins of the oracle's model update (Sec. 2, "Distributed Training": mini-batch SGD) and of
the chain decode -> update against what the mathematics fixes."""
import numpy as np

from oracle import draco_oracle as o


def test_step_on_a_quadratic_lands_on_the_minimiser():
    """loss_i(w) = |w - c_i|^2 / 2 has gradient w - c_i; with learning rate 1 the mini-batch
    step from ANY w lands exactly on the mean of the c_i, the minimiser of the batch loss."""
    rng = np.random.default_rng(0)
    B, d = 12, 7
    c = rng.standard_normal((B, d))
    w = rng.standard_normal(d) * 10
    grads = w[None, :] - c
    got = o.sgd_update(w, grads.sum(0), gamma=1.0, batch=B)
    assert np.allclose(got, c.mean(0), rtol=0, atol=1e-13)
    # half the learning rate goes half the way
    half = o.sgd_update(w, grads.sum(0), gamma=0.5, batch=B)
    assert np.allclose(half, 0.5 * (w + c.mean(0)), rtol=0, atol=1e-13)


def test_invariants_of_the_step():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(9)
    u = rng.standard_normal(9)
    assert np.array_equal(o.sgd_update(w, np.zeros(9), 0.3, 4), w)            # no gradient, no move
    assert np.array_equal(o.sgd_update(w, u, 0.0, 4), w)                      # no learning rate, no move
    two = o.sgd_update(o.sgd_update(w, u, 0.1, 5), u, 0.1, 5)
    assert np.allclose(two, o.sgd_update(w, u, 0.2, 5), rtol=0, atol=1e-15)   # steps with one gradient add up
    assert np.allclose(o.sgd_update(w, 3 * u, 0.1, 3), o.sgd_update(w, u, 0.1, 1), rtol=0, atol=1e-15)
    # the sign: a positive gradient coordinate lowers the parameter
    assert o.sgd_update(np.zeros(1), np.ones(1), 1.0, 1)[0] == -1.0
    assert o.sgd_update(np.float32([1.5]), np.float32([0.25]), 2, 4).dtype == np.float64


def test_decode_then_update_equals_the_step_on_the_clean_gradients():
    """Definition 2 chained with the update: with s adversaries the model after the step is
    the one plain mini-batch SGD would reach on the honest gradients."""
    rng = np.random.default_rng(2)
    P, s, d = 9, 1, 20
    G = rng.standard_normal((P, d))
    w = rng.standard_normal(d)
    Z = o.encode_repetition(G, s).astype(np.float32)
    Z[4] = -100.0 * Z[4]
    u, mask, st = o.decode_repetition(Z, s)
    assert st == o.OK and list(np.flatnonzero(mask)) == [4]
    want = w - 0.05 / P * G.sum(0)
    assert np.allclose(o.sgd_update(w, u, 0.05, P), want, rtol=0, atol=1e-6)
