"""Pins for the oracle's bias gradient (the chain rule behind Eq. 5 applied to z = W a + b)."""
import numpy as np

from oracle import psd_oracle as orc
from paper_1512_06216_amd import inputs


def _loss(W, b, A, y):
    Z = A @ W.T + b
    Z = Z - Z.max(axis=1, keepdims=True)
    logp = Z - np.log(np.exp(Z).sum(axis=1, keepdims=True))
    return -logp[np.arange(len(y)), y].sum()


def _delta(W, b, A, y):
    Z = A @ W.T + b
    Z = Z - Z.max(axis=1, keepdims=True)
    p = np.exp(Z)
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(len(y)), y] -= 1.0
    return p


def test_bias_gradient_is_the_finite_difference_gradient():
    rng = np.random.default_rng(0)
    K, M, N = 7, 5, 4
    A = np.maximum(rng.integers(-8, 9, size=(K, M)) / 8.0, 0.0)
    W = rng.integers(-16, 17, size=(N, M)) / 32.0
    b = rng.integers(-8, 9, size=N) / 16.0
    y = rng.integers(0, N, size=K)
    fd = np.zeros(N)
    h = 1e-6
    for n in range(N):
        bp, bm = b.copy(), b.copy()
        bp[n] += h
        bm[n] -= h
        fd[n] = (_loss(W, bp, A, y) - _loss(W, bm, A, y)) / (2 * h)
    U = _delta(W, b, A, y).astype(np.float32)
    db = orc.bias_grad(U)
    assert db.shape == (N,)
    assert np.allclose(db, fd, rtol=0, atol=2e-6)
    # the update moves the bias downhill
    b2, mom2 = orc.sync_fc_bias(U, b.astype(np.float32), np.zeros(N, np.float32), lr=1e-2, mu=0.9)
    assert _loss(W, b2.astype(np.float64), A, y) < _loss(W, b, A, y)
    assert np.allclose(mom2, np.float64(np.float32(1e-2)) * U.astype(np.float64).sum(axis=0), rtol=1e-6)


def test_bias_gradient_special_cases_and_library_sum():
    U = np.array([[1.5, -2.0, 0.25]], np.float32)
    assert orc.bias_grad(U).tolist() == [1.5, -2.0, 0.25]                  # one sample: the error itself
    d = inputs.fc_layer_integer(M=9, N=33, B=5, P=3, seed=17)
    Us, _ = orc.pack_factors(d["delta"], d["act"])
    assert np.array_equal(orc.bias_grad(Us), np.concatenate(d["delta"]).astype(np.int64).sum(axis=0))
    Ub, _ = orc.pack_factors(d["delta"], d["act"], "bf16")
    assert np.array_equal(orc.bias_grad(Ub), orc.bias_grad(Us))            # small integers survive bf16
    g = inputs.fc_config(1)
    Ug, _ = orc.pack_factors(g["delta"], g["act"])
    assert np.allclose(orc.bias_grad(Ug), Ug.astype(np.float64).sum(axis=0), rtol=1e-13, atol=1e-18)
    # linear in the stacked samples, blind to their order
    assert np.allclose(orc.bias_grad(Ug[::-1]), orc.bias_grad(Ug), rtol=1e-12, atol=1e-18)
    assert np.allclose(orc.bias_grad(Ug[:50]) + orc.bias_grad(Ug[50:]), orc.bias_grad(Ug), rtol=1e-12, atol=1e-18)
    # softmax errors sum to zero over the classes, so the bias gradient sums to zero
    s = inputs.fc_layer(M=8, N=40, B=6, P=2, seed=18, delta_kind="softmax")
    Uz, _ = orc.pack_factors(s["delta"], s["act"])
    assert abs(orc.bias_grad(Uz).sum()) < 1e-7


def test_bias_update_with_weight_decay_closed_form():
    U = np.array([[2.0, -4.0], [6.0, 8.0]], np.float32)
    b = np.array([16.0, -32.0], np.float32)
    m = np.array([4.0, 8.0], np.float32)
    b2, m2 = orc.sync_fc_bias(U, b, m, lr=0.25, mu=0.5, wd=0.5)
    want_m = 0.5 * m + 0.25 * (np.array([8.0, 4.0]) + 0.5 * b)
    assert np.array_equal(m2, want_m) and np.array_equal(b2, b - want_m)
