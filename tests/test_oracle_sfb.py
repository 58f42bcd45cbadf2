"""Pins for the oracle's reconstruction (Eq. 5, SFB step 3) and momentum-SGD update.

Expected values come from mathematics the paper fixes (the reconstructed matrix IS the
gradient of the loss w.r.t. W), from numpy's own matmul / SVD, or from closed forms
worked out by hand; never from the oracle.
"""
import numpy as np
import pytest

from oracle import psd_oracle as orc
from paper_1512_06216_amd import inputs


# ---------------------------------------------------------------------------------------
# Eq. 5: sum_i delta_i a_i^T equals dLoss/dW of the layer z = W a, summed over all samples
# ---------------------------------------------------------------------------------------
def _softmax_ce_loss(W, A, y):
    Z = A @ W.T                      # K x N, row k = W a_k
    Z = Z - Z.max(axis=1, keepdims=True)
    logp = Z - np.log(np.exp(Z).sum(axis=1, keepdims=True))
    return -logp[np.arange(len(y)), y].sum()


def _softmax_ce_delta(W, A, y):
    Z = A @ W.T
    Z = Z - Z.max(axis=1, keepdims=True)
    p = np.exp(Z)
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(len(y)), y] -= 1.0
    return p                          # dLoss/dz per sample


def _tiny_problem(seed=0, P=3, B=2, M=5, N=4):
    rng = np.random.default_rng(seed)
    K = P * B
    # values exactly representable in fp32 so oracle inputs == float64 inputs of the check
    A = np.maximum(rng.integers(-8, 9, size=(K, M)) / 8.0, 0.0)
    W = rng.integers(-16, 17, size=(N, M)) / 32.0
    y = rng.integers(0, N, size=K)
    return P, B, M, N, A, W, y


def test_reconstruction_is_the_finite_difference_gradient():
    P, B, M, N, A, W, y = _tiny_problem()
    delta = _softmax_ce_delta(W, A, y).astype(np.float32)   # fp32 factors, as transmitted
    # finite differences of the loss whose per-sample dLoss/dz is exactly `delta` in fp64
    d64 = _softmax_ce_delta(W, A, y)
    fd = np.zeros_like(W)
    h = 1e-6
    for n in range(N):
        for m in range(M):
            Wp, Wm = W.copy(), W.copy()
            Wp[n, m] += h
            Wm[n, m] -= h
            fd[n, m] = (_softmax_ce_loss(Wp, A, y) - _softmax_ce_loss(Wm, A, y)) / (2 * h)
    deltas = [delta[p * B:(p + 1) * B] for p in range(P)]
    acts = [A[p * B:(p + 1) * B].astype(np.float32) for p in range(P)]
    U, V = orc.pack_factors(deltas, acts)
    dW = orc.rebuild(U, V)
    assert dW.shape == (N, M)
    assert np.allclose(dW, fd, rtol=0, atol=2e-6)          # fp32 delta rounding + FD error
    # a transposed / swapped reconstruction would have the wrong shape or values:
    assert not np.allclose(dW, (A.T @ d64).T[::-1], atol=1e-3)


def test_quadratic_loss_gradient_and_sum_not_mean():
    # loss = 1/2 sum_k ||W a_k - t_k||^2  ->  delta_k = W a_k - t_k,  dL/dW = sum_k delta_k a_k^T
    rng = np.random.default_rng(1)
    K, M, N = 6, 4, 3
    A = rng.integers(0, 5, size=(K, M)).astype(np.float64)
    W = rng.integers(-3, 4, size=(N, M)).astype(np.float64)
    T = rng.integers(-3, 4, size=(K, N)).astype(np.float64)
    D = A @ W.T - T
    loss = lambda Wx: 0.5 * ((A @ Wx.T - T) ** 2).sum()
    fd = np.zeros_like(W)
    for n in range(N):
        for m in range(M):
            Wp, Wm = W.copy(), W.copy()
            Wp[n, m] += 0.5
            Wm[n, m] -= 0.5
            fd[n, m] = loss(Wp) - loss(Wm)                 # exact for a quadratic
    dW = orc.rebuild(D.astype(np.float32), A.astype(np.float32))
    assert np.array_equal(dW, fd)                          # integers: exact, and no 1/K


def test_update_decreases_the_loss():
    # sign of the step: with momentum zero and a small rate the loss must go down
    P, B, M, N, A, W, y = _tiny_problem(seed=5)
    delta = _softmax_ce_delta(W, A, y).astype(np.float32)
    W2, Mom2 = orc.sync_fc_sfb(delta, A.astype(np.float32), W.astype(np.float32),
                               np.zeros_like(W, dtype=np.float32), lr=1e-2, mu=0.9)
    assert _softmax_ce_loss(W2.astype(np.float64), A, y) < _softmax_ce_loss(W, A, y)
    # and Mom' = lr * gradient when the buffer starts at zero
    g = _softmax_ce_delta(W, A, y).astype(np.float32).astype(np.float64).T @ A
    assert np.allclose(Mom2, np.float64(np.float32(1e-2)) * g, rtol=1e-6, atol=1e-12)


def test_single_sample_is_one_outer_product():
    u = np.array([[1.5, -2.0, 0.25]], np.float32)
    v = np.array([[2.0, 0.0, -4.0, 8.0]], np.float32)
    dW = orc.rebuild(u, v)
    want = [[3.0, 0.0, -6.0, 12.0], [-4.0, 0.0, 8.0, -16.0], [0.5, 0.0, -1.0, 2.0]]
    assert dW.tolist() == want


def test_rank_is_bounded_by_number_of_samples():
    rng = np.random.default_rng(2)
    for K in (1, 2, 5):
        U = rng.standard_normal((K, 12), dtype=np.float32)
        V = rng.standard_normal((K, 17), dtype=np.float32)
        s = np.linalg.svd(orc.rebuild(U, V), compute_uv=False)
        assert (s > 1e-10 * s[0]).sum() == K


def test_linearity_and_worker_order():
    rng = np.random.default_rng(3)
    U1, V1 = rng.standard_normal((4, 6), dtype=np.float32), rng.standard_normal((4, 9), dtype=np.float32)
    U2, V2 = rng.standard_normal((3, 6), dtype=np.float32), rng.standard_normal((3, 9), dtype=np.float32)
    both = orc.rebuild(np.vstack([U1, U2]), np.vstack([V1, V2]))
    assert np.allclose(both, orc.rebuild(U1, V1) + orc.rebuild(U2, V2), rtol=1e-14, atol=1e-15)
    assert np.array_equal(orc.rebuild(4 * U1, V1), 4 * orc.rebuild(U1, V1))   # power of 2: exact
    perm = rng.permutation(7)
    Us, Vs = np.vstack([U1, U2]), np.vstack([V1, V2])
    assert np.allclose(orc.rebuild(Us[perm], Vs[perm]), both, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("cfg", [1, 2])
def test_matches_numpy_float64_matmul(cfg):
    d = inputs.fc_config(cfg)
    U, V = orc.pack_factors(d["delta"], d["act"])
    dW = orc.rebuild(U, V)
    want = np.concatenate(d["delta"]).astype(np.float64).T @ np.concatenate(d["act"]).astype(np.float64)
    assert orc.rel_frob(dW, want) < 1e-14
    rng = np.random.default_rng(0)
    idx_n = rng.integers(0, d["N"], 200)
    idx_m = rng.integers(0, d["M"], 200)
    s = orc.rebuild_samples(U, V, idx_n, idx_m)
    assert np.allclose(s, want[idx_n, idx_m], rtol=1e-12, atol=1e-18)


def test_integer_factors_are_exact():
    d = inputs.fc_layer_integer(M=37, N=29, B=8, P=3, seed=11)
    U, V = orc.pack_factors(d["delta"], d["act"])
    dW = orc.rebuild(U, V)
    want = np.concatenate(d["delta"]).astype(np.int64).T @ np.concatenate(d["act"]).astype(np.int64)
    assert np.array_equal(dW, want.astype(np.float64))
    # bf16 factors hold small integers exactly, so the bf16 route gives the same matrix
    Ub, Vb = orc.pack_factors(d["delta"], d["act"], "bf16")
    assert np.array_equal(orc.rebuild(Ub, Vb), dW)


def test_softmax_errors_give_zero_column_sums():
    # rows of (softmax - onehot) sum to zero, hence sum_n dW[n][m] = 0 for every m
    d = inputs.fc_layer(M=16, N=50, B=4, P=2, seed=9, delta_kind="softmax")
    U, V = orc.pack_factors(d["delta"], d["act"])
    dW = orc.rebuild(U, V)
    assert np.abs(dW.sum(axis=0)).max() < 1e-7 * np.abs(dW).sum(axis=0).max()


# ---------------------------------------------------------------------------------------
# update (Eq. 3-4, Alg. 3 update line; momentum reading)
# ---------------------------------------------------------------------------------------
def test_update_special_cases():
    rng = np.random.default_rng(4)
    W = rng.integers(-50, 50, (5, 7)).astype(np.float32)
    Mom = rng.integers(-50, 50, (5, 7)).astype(np.float32)
    dW = rng.integers(-50, 50, (5, 7)).astype(np.float64)
    # mu = 0: plain SGD
    W2, Mom2 = orc.momentum_update(dW, W, Mom, lr=0.25, mu=0.0)
    assert np.array_equal(W2, W - 0.25 * dW) and np.array_equal(Mom2, 0.25 * dW)
    # dW = 0: pure momentum coast
    W2, Mom2 = orc.momentum_update(np.zeros_like(dW), W, Mom, lr=0.25, mu=0.5)
    assert np.array_equal(Mom2, 0.5 * Mom) and np.array_equal(W2, W - 0.5 * Mom)
    # inputs are not modified
    W0, M0 = W.copy(), Mom.copy()
    orc.momentum_update(dW, W, Mom, 0.5, 0.5)
    assert np.array_equal(W, W0) and np.array_equal(Mom, M0)


def test_two_steps_closed_form():
    # Mom0 = 0, same dW twice: Mom2 = (1+mu) lr dW, W2 = W0 - (2+mu) lr dW
    rng = np.random.default_rng(6)
    W0 = rng.integers(-50, 50, (3, 4)).astype(np.float32)
    dW = rng.integers(-50, 50, (3, 4)).astype(np.float64)
    lr, mu = 0.125, 0.5
    W1, M1 = orc.momentum_update(dW, W0, np.zeros_like(W0), lr, mu)
    W2, M2 = orc.momentum_update(dW, W1, M1, lr, mu)
    assert np.array_equal(M2, (1 + mu) * lr * dW)
    assert np.array_equal(W2, W0 - (2 + mu) * lr * dW)


def test_update_uses_fp32_rate_values_and_rounds_once():
    # lr = 0.01f is not 0.01; the oracle must use the fp32 value the GPU receives
    W = np.array([1.0], np.float32)
    Mom = np.array([0.5], np.float32)
    dW = np.array([3.0])
    lr32, mu32 = np.float32(0.01), np.float32(0.9)
    W2, Mom2 = orc.momentum_update(dW, W, Mom, 0.01, 0.9)
    mom = float(mu32) * 0.5 + float(lr32) * 3.0
    assert Mom2[0] == np.float32(mom) and W2[0] == np.float32(1.0 - mom)


# ---------------------------------------------------------------------------------------
# weight decay: the "regularisation" half of Lambda (Section 3.3)
# ---------------------------------------------------------------------------------------
def test_weight_decay_alone_shrinks_the_weights():
    W = np.array([[8.0, -4.0], [2.0, 64.0]], np.float32)
    Z = np.zeros((2, 2))
    W2, Mom2 = orc.momentum_update(Z, W, np.zeros_like(W), lr=0.25, mu=0.0, wd=0.5)
    assert np.array_equal(Mom2, 0.125 * W) and np.array_equal(W2, 0.875 * W)      # (1 - lr*wd) W
    # wd = 0 is the plain update
    a = orc.momentum_update(Z + 3, W, W, 0.25, 0.5)
    b = orc.momentum_update(Z + 3, W, W, 0.25, 0.5, 0.0)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_weight_decay_is_the_gradient_of_the_l2_penalty():
    # loss + wd/2 ||W||^2 has gradient dW + wd W: check against central differences
    P, B, M, N, A, W, y = _tiny_problem(seed=8)
    wd = 0.25
    total = lambda Wx: _softmax_ce_loss(Wx, A, y) + 0.5 * wd * (Wx ** 2).sum()
    fd = np.zeros_like(W)
    h = 1e-6
    for n in range(N):
        for m in range(M):
            Wp, Wm = W.copy(), W.copy()
            Wp[n, m] += h
            Wm[n, m] -= h
            fd[n, m] = (total(Wp) - total(Wm)) / (2 * h)
    delta = _softmax_ce_delta(W, A, y).astype(np.float32)
    W2, Mom2 = orc.sync_fc_sfb(delta, A.astype(np.float32), W.astype(np.float32),
                               np.zeros_like(W, dtype=np.float32), lr=1.0, mu=0.0, wd=wd)
    assert np.allclose(Mom2, fd, rtol=0, atol=5e-6)        # Mom' = lr * (dW + wd W) with lr = 1
    assert total(W2.astype(np.float64) + 0.99 * fd) < total(W)   # W2 = W - fd; a 1 % step along it lowers the penalised loss


def test_dense_route_applies_the_same_weight_decay():
    d = inputs.dense_layer_integer(n=257, P=3, seed=14)
    g = np.sum(np.stack(d["G"]).astype(np.int64), axis=0)
    W2, Mom2 = orc.sync_dense_ps(d["G"], d["W"], d["Mom"], lr=0.25, mu=0.5, S=4, wd=0.5)
    want_m = 0.5 * d["Mom"] + 0.25 * (g + 0.5 * d["W"])
    assert np.array_equal(Mom2, want_m) and np.array_equal(W2, d["W"] - want_m)


def test_rel_frob_against_hand_values():
    # |x - ref|_F / |ref|_F written out: 3-4-5 triangle, a constant matrix, and the zero reference
    assert orc.rel_frob(np.array([3.3, 4.4]), np.array([3.0, 4.0])) == pytest.approx(0.1, rel=1e-12)
    assert orc.rel_frob(np.full((2, 2), 2.0), np.ones((2, 2))) == pytest.approx(1.0, rel=1e-12)
    assert orc.rel_frob(np.array([[1.0, 2.0], [3.0, 4.0]]), np.array([[1.0, 2.0], [3.0, 4.0]])) == 0.0
    assert orc.rel_frob(np.array([0.0, 2.0]), np.zeros(2)) == pytest.approx(2.0)     # zero reference: absolute norm
    # float32 inputs are widened before the subtraction (no fp32 cancellation error)
    a = np.array([1.0 + 2.0 ** -23], dtype=np.float32)
    assert orc.rel_frob(a, np.array([1.0])) == pytest.approx(2.0 ** -23, rel=1e-12)
